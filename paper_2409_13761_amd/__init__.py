"""KDN KV-cache movement (store / load / compose) for AMD MI355X.

`kdn` is the binding of the C-ABI library; `synth` makes seeded synthetic inputs;
`build` compiles the HIP sources.  Nothing here computes on the CPU.
"""
__all__ = ["kdn", "synth", "build"]
