"""Seeded synthetic inputs: KV tensors, block tables, chunk draws, workloads.

This module serves both the CPU oracle's tests and the HIP path's tests and
bench.  It holds none of the method's arithmetic: values are drawn, shaped and
handed over as bf16 bit patterns (uint16) or int32 tables.

The paper's own workload is RAG over real text with a real model (Sec. 3.2,
"Early promise"); the path built here is data independent, so standard-normal
bf16 tensors with a model's KV shape stand in for real KV caches.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    # Philox is counter based: (seed, stream) is the key, the draw index the counter.
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def normal_bf16(seed: int, shape, stream: int = 0) -> np.ndarray:
    """N(0,1) drawn in fp32 and narrowed to bf16 by torch's CPU cast; returned
    as uint16 bit patterns."""
    x = _rng(seed, stream).standard_normal(size=shape, dtype=np.float32)
    b = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy()
    return np.ascontiguousarray(b).view(np.uint16)


def disjoint_block_tables(seed: int, num_blocks: int, lengths, stream: int = 1):
    """Block tables sampled without replacement from one pool, so that no two
    tables (and no two entries) share a physical block."""
    total = int(sum(lengths))
    if total > num_blocks:
        raise ValueError("tables need %d blocks, pool has %d" % (total, num_blocks))
    perm = _rng(seed, stream).permutation(num_blocks)[:total].astype(np.int32)
    out, pos = [], 0
    for n in lengths:
        out.append(np.ascontiguousarray(perm[pos:pos + n]))
        pos += n
    return out


def permutation(seed: int, n: int, stream: int = 2) -> np.ndarray:
    return _rng(seed, stream).permutation(n).astype(np.int32)


def zipf_distinct_draws(seed: int, n_requests: int, k: int, pool: int,
                        alpha: float = 1.0, stream: int = 3) -> np.ndarray:
    """Per request k distinct chunk ids.  Popularity rank r (1-based) has
    probability proportional to r^-alpha; ranks are drawn by inverse CDF and
    redrawn until the k of a request differ; a seeded permutation maps rank to
    chunk id so that popularity is unrelated to address."""
    g = _rng(seed, stream)
    w = 1.0 / np.arange(1, pool + 1, dtype=np.float64) ** alpha
    cdf = np.cumsum(w / w.sum())
    rank_to_chunk = g.permutation(pool)
    out = np.empty((n_requests, k), dtype=np.int32)
    for r in range(n_requests):
        chosen: list[int] = []
        while len(chosen) < k:
            rank = int(np.searchsorted(cdf, g.random(), side="left"))
            rank = min(rank, pool - 1)
            if rank not in chosen:
                chosen.append(rank)
        out[r] = rank_to_chunk[chosen]
    return out


@dataclass(frozen=True)
class KVShape:
    L: int
    H: int
    D: int
    bs: int

    @property
    def paged_bytes_per_token(self) -> int:      # B_p
        return self.L * 2 * self.H * self.D * 2

    @property
    def int8_bytes_per_token(self) -> int:       # B_q
        return self.L * 2 * self.H * (self.D + 4)

    @property
    def int4_bytes_per_token(self) -> int:
        return self.L * 2 * self.H * (self.D // 2 + self.D // 32 * 4)

    def stored_bytes_per_token(self, fmt_name: str) -> int:
        return {"raw": self.paged_bytes_per_token, "int8": self.int8_bytes_per_token,
                "fp8": self.int8_bytes_per_token, "int4": self.int4_bytes_per_token}[fmt_name]


@dataclass(frozen=True)
class Workload:
    """One of the five workloads.  Token counts are per chunk; offsets are the
    RoPE position deltas used when the chunks are composed."""
    name: str
    seed: int
    shape: KVShape
    rope_base: float
    chunk_tokens: tuple
    offsets: tuple
    note: str = ""
    extra: dict = field(default_factory=dict)


TOY = KVShape(L=2, H=4, D=64, bs=16)
LLAMA8B = KVShape(L=32, H=8, D=128, bs=16)
LLAMA70B = KVShape(L=80, H=8, D=128, bs=16)

WORKLOADS = {
    "toy": Workload("toy", 1001, TOY, 10000.0, (256, 256), (0, 256),
                    "2 chunks of 256 tokens, int8 and raw, 128-block pool"),
    "8b_store_reload": Workload("8b_store_reload", 1002, LLAMA8B, 500000.0, (4096,), (0,),
                                "4096 tokens stored to int8, reloaded at offset 0"),
    "rag_compose": Workload("rag_compose", 1003, LLAMA8B, 500000.0, (512,) * 8,
                            tuple(512 * j for j in range(8)),
                            "8 chunks of 512 tokens placed in a seeded order"),
    "70b_long": Workload("70b_long", 1004, LLAMA70B, 500000.0, (8192,) * 4,
                         (0, 8192, 16384, 24576),
                         "32768 tokens stored once, composed back as 4 slices"),
    "batched_reuse": Workload("batched_reuse", 1005, LLAMA8B, 500000.0, (1024,) * 4,
                              (0, 1024, 2048, 3072),
                              "pool of 256 chunks, 64 requests x 4 Zipf(1.0) draws",
                              {"pool": 256, "requests": 64, "alpha": 1.0}),
}
