#!/usr/bin/env python3
"""Throughput of the KDN hot path on one MI355X.

One step carries one 4096-token context of Llama-3-8B-shaped KV (32 layers, 8 KV
heads, head_dim 128, bf16, paged in blocks of 16 tokens) through the whole path:
  store    paged KV -> stored int8 chunk              (kdn_store_chunk)
  load     stored chunk -> a fresh block table        (kdn_load_chunk, no shift)
  compose  the chunk as 8 slices of 512 tokens, in a seeded order, each shifted by
           its cumulative RoPE offset, into another fresh table   (kdn_compose)
Inputs are resident in HBM before the timed region.  Four disjoint buffer sets are
cycled, and a step reads chunks that were stored two or three steps earlier, so that
the 256 MB last-level cache cannot serve a repeat or a just-written chunk.

Prints ONE JSON line: tokens/s over the whole step, the roofline of the dominant
kernel (the place kernel behind load and compose) from HIP-event timings, and the
CPU oracle's throughput on the host cores as a reported baseline.
"""
import argparse
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published peak

# HBM bytes per k_place launch of this workload from the FETCH_SIZE / WRITE_SIZE counter runs
# summarised under profiles/, valid only for the kernel source they were taken with.
COUNTER_TRAFFIC = {"source_sha256_16": "787f6808c77731d9", "k_place_bytes_per_launch": 815509774}


def counter_traffic():
    import hashlib
    src = os.path.join(ROOT, "paper_2409_13761_amd", "csrc", "kdn.hip")
    sha = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
    return COUNTER_TRAFFIC["k_place_bytes_per_launch"] if sha == COUNTER_TRAFFIC["source_sha256_16"] else None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=8)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, a dispatch of known size for "
                         "scaling hardware byte counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; the path shards without any exchange "
              "(by KV head, layer or request), so --gpus N > 1 is not measured", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2409_13761_amd import kdn, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        return 3
    kdn.lib()                                   # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    sh = synth.LLAMA8B
    T, n_slices = 4096, 8
    base = synth.WORKLOADS["rag_compose"].rope_base
    seed = synth.WORKLOADS["rag_compose"].seed
    blocks = T // sh.bs
    n_sets = 4
    nb = n_sets * 3 * blocks
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    shape = (sh.L, nb, sh.bs, sh.H, sh.D)
    k = torch.empty(shape, device=dev, dtype=torch.bfloat16)
    v = torch.empty(shape, device=dev, dtype=torch.bfloat16)
    for t in (k, v):                            # N(0,1) in slabs, to bound the fp32 temporary
        for l in range(sh.L):
            t[l].copy_(torch.randn(shape[1:], generator=g, device=dev, dtype=torch.float32))
    cache = kdn.PagedCache(k, v)
    tables = synth.disjoint_block_tables(seed, nb, [blocks] * (3 * n_sets))
    order = synth.permutation(seed, n_slices)
    offsets = [int(j * (T // n_slices)) for j in range(n_slices)]   # j-th placed slice moves by 512*j
    sets = []
    for s in range(n_sets):
        src, dst_a, dst_b = (torch.from_numpy(tables[3 * s + i]).to(dev) for i in range(3))
        chunk = kdn.alloc_chunk(cache, T, kdn.FMT_INT8_ROWSCALE)
        slices = [chunk.slice(int(i) * (T // n_slices), T // n_slices) for i in order]
        sets.append((src, dst_a, dst_b, chunk, slices))
    kdn.kdn_rope_prepare(base, sh.D, offsets)

    names = ("store", "load", "compose")
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in names] for _ in range(args.steps)]

    def step(i, events=None):
        # The chunk a step loads or composes was stored two or three steps earlier, with
        # gigabytes of traffic in between, so it comes from HBM, not from the cache.
        src, dst_a, dst_b, chunk, _ = sets[i % n_sets]
        load_chunk = sets[(i + 2) % n_sets][3]
        compose_slices = sets[(i + 1) % n_sets][4]
        if events:
            events[0][0].record()
        kdn.kdn_store_chunk(cache, src, 0, T, chunk)
        if events:
            events[0][1].record()
            events[1][0].record()
        kdn.kdn_load_chunk(load_chunk, cache, dst_a, 0)
        if events:
            events[1][1].record()
            events[2][0].record()
        kdn.kdn_compose(compose_slices, offsets, cache, dst_b, base)
        if events:
            events[2][1].record()

    for s in range(n_sets):                     # every chunk exists before any is read
        kdn.kdn_store_chunk(cache, sets[s][0], 0, T, sets[s][3])
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, ev[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    if args.calibration_copy:
        a = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                              # 1 GiB read, 1 GiB written
        torch.cuda.synchronize()
        del a, b

    ms = {n: float(np.mean([ev[i][j][0].elapsed_time(ev[i][j][1]) for i in range(args.steps)]))
          for j, n in enumerate(names)}
    bytes_call = T * (sh.paged_bytes_per_token + sh.int8_bytes_per_token)    # B_p + B_q per token
    place_ms = 0.5 * (ms["load"] + ms["compose"])
    achieved = bytes_call / (place_ms * 1e-3) / 1e9
    tokens_per_s = T * args.steps / wall

    out = {
        "metric": "KV tokens composed/sec (store+load+RoPE shift) and achieved HBM GB/s",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 KV, int8 codes + fp32 scales stored, fp32 arithmetic",
        "data": "synthetic N(0,1) bf16 KV, seeded; random disjoint block tables",
        "config": {
            "workload": "Llama-3-8B-shaped KV (L32 H8 D128 bs16): per step store 4096 tokens to int8, "
                        "load them at offset 0, compose them as 8x512-token slices in seeded order with "
                        "RoPE offsets 0..3584 (base %g); %d buffer sets cycled" % (base, n_sets),
            "tokens_per_step": T,
            "algorithmic_bytes_per_call": bytes_call,
            "calls_per_step": 3,
        },
        "breakdown": {n: {"ms": ms[n], "GBps": bytes_call / (ms[n] * 1e-3) / 1e9,
                          "frac_of_peak": bytes_call / (ms[n] * 1e-3) / 1e9 / HBM_PEAK_GBPS}
                      for n in names},
        "roofline": {
            "bound": "hbm",
            "kernel": "k_place (load and compose launches)",
            "achieved": achieved,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": counter_traffic(),
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cache, sets[0], order, offsets, base, T, n_slices, args.cpu_steps)
    print(json.dumps(out))
    return 0


def cpu_baseline(cache, buf_set, order, offsets, base, T, n_slices, steps):
    """The oracle as it stands, on the host cores: the same step (store, load, compose
    of one 4096-token context, all layers), layers split over threads."""
    import numpy as np
    import torch
    from oracle import kdn_oracle as O

    L, nb, bs, H, D = cache.shape
    src, _, _, _, _ = buf_set
    blocks = T // bs
    # host copy of the source blocks only; destination blocks start as zeros
    hk = np.zeros((L, 3 * blocks, bs, H, D), dtype=np.uint16)
    hv = np.zeros_like(hk)
    hk[:, :blocks] = cache.k[:, src.long()].view(torch.int16).cpu().numpy().view(np.uint16)
    hv[:, :blocks] = cache.v[:, src.long()].view(torch.int16).cpu().numpy().view(np.uint16)
    host = O.PagedCache(hk, hv)
    t_src = np.arange(0, blocks, dtype=np.int32)
    t_a = np.arange(blocks, 2 * blocks, dtype=np.int32)
    t_b = np.arange(2 * blocks, 3 * blocks, dtype=np.int32)
    chunk = O.Chunk(np.zeros(O.chunk_bytes(L, H, D, T, O.FMT_INT8_ROWSCALE), dtype=np.uint8),
                    O.FMT_INT8_ROWSCALE, L, H, D, T)
    cores = max(1, min(len(os.sched_getaffinity(0)), 16, L))
    bounds = [(L * i // cores, L * (i + 1) // cores) for i in range(cores)]
    slices = [chunk.slice(int(i) * (T // n_slices), T // n_slices) for i in order]

    def work(lr):
        O.store(host, t_src, 0, T, O.FMT_INT8_ROWSCALE, layers=lr, out=chunk)
        O.load(chunk, host, t_a, 0, layers=lr)
        O.compose(slices, offsets, host, t_b, base, layers=lr)

    t0 = time.perf_counter()
    for _ in range(steps):
        th = [threading.Thread(target=work, args=(b,)) for b in bounds]
        for t in th:
            t.start()
        for t in th:
            t.join()
    dt = time.perf_counter() - t0
    return {"value": T * steps / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "%d full steps of the same workload (store+load+compose of 4096 tokens, "
                      "all %d layers), layers split over %d threads" % (steps, L, cores),
            "seconds": dt}


if __name__ == "__main__":
    sys.exit(main())
