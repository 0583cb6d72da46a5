#!/usr/bin/env python3
"""Throughput of the KDN hot path on one MI355X.

Default workload ("70b_long", the largest of the five that is a whole pass of the path):
one step carries one 32768-token context of Llama-3-70B-shaped KV (80 layers, 8 KV heads,
head_dim 128, bf16, paged in blocks of 16 tokens, random block tables) through the path:
  store    paged KV -> one stored int8 chunk (15.2 GiB moved)      (kdn_store_chunk)
  compose  the chunk as 4 slices of 8192 tokens, shifted by RoPE offsets
           0 / 8192 / 16384 / 24576, into a fresh table (15.2 GiB)  (kdn_compose)
Inputs are resident in HBM before the timed region; two disjoint buffer sets alternate.  The
paged pool is sized as an engine sizes it (K and V tensors of 96 GiB each, --pool-gib) and the
block tables are drawn from all of it.
The default run then also times, more briefly, the "8b" step (4096 tokens of Llama-3-8B
shape: store, load at offset 0, compose of 8 shifted 512-token slices; four buffer sets
cycled so that the 256 MB last-level cache serves no repeat) and the "batched_reuse"
compose (64 requests x 4 chunks of 1024 tokens drawn by Zipf popularity from a resident
pool of 256 chunks, one batched launch), and a plain streaming kernel with the same byte
pattern as a yardstick; these ride in the same JSON line under "other_workloads" and
"stream_ceiling" (--only leaves them out).

Other workloads (--workload): "8b", "batched_reuse", "toy" (latency bound).

"pool_trace" is a serving loop over the text-keyed index (store on miss, compose on
hit) and reports the hit rate; "pool_trace_tiered" adds a host-memory tier under it
(demote on eviction, promote on hit).  "sweep" times store and compose over a range of
model shapes (head_dim 64..512, 1..32 KV heads) and paged block sizes (1..128).  "host_stream_int8" / "host_stream_raw" compose a chunk that lives in pinned host memory
(the rate there includes PCIe and is link bound; its roofline entry is still priced
against HBM and is not a kernel-quality figure).

Prints ONE JSON line: tokens/s over the whole step, the roofline of the dominant
kernel (the place kernel behind load and compose) from HIP-event timings, and the
CPU oracle's throughput on the host cores as a reported baseline.
"""
import argparse
import gc
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published peak
POOL_GIB_DEFAULT = 96.0     # size of each of the paged pool's K and V tensors in the default runs
METRIC = "KV tokens composed/sec (store+load+RoPE shift) and achieved HBM GB/s"
FMT_IDS = {"raw": 0, "int8": 1, "int4": 2, "fp8": 3}

# HBM bytes per k_place launch from the FETCH_SIZE / WRITE_SIZE counter runs summarised
# under profiles/ (the file named here), per workload; valid only for the library sources
# they were taken with, whose fingerprint the library itself carries.
COUNTER_TRAFFIC = {
    "source_fingerprint": "dc77886253ccca53",
    "70b_long": {"k_place_bytes_per_launch": 16274064457, "profile": "profiles/k_store_k_place_llama70b_32768tok.md"},
    "8b": {"k_place_bytes_per_launch": 813883832, "profile": "profiles/k_place_k_store_llama8b_4096tok.md"},
    "batched_reuse": {"k_place_bytes_per_launch": 41283790417, "profile": "profiles/k_place_batched_reuse_64req.md"},
}


def kernel_source_fingerprint():
    """The fingerprint of the library's sources and compiler flags (the one libkdn.so carries)."""
    from paper_2409_13761_amd import build
    return build.source_fingerprint()


def counter_traffic(workload="70b_long"):
    same = kernel_source_fingerprint() == COUNTER_TRAFFIC["source_fingerprint"]
    return COUNTER_TRAFFIC[workload]["k_place_bytes_per_launch"] if same else None


def fill_normal(t, gen):
    """N(0,1) into a bf16 tensor, one leading slab at a time (bounds the fp32 temporary)."""
    import torch
    for i in range(t.shape[0]):
        t[i].copy_(torch.randn(t.shape[1:], generator=gen, device=t.device, dtype=torch.float32))


ARENA = None                # what kdn_arena_create reported, when the run keeps its stored chunks in the striped arena


def chunk_alloc(kdn, cache, T, fmt):
    """A chunk buffer: from the striped arena when the run has one, else from torch."""
    return kdn.alloc_chunk(cache, T, fmt, arena=ARENA is not None)


def pool_tensors(args, kdn, shape, dev):
    """The paged pool's K and V tensors: torch allocations (an engine's own memory), or, with
    --pool-memory arena, cut from the library's arena like the chunks."""
    import torch
    if getattr(args, "pool_memory", "torch") == "arena" and ARENA is not None:
        n = 2
        for d in shape:
            n *= d
        return tuple(kdn.arena_tensor(n).view(torch.bfloat16).view(shape) for _ in range(2))
    k = torch.empty(shape, device=dev, dtype=torch.bfloat16)
    return k, torch.empty_like(k)


def pool_blocks_for(args, need, plane_bytes_per_block):
    """Blocks per (layer, side) plane of the paged pool.  --pool-blocks names it directly;
    otherwise --pool-gib sizes each of the K and V tensors (all layers) to that many GiB, as an
    engine does that gives most of HBM to its KV pool; never fewer than the step's tables use."""
    if args.pool_blocks:
        if args.pool_blocks < need:
            raise SystemExit("bench.py: --pool-blocks must be at least %d" % need)
        return args.pool_blocks
    return max(need, int(args.pool_gib * (1 << 30)) // plane_bytes_per_block)


class Timed:
    """Runs `step(i, rec)` W + K times; `rec(name, fn)` brackets a call with HIP events on
    the current stream (the one the library launches on) during the K timed steps."""

    def __init__(self, names, steps):
        import torch
        self.names, self.steps = names, steps
        self.ev = [{n: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                    for n in names} for _ in range(steps)]

    def run(self, step, warmup):
        import numpy as np
        import torch

        def plain(name, fn):
            fn()

        def recorder(ev):
            def rec(name, fn):
                ev[name][0].record()
                fn()
                ev[name][1].record()
            return rec

        for i in range(warmup):
            step(i, plain)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(self.steps):
            step(warmup + i, recorder(self.ev[i]))
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms = {n: float(np.mean([e[n][0].elapsed_time(e[n][1]) for e in self.ev])) for n in self.names}
        return wall, ms


def _probe_rate(kdn, torch, small, big, tiles, ids, tile_kib, direction, cap, reps):
    """GB/s of kdn_probe_stream over rotating buffer sets (HIP events on the launch stream).  Bytes per
    tile: tile_kib of the big buffer, and half as much of the small one in directions 0 and 1."""
    sets = len(small)
    for i in range(sets):
        kdn.kdn_probe_stream(small[i], big[i], tiles, ids, tile_kib, direction, cap)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        kdn.kdn_probe_stream(small[i % sets], big[i % sets], tiles, ids, tile_kib, direction, cap)
    e1.record()
    torch.cuda.synchronize()
    per_tile = tile_kib * (1536 if direction in (0, 1) else 1024)
    return tiles * per_tile / (e0.elapsed_time(e1) / reps * 1e-3) / 1e9


def stream_ceiling(dev, pool_gib):
    """The box's own yardstick: the library's plain streaming kernel (kdn_probe_stream: per
    workgroup one 32 KiB tile of the big buffer and 16 KiB of the small one, no arithmetic, no
    table walk), 32768 tiles = 1.61 GB per launch.  The big buffer is as large as the paged
    pool's two tensors; in the pattern of load and compose (small -> big) the written tiles
    are taken in order, scattered over the whole of it (as the blocks of a random table over an
    engine-sized pool are) and scattered inside 16 GiB of it; in the pattern of store
    (big -> small) the read tiles are scattered over the whole of it."""
    import numpy as np
    import torch
    from paper_2409_13761_amd import kdn, synth
    tiles, sets, reps = 32768, 3, 12
    big_gib = max(16, int(2 * pool_gib))
    plain = [torch.empty(tiles * 16384, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(sets)]
    small = plain
    if ARENA is not None:       # the small buffers stand for the stored chunks: they lie where the chunks lie
        small = [kdn.arena_tensor(tiles * 16384) for _ in range(sets)]
        for a, b in zip(small, plain):
            a.copy_(b)
    big = [torch.empty(big_gib << 30, dtype=torch.uint8, device=dev)] * sets
    rng = synth._rng(4242, 1)
    wide = torch.from_numpy(rng.permutation(big_gib * 32768)[:tiles].astype(np.int32)).to(dev)
    narrow = torch.from_numpy(rng.permutation(16 * 32768)[:tiles].astype(np.int32)).to(dev)
    out = {"place_pattern_contiguous_GBps": _probe_rate(kdn, torch, small, big, tiles, None, 32, 0, 0, reps),
           "place_pattern_scattered_GBps": _probe_rate(kdn, torch, small, big, tiles, wide, 32, 0, 0, reps),
           "place_pattern_scattered_within_16GiB_GBps": _probe_rate(kdn, torch, small, big, tiles, narrow, 32, 0, 0, reps),
           "store_pattern_scattered_GBps": _probe_rate(kdn, torch, small, big, tiles, wide, 32, 1, 0, reps)}
    # the two directions of the memory on their own, over the same big buffer (1.07 GB per launch)
    out["one_direction_GBps"] = {
        "read_in_order": _probe_rate(kdn, torch, small, big, tiles, None, 32, 3, 0, reps),
        "read_scattered": _probe_rate(kdn, torch, small, big, tiles, wide, 32, 3, 0, reps),
        "write_in_order": _probe_rate(kdn, torch, small, big, tiles, None, 32, 2, 0, reps),
        "write_scattered": _probe_rate(kdn, torch, small, big, tiles, wide, 32, 2, 0, reps),
        "write_scattered_within_16GiB": _probe_rate(kdn, torch, small, big, tiles, narrow, 32, 2, 0, reps)}
    if ARENA is not None:
        out["store_pattern_scattered_small_buffer_in_plain_memory_GBps"] = _probe_rate(kdn, torch, plain, big, tiles, wide,
                                                                                       32, 1, 0, reps)
        out["place_pattern_scattered_small_buffer_in_plain_memory_GBps"] = _probe_rate(kdn, torch, plain, big, tiles, wide,
                                                                                       32, 0, 0, reps)
    out["what"] = ("kdn_probe_stream, one workgroup per tile (32 KiB of the big buffer, 16 KiB of the small one), streamed, "
                   "no arithmetic; %d tiles (%.2f GB) per launch, HIP events; big buffer of %d GiB (the size of the paged "
                   "pool). place pattern = read small, write big (load, compose); store pattern = read big, write small; "
                   "scattered = the big buffer's tiles drawn at random from all of it (or from its first 16 GiB), like "
                   "the blocks of a random table; the small buffers lie in %s"
                   % (tiles, tiles * 49152 / 1e9, big_gib, "the striped arena, as the stored chunks do" if ARENA is not None
                      else "plain device memory"))
    return out


def workload_stream_probe(args, dev):
    """The streaming yardstick over tile sizes and launch widths: what a kernel with nothing to
    compute reaches with the byte pattern of load/compose (16 KiB read, 32 KiB written per tile at the
    Llama shapes and block size 16) when the written tiles are in order or scattered, and how that moves
    with the tile size (the engine's block size) and with the number of workgroups in flight."""
    import numpy as np
    import torch
    from paper_2409_13761_amd import kdn, synth
    sets, reps, total_kib = 3, args.steps, 1 << 20            # 1 GiB of the big buffer per launch
    small = [torch.empty(total_kib * 512, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(sets)]
    big = [torch.empty(total_kib * 1024, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(sets)]
    rows = []
    for tile_kib in (8, 16, 32, 64, 128, 256, 1024, 4096):
        tiles = total_kib // tile_kib
        ids = torch.from_numpy(synth.permutation(4242 + tile_kib, tiles).astype("int32")).to(dev)
        rows.append({"tile_KiB": tile_kib, "workgroups": tiles,
                     "place_contiguous_GBps": _probe_rate(kdn, torch, small, big, tiles, None, tile_kib, 0, 0, reps),
                     "place_scattered_GBps": _probe_rate(kdn, torch, small, big, tiles, ids, tile_kib, 0, 0, reps),
                     "store_scattered_GBps": _probe_rate(kdn, torch, small, big, tiles, ids, tile_kib, 1, 0, reps)})
    tiles = total_kib // 32
    ids = torch.from_numpy(synth.permutation(4242 + 32, tiles).astype("int32")).to(dev)
    caps = []
    for cap in (256, 512, 1024, 2048, 4096, 0):
        caps.append({"max_workgroups": cap or tiles,
                     "place_contiguous_GBps": _probe_rate(kdn, torch, small, big, tiles, None, 32, 0, cap, reps),
                     "place_scattered_GBps": _probe_rate(kdn, torch, small, big, tiles, ids, 32, 0, cap, reps)})
    windows = []
    rng = np.random.default_rng(4242)
    for w_tiles in (1, 64, 256, 1024, 4096, tiles):      # tiles shuffled only within windows of this many tiles
        local = np.stack([rng.permutation(r) for r in np.arange(tiles).reshape(-1, w_tiles)]).reshape(-1)
        local_ids = torch.from_numpy(local.astype(np.int32)).to(dev)
        windows.append({"window_MiB": w_tiles / 32,
                        "place_scattered_GBps": _probe_rate(kdn, torch, small, big, tiles, local_ids, 32, 0, 0, reps)})
    # where in the device memory the scattered tiles lie: one 200 GiB allocation, tiles drawn from parts of it
    spans = []
    del big
    torch.cuda.empty_cache()
    huge = torch.empty(200 << 30, dtype=torch.uint8, device=dev)
    per_gib = (1 << 30) // 32768
    for what, parts in (("16 GiB at the start", [(0, 16)]), ("16 GiB, 100 GiB in", [(100, 16)]),
                        ("8 GiB at the start + 8 GiB, 104 GiB in", [(0, 8), (104, 8)]),
                        ("8 GiB at 40 GiB + 8 GiB at 72 GiB", [(40, 8), (72, 8)]),
                        ("three times 5 GiB, 96 GiB apart", [(0, 5), (96, 5), (192, 5)]),
                        ("all 200 GiB", [(0, 200)])):
        pool_ids = np.concatenate([np.arange(a * per_gib, (a + n) * per_gib) for a, n in parts])
        pick = rng.permutation(pool_ids.size)[:tiles]
        span_ids = torch.from_numpy(pool_ids[pick].astype(np.int32)).to(dev)
        spans.append({"tiles_drawn_from": what,
                      "place_scattered_GBps": _probe_rate(kdn, torch, small, [huge] * sets, tiles, span_ids, 32, 0, 0, reps),
                      "store_scattered_GBps": _probe_rate(kdn, torch, small, [huge] * sets, tiles, span_ids, 32, 1, 0, reps),
                      "write_only_scattered_GBps": _probe_rate(kdn, torch, small, [huge] * sets, tiles, span_ids, 32, 2, 0, reps),
                      "read_only_scattered_GBps": _probe_rate(kdn, torch, small, [huge] * sets, tiles, span_ids, 32, 3, 0, reps)})
    # tile sizes again, now with the tiles scattered over all 200 GiB (the regime an engine-sized pool is in)
    wide_rows = []
    for tile_kib in (4, 8, 16, 32, 64, 256, 1024):
        n_t = (1 << 30) // (tile_kib << 10)
        wide_ids = torch.from_numpy(rng.permutation((200 << 30) // (tile_kib << 10))[:n_t].astype(np.int32)).to(dev)
        wide_rows.append({"tile_KiB": tile_kib,
                          "place_scattered_GBps": _probe_rate(kdn, torch, small, [huge] * sets, n_t, wide_ids, tile_kib, 0, 0, reps),
                          "store_scattered_GBps": _probe_rate(kdn, torch, small, [huge] * sets, n_t, wide_ids, tile_kib, 1, 0, reps)})
    one_way = {"read_in_order_GBps": _probe_rate(kdn, torch, small, [huge] * sets, tiles, None, 32, 3, 0, reps),
               "write_in_order_GBps": _probe_rate(kdn, torch, small, [huge] * sets, tiles, None, 32, 2, 0, reps)}
    del huge
    r32 = rows[2]
    ms = {"place_scattered": 1.5 * (1 << 30) / r32["place_scattered_GBps"] / 1e6}
    return {
        "tokens_per_step": 0, "wall": ms["place_scattered"] * 1e-3 * args.steps, "ms": ms,
        "bytes": {"place_scattered": int(1.5 * (1 << 30))},
        "place_calls": ("place_scattered",),
        "workload": "stream_probe: kdn_probe_stream (no arithmetic, no table walk) moving 0.5 GiB of a small buffer and 1 GiB "
                    "of a big one per launch, by tile size and by launch width; the headline fields are the 32 KiB-tile, "
                    "scattered, place-pattern row (no tokens are moved: value is 0)",
        "extra": {"by_tile_size": rows, "by_launch_width_at_32KiB_tiles": caps,
                  "by_scatter_window_at_32KiB_tiles": windows,
                  "by_span_of_device_memory_at_32KiB_tiles": spans,
                  "one_direction_in_order_at_32KiB_tiles": one_way,
                  "by_tile_size_scattered_over_200GiB": wide_rows},
        "traffic": None,
    }


def workload_8b(args, dev):
    import torch
    from paper_2409_13761_amd import kdn, synth

    sh = synth.LLAMA8B
    T, n_slices = 4096, 8
    w = synth.WORKLOADS["rag_compose"]
    blocks = T // sh.bs
    n_sets = 4
    nb = pool_blocks_for(args, n_sets * 3 * blocks, sh.L * sh.bs * sh.H * sh.D * 2)
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    if args.layout == "planes":         # K and V tensors [L][num_blocks][bs][H][D]
        k, v = pool_tensors(args, kdn, (sh.L, nb, sh.bs, sh.H, sh.D), dev)
    elif args.layout == "kv_pair":      # one tensor [L][num_blocks][2][bs][H][D]: a block's K and V adjoin
        big = torch.empty((sh.L, nb, 2, sh.bs, sh.H, sh.D), device=dev, dtype=torch.bfloat16)
        k, v = big[:, :, 0], big[:, :, 1]
    else:                               # block_major: [num_blocks][L][2][bs][H][D], a block is one 2 MiB run
        big = torch.empty((nb, sh.L, 2, sh.bs, sh.H, sh.D), device=dev, dtype=torch.bfloat16)
        k, v = big[:, :, 0].permute(1, 0, 2, 3, 4), big[:, :, 1].permute(1, 0, 2, 3, 4)
    fill_normal(k, g)
    fill_normal(v, g)
    cache = kdn.PagedCache(k, v)
    if args.tables == "random":
        tables = synth.disjoint_block_tables(w.seed, nb, [blocks] * (3 * n_sets))
    else:   # every table a run of consecutive blocks: what the kernels do when the engine places a request so
        import numpy as np
        tables = [np.arange(i * blocks, (i + 1) * blocks, dtype=np.int32) for i in range(3 * n_sets)]
    order = synth.permutation(w.seed, n_slices)
    offsets = [int(j * (T // n_slices)) for j in range(n_slices)]   # j-th placed slice moves by 512*j
    sets = []
    for s in range(n_sets):
        src, dst_a, dst_b = (torch.from_numpy(tables[3 * s + i]).to(dev) for i in range(3))
        chunk = chunk_alloc(kdn, cache, T, FMT_IDS[args.fmt])
        slices = [chunk.slice(int(i) * (T // n_slices), T // n_slices) for i in order]
        sets.append((src, dst_a, dst_b, chunk, slices))
    kdn.kdn_rope_prepare(w.rope_base, sh.D, offsets)
    for s in range(n_sets):                     # every chunk exists before any is read
        kdn.kdn_store_chunk(cache, sets[s][0], 0, T, sets[s][3])

    def step(i, rec):
        # The chunk a step loads or composes was stored two or three steps earlier, with
        # gigabytes of traffic in between, so it comes from HBM, not from the cache.
        src, dst_a, dst_b, chunk, _ = sets[i % n_sets]
        load_chunk = sets[(i + 2) % n_sets][3]
        compose_slices = sets[(i + 1) % n_sets][4]
        rec("store", lambda: kdn.kdn_store_chunk(cache, src, 0, T, chunk))
        rec("load", lambda: kdn.kdn_load_chunk(load_chunk, cache, dst_a, 0))
        rec("compose", lambda: kdn.kdn_compose(compose_slices, offsets, cache, dst_b, w.rope_base))

    wall, ms = Timed(("store", "load", "compose"), args.steps).run(step, args.warmup)
    bytes_call = T * (sh.paged_bytes_per_token + sh.stored_bytes_per_token(args.fmt))   # B_p + B_q per token
    res = {
        "tokens_per_step": T, "wall": wall, "ms": ms,
        "bytes": {n: bytes_call for n in ms},
        "place_calls": ("load", "compose"),
        "workload": "Llama-3-8B-shaped KV (L32 H8 D128 bs16): per step store 4096 tokens to %s, "
                    "load them at offset 0, compose them as 8x512-token slices in seeded order with "
                    "RoPE offsets 0..3584 (base %g); %d buffer sets cycled; cache layout %s, pool of %d blocks (%s); %s block "
                    "tables; chunk buffers in %s"
                    % (args.fmt, w.rope_base, n_sets, args.layout, nb,
                       "in the striped arena" if args.pool_memory == "arena" and ARENA is not None else "a torch allocation",
                       "random disjoint" if args.tables == "random" else "consecutive-block",
                       "the striped arena" if ARENA is not None else "plain device memory"),
        "traffic": counter_traffic("8b") if args.fmt == "int8" and args.tables == "random" and args.layout == "planes"
        and not args.pool_blocks and args.pool_gib == POOL_GIB_DEFAULT and args.pool_memory == "torch" else None,
    }
    if not args.no_cpu_baseline and args.fmt == "int8":
        res["cpu_baseline"] = cpu_baseline(kdn, cache, sets[0], order, offsets, w.rope_base, T, n_slices,
                                           args.cpu_steps)
    return res


def workload_toy(args, dev):
    """The toy workload: 2 layers, 4 KV heads, head_dim 64, 128 blocks; two 256-token chunks
    stored, then composed at offsets 0 and 256.  About 1.5 MB per call: launch latency, not
    bandwidth, is what this measures."""
    import torch
    from paper_2409_13761_amd import kdn, synth

    w = synth.WORKLOADS["toy"]
    sh, nb = w.shape, 128
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    k = torch.empty((sh.L, nb, sh.bs, sh.H, sh.D), device=dev, dtype=torch.bfloat16)
    v = torch.empty_like(k)
    fill_normal(k, g)
    fill_normal(v, g)
    cache = kdn.PagedCache(k, v)
    t1, t2, dst = (torch.from_numpy(t).to(dev) for t in synth.disjoint_block_tables(w.seed, nb, [16, 16, 32]))
    c1 = kdn.alloc_chunk(cache, 256, FMT_IDS[args.fmt])
    c2 = kdn.alloc_chunk(cache, 256, FMT_IDS[args.fmt])
    offsets = list(w.offsets)
    kdn.kdn_rope_prepare(w.rope_base, sh.D, offsets)

    def step(i, rec):
        rec("store", lambda: (kdn.kdn_store_chunk(cache, t1, 0, 256, c1), kdn.kdn_store_chunk(cache, t2, 0, 256, c2)))
        rec("compose", lambda: kdn.kdn_compose([c1, c2], offsets, cache, dst, w.rope_base))

    wall, ms = Timed(("store", "compose"), args.steps).run(step, args.warmup)
    # the same three launches captured once into a HIP graph and replayed (kernels only: the
    # cos/sin rows are resident and the segments travel in the kernel arguments)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(0, lambda name, fn: fn())
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    graph_wall = time.perf_counter() - t0
    bytes_call = 512 * (sh.paged_bytes_per_token + sh.stored_bytes_per_token(args.fmt))
    return {
        "tokens_per_step": 512, "wall": wall, "ms": ms, "bytes": {n: bytes_call for n in ms},
        "place_calls": ("compose",),
        "workload": "toy KV (L2 H4 D64 bs16, 128 blocks): per step store two 256-token chunks to %s "
                    "(two calls) and compose them at offsets 0 and 256, base 10000; latency bound" % args.fmt,
        "extra": {"ms_per_step_as_hip_graph_replay": graph_wall / args.steps * 1e3,
                  "tokens_per_s_as_hip_graph_replay": 512 * args.steps / graph_wall},
        "traffic": None,
    }


def workload_70b(args, dev):
    import torch
    from paper_2409_13761_amd import kdn, synth

    w = synth.WORKLOADS["70b_long"]
    sh, T = w.shape, 32768
    blocks = T // sh.bs
    n_sets = 2
    nb = pool_blocks_for(args, n_sets * 2 * blocks, sh.L * sh.bs * sh.H * sh.D * 2)
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    k, v = pool_tensors(args, kdn, (sh.L, nb, sh.bs, sh.H, sh.D), dev)
    fill_normal(k, g)
    fill_normal(v, g)
    cache = kdn.PagedCache(k, v)
    tables = synth.disjoint_block_tables(w.seed, nb, [blocks] * (2 * n_sets))
    offsets = list(w.offsets)
    sets = []
    for s in range(n_sets):
        src, dst = (torch.from_numpy(tables[2 * s + i]).to(dev) for i in range(2))
        chunk = chunk_alloc(kdn, cache, T, FMT_IDS[args.fmt])
        sets.append((src, dst, chunk, [chunk.slice(i * 8192, 8192) for i in range(4)]))
    kdn.kdn_rope_prepare(w.rope_base, sh.D, offsets)

    def step(i, rec):
        src, dst, chunk, slices = sets[i % n_sets]
        rec("store", lambda: kdn.kdn_store_chunk(cache, src, 0, T, chunk))
        rec("compose", lambda: kdn.kdn_compose(slices, offsets, cache, dst, w.rope_base))

    wall, ms = Timed(("store", "compose"), args.steps).run(step, args.warmup)
    bytes_call = T * (sh.paged_bytes_per_token + sh.stored_bytes_per_token(args.fmt))
    extra = {}
    if ARENA is not None and not args.only:     # the same two calls with the chunk in plain device memory, for the difference
        plain = kdn.alloc_chunk(cache, T, FMT_IDS[args.fmt])
        plain_slices = [plain.slice(i * 8192, 8192) for i in range(4)]

        def plain_step(i, rec):
            src, dst = sets[i % n_sets][:2]
            rec("store", lambda: kdn.kdn_store_chunk(cache, src, 0, T, plain))
            rec("compose", lambda: kdn.kdn_compose(plain_slices, offsets, cache, dst, w.rope_base))

        _, plain_ms = Timed(("store", "compose"), max(4, args.steps // 2)).run(plain_step, 2)
        extra["GBps_with_the_chunk_in_plain_device_memory"] = {n: bytes_call / (plain_ms[n] * 1e-3) / 1e9
                                                               for n in plain_ms}
        del plain, plain_slices
    res = {
        "tokens_per_step": T, "wall": wall, "ms": ms, "bytes": {n: bytes_call for n in ms},
        "place_calls": ("compose",),
        "workload": "70b_long: Llama-3-70B-shaped KV (L80 H8 D128 bs16), per step store 32768 tokens to %s (one call) "
                    "and compose them back as 4x8192-token slices with RoPE offsets 0/8192/16384/24576 (base %g) "
                    "into a fresh table; random disjoint block tables in a paged pool of %d blocks (K and V tensors of "
                    "%.1f GiB each); %d buffer sets cycled; chunk buffers in %s"
                    % (args.fmt, w.rope_base, nb, nb * sh.L * sh.bs * sh.H * sh.D * 2 / 2 ** 30, n_sets,
                       "the striped arena" if ARENA is not None else "plain device memory"),
        "extra": extra,
        "traffic": counter_traffic("70b_long") if args.fmt == "int8" and not args.pool_blocks
        and args.pool_gib == POOL_GIB_DEFAULT and args.pool_memory == "torch" else None,
    }
    if not args.no_cpu_baseline and args.fmt == "int8":
        res["cpu_baseline"] = cpu_baseline_70b(kdn, cache, sets[0], offsets, w.rope_base, T, args.cpu_layers)
    return res


def workload_batched(args, dev):
    import numpy as np
    import torch
    from paper_2409_13761_amd import kdn, synth

    w = synth.WORKLOADS["batched_reuse"]
    sh = w.shape
    n_pool, n_req, per_req, Tc = w.extra["pool"], w.extra["requests"], 4, 1024
    cb = Tc // sh.bs
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    # the pool: 256 chunks stored from 16 rounds of a 16384-token source cache
    rb = 16 * cb
    k = torch.empty((sh.L, rb, sh.bs, sh.H, sh.D), device=dev, dtype=torch.bfloat16)
    v = torch.empty_like(k)
    src_cache = kdn.PagedCache(k, v)
    pool = []
    for rnd in range(n_pool // 16):
        fill_normal(k, g)
        fill_normal(v, g)
        perm = synth.permutation(w.seed + 100 + rnd, rb)
        for i in range(16):
            out = chunk_alloc(kdn, src_cache, Tc, kdn.FMT_INT8_ROWSCALE)
            kdn.kdn_store_chunk(src_cache, torch.from_numpy(perm[i * cb:(i + 1) * cb].copy()).to(dev), 0, Tc, out)
            pool.append(out)
        torch.cuda.synchronize()
    del k, v, src_cache
    draws = synth.zipf_distinct_draws(w.seed, n_req, per_req, n_pool, w.extra["alpha"])
    blocks_req = per_req * cb
    nb = pool_blocks_for(args, n_req * blocks_req, sh.L * sh.bs * sh.H * sh.D * 2)
    tables = synth.disjoint_block_tables(w.seed, nb, [blocks_req] * n_req)
    dst = kdn.PagedCache(torch.empty((sh.L, nb, sh.bs, sh.H, sh.D), device=dev, dtype=torch.bfloat16),
                         torch.empty((sh.L, nb, sh.bs, sh.H, sh.D), device=dev, dtype=torch.bfloat16))
    offsets = list(w.offsets)
    plan = kdn.BatchPlan([([pool[int(c)] for c in draws[r]], offsets, torch.from_numpy(tables[r]).to(dev), 0)
                          for r in range(n_req)])
    kdn.kdn_rope_prepare(w.rope_base, sh.D, offsets)

    def step(i, rec):
        rec("compose_batch", lambda: kdn.kdn_compose_batch(plan, dst, w.rope_base))

    wall, ms = Timed(("compose_batch",), args.steps).run(step, args.warmup)
    tokens = n_req * per_req * Tc
    unique = int(len(np.unique(draws)))
    # HBM bytes: every destination row written once, every DISTINCT chunk read once (a chunk that
    # several requests draw is served from the caches after its first reader)
    once = unique * Tc * sh.int8_bytes_per_token + tokens * sh.paged_bytes_per_token
    naive = tokens * (sh.paged_bytes_per_token + sh.int8_bytes_per_token)
    return {
        "tokens_per_step": tokens, "wall": wall, "ms": ms,
        "bytes": {"compose_batch": once},
        "place_calls": ("compose_batch",),
        "workload": "batched_reuse (L32 H8 D128 bs16): 64 requests x 4 chunks of 1024 tokens drawn by "
                    "Zipf(1.0) from a resident pool of 256 int8 chunks (%d distinct drawn), one batched "
                    "compose per step into 64 disjoint random tables in a paged pool of %d blocks (K and V tensors of "
                    "%.1f GiB each)" % (unique, nb, nb * sh.L * sh.bs * sh.H * sh.D * 2 / 2 ** 30),
        "extra": {"distinct_chunks": unique,
                  "bytes_counted": "each distinct chunk read once + every destination row written",
                  "bytes_if_every_draw_were_read_from_hbm": naive,
                  "GBps_if_every_draw_were_read_from_hbm": naive / (ms["compose_batch"] * 1e-3) / 1e9},
        "traffic": counter_traffic("batched_reuse") if not args.pool_blocks and args.pool_gib == POOL_GIB_DEFAULT
        else None,
    }


def workload_host_stream(args, dev, fmt_name):
    """A 4096-token context is stored into pinned host memory and composed back from there as
    8 shifted slices, two ways: with the kernels addressing the host chunk themselves
    ("direct"), and staged through HBM by the copy engines, 8 layers per stage, while the
    neighbouring stage is quantised (store) or dequantised and scattered (compose).  In both
    only the compact rows cross PCIe.  The rates are link bound (PCIe-inclusive)."""
    import torch
    from paper_2409_13761_amd import kdn, synth

    sh = synth.LLAMA8B
    T, n_slices = 4096, 8
    w = synth.WORKLOADS["rag_compose"]
    fmt = kdn.FMT_INT8_ROWSCALE if fmt_name == "int8" else kdn.FMT_RAW_BF16
    blocks = T // sh.bs
    nb = 3 * blocks
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    k = torch.empty((sh.L, nb, sh.bs, sh.H, sh.D), device=dev, dtype=torch.bfloat16)
    v = torch.empty_like(k)
    fill_normal(k, g)
    fill_normal(v, g)
    cache = kdn.PagedCache(k, v)
    src, dst_a, dst_b = (torch.from_numpy(t).to(dev) for t in
                         synth.disjoint_block_tables(w.seed, nb, [blocks] * 3))
    chunk = kdn.alloc_chunk(cache, T, fmt)
    kdn.kdn_store_chunk(cache, src, 0, T, chunk)
    torch.cuda.synchronize()
    host = kdn.pinned_host_copy(chunk)
    order = synth.permutation(w.seed, n_slices)
    slices = [host.slice(int(i) * (T // n_slices), T // n_slices) for i in order]
    offsets = [int(j * (T // n_slices)) for j in range(n_slices)]
    lps = 8        # 4 stages: few copies outstanding at a time (the runtime slows down beyond about a dozen)
    staging = torch.empty(max(kdn.kdn_staging_bytes(slices, lps), kdn.kdn_store_staging_bytes(cache, T, fmt, lps)),
                          dtype=torch.uint8, device=dev)
    kdn.kdn_rope_prepare(w.rope_base, sh.D, offsets)
    dsts = (dst_a, dst_b)

    def step(i, rec):
        # the host chunk is rewritten with the same bytes it already holds
        rec("store_direct", lambda: kdn.kdn_store_chunk(cache, src, 0, T, host))
        rec("compose_direct", lambda: kdn.kdn_compose(slices, offsets, cache, dsts[i % 2], w.rope_base))
        rec("store_to_host", lambda: kdn.kdn_store_to_host(cache, src, 0, T, host, staging, lps))
        rec("compose_from_host", lambda: kdn.kdn_compose_from_host(
            slices, offsets, cache, dsts[i % 2], w.rope_base, staging, lps))
        # one step at a time: with hundreds of staged copies queued ahead the runtime now and then runs
        # a call's copies several times slower (seen with any copy path, not with the kernels)
        torch.cuda.current_stream().synchronize()

    names = ("store_direct", "compose_direct", "store_to_host", "compose_from_host")
    wall, ms = Timed(names, args.steps).run(step, args.warmup)
    stored = T * (sh.int8_bytes_per_token if fmt_name == "int8" else sh.paged_bytes_per_token)
    moved = stored + T * sh.paged_bytes_per_token
    return {
        "tokens_per_step": 2 * T, "wall": wall, "ms": ms,
        "bytes": {n: moved for n in names},
        "place_calls": ("compose_direct",),
        "workload": "Llama-3-8B-shaped KV: 4096 tokens stored as one %s chunk into pinned host memory and "
                    "composed back from there as 8x512-token shifted slices, once by kernels addressing "
                    "host memory and once staged by the copy engines, %d layers per stage "
                    "(PCIe-inclusive, link bound)" % (fmt_name, lps),
        "extra": {"stored_bytes_over_link_each_way": stored,
                  "link_GBps": {n: stored / (ms[n] * 1e-3) / 1e9 for n in ms}},
        "traffic": None,
    }


def workload_pool_trace(args, dev):
    """Serving loop over the text-keyed index: each step is one request that names 4 of 256
    texts by Zipf(1.0) popularity.  A text whose KV is resident is a hit; on a miss its KV
    is stored (int8) from the engine's paged memory into a buffer taken from the evicted
    entries, and indexed.  The 4 chunks are then composed into the request's block table.
    The index holds 64 chunks of 1024 tokens."""
    import numpy as np
    import torch
    from paper_2409_13761_amd import kdn, synth

    w = synth.WORKLOADS["batched_reuse"]
    sh = w.shape
    n_texts, per_req, Tc, resident = w.extra["pool"], 4, 1024, 64
    cb = Tc // sh.bs
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    n_src = 16                                   # distinct source contexts standing in for 256 texts
    nb = n_src * cb + 2 * per_req * cb
    k = torch.empty((sh.L, nb, sh.bs, sh.H, sh.D), device=dev, dtype=torch.bfloat16)
    v = torch.empty_like(k)
    fill_normal(k, g)
    fill_normal(v, g)
    cache = kdn.PagedCache(k, v)
    tabs = synth.disjoint_block_tables(w.seed, nb, [cb] * n_src + [per_req * cb] * 2)
    src_tabs = [torch.from_numpy(t).to(dev) for t in tabs[:n_src]]
    dst_tabs = [torch.from_numpy(t).to(dev) for t in tabs[n_src:]]
    chunk_bytes = kdn.kdn_chunk_bytes(sh.L, sh.H, sh.D, Tc, kdn.FMT_INT8_ROWSCALE)
    free = [chunk_alloc(kdn, cache, Tc, kdn.FMT_INT8_ROWSCALE) for _ in range(resident + per_req)]
    by_ptr = {c.data.data_ptr(): c for c in free}
    pool = kdn.Pool(resident * chunk_bytes, 0)
    total = args.warmup + args.steps
    draws = synth.zipf_distinct_draws(w.seed, total, per_req, n_texts, w.extra["alpha"])
    text_ids = [np.ascontiguousarray(synth._rng(w.seed + 7, 100 + t).integers(0, 128000, size=Tc), dtype=np.int32)
                for t in range(n_texts)]
    offsets = list(w.offsets)
    kdn.kdn_rope_prepare(w.rope_base, sh.D, offsets)
    counts = {"hit": 0, "miss": 0}

    def step(i, rec):
        def body():
            chunks = []
            for t in draws[i]:
                t = int(t)
                d = pool.lookup(text_ids[t])
                if d is None:
                    counts["miss"] += 1
                    buf = free.pop()
                    kdn.kdn_store_chunk(cache, src_tabs[t % n_src], 0, Tc, buf)
                    for e in pool.insert(text_ids[t], buf.desc):
                        free.append(by_ptr[e.data])
                    chunks.append(buf)
                else:
                    counts["hit"] += 1
                    chunks.append(by_ptr[d.data])
            kdn.kdn_compose(chunks, offsets, cache, dst_tabs[i % 2], w.rope_base)
        rec("request", body)

    wall, ms = Timed(("request",), args.steps).run(step, args.warmup)
    st = pool.stats()
    tokens = per_req * Tc
    return {
        "tokens_per_step": tokens, "wall": wall, "ms": ms,
        "bytes": {"request": tokens * (sh.paged_bytes_per_token + sh.int8_bytes_per_token)},
        "place_calls": ("request",),
        "workload": "serving loop over the text-keyed index (L32 H8 D128 bs16): per step one request of 4 "
                    "texts of 1024 tokens drawn by Zipf(1.0) from 256; store-on-miss (int8) into an index of "
                    "%d resident chunks (LRU), then one compose of the 4 chunks" % resident,
        "extra": {"hit_rate": st.hits / max(1, st.hits + st.misses), "hits": st.hits, "misses": st.misses,
                  "evictions": st.evictions,
                  "note": "the request figure counts the compose bytes only; misses add a store each"},
        "traffic": None,
    }


def workload_pool_trace_tiered(args, dev):
    """The serving loop of "pool_trace" with a second tier: 64 chunks resident in HBM, 128 more
    in pinned host memory, each with its own text-keyed index (LRU).  A chunk evicted from HBM
    is demoted to the host tier (its compact bytes copied out); a text found there is promoted
    back (copied in, host entry released); a text found nowhere is stored from paged memory.
    The request's 4 chunks are then composed from HBM."""
    import numpy as np
    import torch
    from paper_2409_13761_amd import kdn, synth

    w = synth.WORKLOADS["batched_reuse"]
    sh = w.shape
    n_texts, per_req, Tc, in_hbm, in_host = w.extra["pool"], 4, 1024, 64, 128
    cb = Tc // sh.bs
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    n_src = 16
    nb = n_src * cb + 2 * per_req * cb
    k = torch.empty((sh.L, nb, sh.bs, sh.H, sh.D), device=dev, dtype=torch.bfloat16)
    v = torch.empty_like(k)
    fill_normal(k, g)
    fill_normal(v, g)
    cache = kdn.PagedCache(k, v)
    tabs = synth.disjoint_block_tables(w.seed, nb, [cb] * n_src + [per_req * cb] * 2)
    src_tabs = [torch.from_numpy(t).to(dev) for t in tabs[:n_src]]
    dst_tabs = [torch.from_numpy(t).to(dev) for t in tabs[n_src:]]
    fmt = kdn.FMT_INT8_ROWSCALE
    chunk_bytes = kdn.kdn_chunk_bytes(sh.L, sh.H, sh.D, Tc, fmt)
    dev_free = [chunk_alloc(kdn, cache, Tc, fmt) for _ in range(in_hbm + per_req)]
    host_free = [kdn.alloc_host_chunk(cache, Tc, fmt) for _ in range(in_host + per_req)]
    by_ptr = {c.data.data_ptr(): c for c in dev_free + host_free}
    text_of = {}                                  # buffer address -> text it holds
    hbm, host = kdn.Pool(in_hbm * chunk_bytes, 0), kdn.Pool(in_host * chunk_bytes, 0)
    total = args.warmup + args.steps
    draws = synth.zipf_distinct_draws(w.seed, total, per_req, n_texts, w.extra["alpha"])
    text_ids = [np.ascontiguousarray(synth._rng(w.seed + 7, 100 + t).integers(0, 128000, size=Tc), dtype=np.int32)
                for t in range(n_texts)]
    offsets = list(w.offsets)
    kdn.kdn_rope_prepare(w.rope_base, sh.D, offsets)
    counts = {"hbm_hit": 0, "host_hit": 0, "miss": 0, "demoted": 0}

    def into_hbm(t, buf):
        """Index `buf` (already holding text t) in the HBM tier; what falls out goes to the host tier."""
        text_of[buf.data.data_ptr()] = t
        for e in hbm.insert(text_ids[t], buf.desc):
            out_dev = by_ptr[e.data]
            out_t = text_of.pop(e.data)
            hbuf = host_free.pop()
            hbuf.data.copy_(out_dev.data, non_blocking=True)          # compact bytes, device to host
            counts["demoted"] += 1
            text_of[hbuf.data.data_ptr()] = out_t
            for he in host.insert(text_ids[out_t], hbuf.desc):
                text_of.pop(he.data)
                host_free.append(by_ptr[he.data])
            dev_free.append(out_dev)

    def step(i, rec):
        def body():
            chunks = []
            for t in draws[i]:
                t = int(t)
                d = hbm.lookup(text_ids[t])
                if d is not None:
                    counts["hbm_hit"] += 1
                    chunks.append(by_ptr[d.data])
                    continue
                buf = dev_free.pop()
                hd = host.remove(text_ids[t])
                if hd is not None:
                    counts["host_hit"] += 1
                    hbuf = by_ptr[hd.data]
                    buf.data.copy_(hbuf.data, non_blocking=True)      # promotion: host to device
                    text_of.pop(hd.data)
                    host_free.append(hbuf)
                else:
                    counts["miss"] += 1
                    kdn.kdn_store_chunk(cache, src_tabs[t % n_src], 0, Tc, buf)
                into_hbm(t, buf)
                chunks.append(buf)
            kdn.kdn_compose(chunks, offsets, cache, dst_tabs[i % 2], w.rope_base)
        rec("request", body)

    wall, ms = Timed(("request",), args.steps).run(step, args.warmup)
    tokens = per_req * Tc
    n = sum(counts[k_] for k_ in ("hbm_hit", "host_hit", "miss"))
    return {
        "tokens_per_step": tokens, "wall": wall, "ms": ms,
        "bytes": {"request": tokens * (sh.paged_bytes_per_token + sh.int8_bytes_per_token)},
        "place_calls": ("request",),
        "workload": "serving loop over two tiers of the text-keyed index (L32 H8 D128 bs16): per step one request "
                    "of 4 texts of 1024 tokens drawn by Zipf(1.0) from 256; %d chunks resident in HBM, %d in pinned "
                    "host memory (LRU each); demote on HBM eviction, promote on host hit, store (int8) on miss; "
                    "then one compose of the 4 chunks" % (in_hbm, in_host),
        "extra": {"hbm_hit_rate": counts["hbm_hit"] / n, "host_hit_rate": counts["host_hit"] / n,
                  "miss_rate": counts["miss"] / n, "demotions": counts["demoted"],
                  "link_bytes_per_promotion_or_demotion": chunk_bytes,
                  "note": "counts include the warm-up requests; the request figure counts the compose bytes only; "
                          "a miss adds a store, a host hit a copy over the link, an HBM eviction another; the "
                          "prefill that would produce a missing text's KV is outside this path"},
        "traffic": None,
    }


SWEEP_SHAPES = (
    # (L, H, D, block size, note): 4096 tokens each, stored and composed back as 8 shifted slices
    (32, 8, 128, 16, "Llama-3-8B shape (the default workload's)"),
    (32, 32, 128, 16, "32 KV heads (no grouped-query sharing)"),
    (32, 16, 64, 16, "head_dim 64"),
    (32, 8, 96, 16, "head_dim 96"),
    (24, 8, 192, 16, "head_dim 192"),
    (16, 8, 256, 16, "head_dim 256"),
    (8, 8, 512, 16, "head_dim 512"),
    (80, 1, 128, 16, "one KV head: Llama-3-70B, one GPU's share of 8 under tensor parallelism"),
    (80, 2, 128, 16, "two KV heads: the same model's share of 4"),
    (64, 2, 64, 16, "two KV heads of 64"),
    (32, 8, 128, 1, "block size 1 (paging by the token)"),
    (32, 8, 128, 2, "block size 2"),
    (32, 8, 128, 8, "block size 8"),
    (32, 8, 128, 32, "block size 32"),
    (32, 8, 128, 128, "block size 128"),
)


def workload_sweep(args, dev):
    """The store and compose kernels over a range of model shapes and paged block sizes:
    4096 tokens stored and composed back as 8 shifted slices, per shape, stored form
    (--fmt) and RoPE pairing.  One row of config.rows per shape; `value` is the default
    shape's tokens/s over store + compose."""
    import torch
    from paper_2409_13761_amd import kdn, synth

    T, n_slices, n_sets = 4096, 8, 4
    fmt = FMT_IDS[args.fmt]
    offsets = [j * (T // n_slices) for j in range(n_slices)]
    rows, first = [], None

    def ev():
        return torch.cuda.Event(enable_timing=True)

    for (L, H, D, bs, note) in SWEEP_SHAPES:
        if args.fmt == "int4" and D % 32:
            continue
        blocks = T // bs
        nb = pool_blocks_for(args, blocks * 2 * n_sets, L * bs * H * D * 2)
        g = torch.Generator(device=dev)
        g.manual_seed(1002)
        k = torch.empty((L, nb, bs, H, D), device=dev, dtype=torch.bfloat16)
        v = torch.empty_like(k)
        fill_normal(k, g)
        fill_normal(v, g)
        cache = kdn.PagedCache(k, v)
        tabs = [torch.from_numpy(t).to(dev) for t in synth.disjoint_block_tables(1002, nb, [blocks] * (2 * n_sets))]
        chunks = [chunk_alloc(kdn, cache, T, fmt) for _ in range(n_sets)]
        kdn.kdn_rope_prepare(500000.0, D, offsets)
        per_tok = L * 2 * H * D * 2 + kdn.kdn_chunk_bytes(L, H, D, 1, fmt)
        row = {"L": L, "H": H, "D": D, "block_size": bs, "note": note, "bytes_per_call": T * per_tok}
        for pairing in ("half_split", "interleaved"):
            spec = kdn.rope_spec(500000.0, None, 0, kdn.ROPE_INTERLEAVED if pairing == "interleaved"
                                 else kdn.ROPE_HALF_SPLIT)

            def store(i):
                kdn.kdn_store_chunk(cache, tabs[2 * (i % n_sets)], 0, T, chunks[i % n_sets])

            def compose(i):
                s = (i + 2) % n_sets              # a chunk stored two steps ago, not the cached one
                views = [chunks[s].slice(j * (T // n_slices), T // n_slices) for j in range(n_slices)]
                kdn.kdn_compose_rope(views, offsets, cache, tabs[2 * s + 1], spec)

            for i in range(n_sets):
                store(i)
            for i in range(n_sets):
                compose(i)
            torch.cuda.synchronize()
            marks = []
            for i in range(args.steps):
                a_, b_, c_ = ev(), ev(), ev()
                a_.record()
                store(i)
                b_.record()
                compose(i)
                c_.record()
                marks.append((a_, b_, c_))
            torch.cuda.synchronize()
            ms_store = sum(x.elapsed_time(y) for x, y, _ in marks) / args.steps
            ms_comp = sum(y.elapsed_time(z) for _, y, z in marks) / args.steps
            row[pairing] = {"store_ms": ms_store, "store_GBps": T * per_tok / ms_store / 1e6,
                            "compose_ms": ms_comp, "compose_GBps": T * per_tok / ms_comp / 1e6}
        rows.append(row)
        if first is None:
            first = row
        del k, v, cache, chunks, tabs
        torch.cuda.empty_cache()
    ms = {"store": first["half_split"]["store_ms"], "compose": first["half_split"]["compose_ms"]}
    return {
        "tokens_per_step": T, "wall": (ms["store"] + ms["compose"]) * 1e-3 * args.steps, "ms": ms,
        "bytes": {n: first["bytes_per_call"] for n in ms},
        "place_calls": ("compose",),
        "workload": "sweep over KV shapes and paged block sizes, %s stored form: per shape 4096 tokens stored "
                    "and composed back as 8x512-token shifted slices (base 500000), half-split and interleaved "
                    "RoPE pairing; the headline fields are the first row's" % args.fmt,
        "extra": {"rows": rows},
        "traffic": None,
    }


def cpu_baseline(kdn, cache, buf_set, order, offsets, base, T, n_slices, steps):
    """The oracle as it stands, on the host cores: the same step (store, load, compose
    of one 4096-token context, all layers), layers split over threads; once more on one
    thread; and, untimed, a comparison of one coherent GPU pass (store -> load -> compose
    of this buffer set) with what the oracle computed from the same source blocks."""
    import numpy as np
    import torch
    from oracle import kdn_oracle as O

    L, nb, bs, H, D = cache.shape
    src, dst_a, dst_b, gpu_chunk, gpu_slices = buf_set
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
    slices = [chunk.slice(int(i) * (T // n_slices), T // n_slices) for i in order]

    def work(lr):
        O.store(host, t_src, 0, T, O.FMT_INT8_ROWSCALE, layers=lr, out=chunk)
        O.load(chunk, host, t_a, 0, layers=lr)
        O.compose(slices, offsets, host, t_b, base, layers=lr)

    def run(n_threads, n_steps):
        bounds = [(L * i // n_threads, L * (i + 1) // n_threads) for i in range(n_threads)]
        t0 = time.perf_counter()
        for _ in range(n_steps):
            th = [threading.Thread(target=work, args=(b,)) for b in bounds]
            for t in th:
                t.start()
            for t in th:
                t.join()
        return time.perf_counter() - t0

    dt = run(cores, steps)
    dt1 = run(1, 1)

    # one coherent pass of the HIP path on the same buffer set, compared with the oracle's result
    kdn.kdn_store_chunk(cache, src, 0, T, gpu_chunk)
    kdn.kdn_load_chunk(gpu_chunk, cache, dst_a, 0)
    kdn.kdn_compose(gpu_slices, offsets, cache, dst_b, base)
    torch.cuda.synchronize()

    def bits(t):
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)

    def f64(b):
        return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)

    parity = {"stored_chunk_equal": bool(np.array_equal(gpu_chunk.data.cpu().numpy(), chunk.data))}
    gk_a, gv_a = bits(cache.k[:, dst_a.long()]), bits(cache.v[:, dst_a.long()])
    gk_b, gv_b = bits(cache.k[:, dst_b.long()]), bits(cache.v[:, dst_b.long()])
    parity["load_equal"] = bool(np.array_equal(gk_a, hk[:, blocks:2 * blocks])
                                and np.array_equal(gv_a, hv[:, blocks:2 * blocks]))
    parity["compose_v_equal"] = bool(np.array_equal(gv_b, hv[:, 2 * blocks:]))
    want_k = hk[:, 2 * blocks:]
    parity["compose_k_differing_elements"] = int(np.count_nonzero(gk_b != want_k))
    parity["compose_k_max_abs_diff"] = float(np.max(np.abs(f64(gk_b) - f64(want_k))))
    return {"value": T * steps / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "%d full steps of the same workload (store+load+compose of 4096 tokens, "
                      "all %d layers), layers split over %d threads" % (steps, L, cores),
            "seconds": dt, "single_thread_value": T / dt1,
            "parity_of_one_gpu_pass": parity}


def cpu_baseline_70b(kdn, cache, buf_set, offsets, base, T, n_layers):
    """The oracle as it stands on the host cores, on a bounded sample of the same step: store
    and compose of all 32768 tokens for n_layers of the 80 layers (evenly spaced), one layer
    per task over the host threads; and, untimed, one coherent GPU pass (store -> compose of
    this buffer set) compared with what the oracle computed for those layers from the same
    source blocks."""
    import numpy as np
    import torch
    from oracle import kdn_oracle as O

    L, nb, bs, H, D = cache.shape
    src, dst, gpu_chunk, gpu_slices = buf_set
    blocks = T // bs
    layers = [int(x) for x in np.linspace(0, L - 1, n_layers).round()]
    Ls = len(layers)
    hk = np.zeros((Ls, 2 * blocks, bs, H, D), dtype=np.uint16)      # source blocks, then zeroed destination blocks
    hv = np.zeros_like(hk)
    for i, l in enumerate(layers):
        hk[i, :blocks] = cache.k[l, src.long()].view(torch.int16).cpu().numpy().view(np.uint16)
        hv[i, :blocks] = cache.v[l, src.long()].view(torch.int16).cpu().numpy().view(np.uint16)
    host = O.PagedCache(hk, hv)
    t_src = np.arange(0, blocks, dtype=np.int32)
    t_dst = np.arange(blocks, 2 * blocks, dtype=np.int32)
    chunk = O.Chunk(np.zeros(O.chunk_bytes(Ls, H, D, T, O.FMT_INT8_ROWSCALE), dtype=np.uint8),
                    O.FMT_INT8_ROWSCALE, Ls, H, D, T)
    slices = [chunk.slice(i * (T // 4), T // 4) for i in range(4)]
    cores = max(1, min(len(os.sched_getaffinity(0)), 16, Ls))

    def work(i):
        O.store(host, t_src, 0, T, O.FMT_INT8_ROWSCALE, layers=(i, i + 1), out=chunk)
        O.compose(slices, offsets, host, t_dst, base, layers=(i, i + 1))

    from concurrent.futures import ThreadPoolExecutor
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        list(ex.map(work, range(Ls)))
    dt = time.perf_counter() - t0
    t0 = time.perf_counter()
    work(0)                                                          # one layer again, alone on one thread
    dt1 = time.perf_counter() - t0

    kdn.kdn_store_chunk(cache, src, 0, T, gpu_chunk)
    kdn.kdn_compose(gpu_slices, offsets, cache, dst, base)
    torch.cuda.synchronize()

    def bits(t):
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)

    def f64(b):
        return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)

    gc, gs = gpu_chunk.codes(), gpu_chunk.scales()
    parity = {"layers_compared": layers, "stored_chunk_equal": True, "compose_v_equal": True,
              "compose_k_differing_elements": 0, "compose_k_max_abs_diff": 0.0}
    for i, l in enumerate(layers):
        parity["stored_chunk_equal"] &= bool(np.array_equal(gc[l].cpu().numpy(), chunk.codes()[i])
                                             and np.array_equal(gs[l].cpu().numpy(), chunk.scales()[i]))
        gk, gv = bits(cache.k[l, dst.long()]), bits(cache.v[l, dst.long()])
        parity["compose_v_equal"] &= bool(np.array_equal(gv, hv[i, blocks:]))
        want_k = hk[i, blocks:]
        parity["compose_k_differing_elements"] += int(np.count_nonzero(gk != want_k))
        parity["compose_k_max_abs_diff"] = max(parity["compose_k_max_abs_diff"],
                                               float(np.max(np.abs(f64(gk) - f64(want_k)))))
    return {"value": T / (dt * L / Ls), "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "store + compose of all %d tokens for %d of the %d layers (layers %s), one layer per task on "
                      "%d threads, %.2f s; value = tokens / (that time x %d/%d), i.e. the whole step at this rate"
                      % (T, Ls, L, layers, cores, dt, L, Ls),
            "seconds": dt, "single_thread_value": T / (dt1 * L),
            "parity_of_one_gpu_pass": parity}


def summarise(res, steps, warmup, fmt_note):
    """The JSON fields of one workload's result."""
    ms, nbytes = res["ms"], res["bytes"]
    gbps = {n: nbytes[n] / (ms[n] * 1e-3) / 1e9 for n in ms}
    place = res["place_calls"]
    place_ms = sum(ms[n] for n in place) / len(place)
    achieved = nbytes[place[0]] / (place_ms * 1e-3) / 1e9
    out = {
        "value": res["tokens_per_step"] * steps / res["wall"],
        "unit": "tokens/s",
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": res["wall"] / steps * 1e3,
        "dtype": fmt_note,
        "config": {
            "workload": res["workload"],
            "tokens_per_step": res["tokens_per_step"],
            "algorithmic_bytes_per_call": nbytes,
            "calls_per_step": len(ms),
        },
        "breakdown": {n: {"ms": ms[n], "GBps": gbps[n], "frac_of_peak": gbps[n] / HBM_PEAK_GBPS} for n in ms},
        "roofline": {
            "bound": "hbm",
            "kernel": "k_place (%s launches)" % " and ".join(place),
            "achieved": achieved,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": res["traffic"],
        },
    }
    if "extra" in res:
        out["config"].update(res["extra"])
    if "cpu_baseline" in res:
        out["cpu_baseline"] = res["cpu_baseline"]
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", choices=("70b_long", "8b", "toy", "batched_reuse", "host_stream_int8",
                             "host_stream_raw", "pool_trace", "pool_trace_tiered", "sweep", "stream_probe"),
                    default="70b_long")
    ap.add_argument("--only", action="store_true",
                    help="the named workload alone: the default run's shorter 8b and batched_reuse passes, the "
                         "streaming yardstick and the plain-memory comparison are left out (for profiling)")
    ap.add_argument("--fmt", choices=("int8", "int4", "fp8", "raw"), default="int8",
                    help="stored form used by the 8b and 70b_long workloads")
    ap.add_argument("--layout", choices=("planes", "kv_pair", "block_major"), default="planes",
                    help="paged cache layout of the 8b workload, all expressed through the "
                         "descriptor's strides: separate K and V tensors [L][blocks][bs][H][D] "
                         "(default), K and V of a block adjoining, or all layers of a block adjoining")
    ap.add_argument("--tables", choices=("random", "consecutive"), default="random",
                    help="block tables of the 8b workload: sampled without replacement from the pool "
                         "(default, the stated workload) or runs of consecutive blocks")
    ap.add_argument("--pool-gib", type=float, default=POOL_GIB_DEFAULT,
                    help="size in GiB of each of the paged pool's K and V tensors (8b, 70b_long, batched_reuse): an "
                         "engine gives most of HBM to its KV pool, and the block tables are drawn from all of it; 0 "
                         "makes the pool only as large as the tables the step uses")
    ap.add_argument("--pool-blocks", type=int, default=0,
                    help="blocks per (layer, side) plane of the paged pool, instead of --pool-gib")
    ap.add_argument("--chunk-memory", choices=("arena", "plain"), default="arena",
                    help="where the stored chunks lie: in the library's arena, whose neighbouring 16 MiB granules "
                         "lie far apart in the device memory (created first, before the pool), or in plain torch "
                         "allocations")
    ap.add_argument("--arena-gib", type=float, default=24.0, help="size of the arena")
    ap.add_argument("--pool-memory", choices=("torch", "arena"), default="torch",
                    help="where the paged pool of the 8b and 70b_long workloads lies: a torch allocation (the engine's "
                         "own memory, the default) or the arena (give --arena-gib room for it): a pool much smaller "
                         "than the device memory then still has its blocks spread over all of it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=8, help="oracle steps of the 8b workload's CPU baseline")
    ap.add_argument("--cpu-layers", type=int, default=20,
                    help="layers (of 80) the 70b_long workload's CPU baseline runs the oracle on")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, a dispatch of known size for "
                         "scaling hardware byte counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on one GPU only; the path shards without any exchange "
              "(by KV head, layer or request), so --gpus N > 1 is not measured", file=sys.stderr)
        return 2
    from paper_2409_13761_amd import build as lib_build
    lib_build.ensure_built()
    defaults_of = {"8b": (40, 8), "toy": (200, 20), "70b_long": (12, 3), "batched_reuse": (10, 3),
                   "host_stream_int8": (10, 3), "host_stream_raw": (10, 3), "pool_trace": (400, 100),
                   "pool_trace_tiered": (400, 100), "sweep": (8, 0), "stream_probe": (12, 0)}
    defaults = defaults_of[args.workload]
    args.steps = defaults[0] if args.steps is None else args.steps
    args.warmup = defaults[1] if args.warmup is None else args.warmup

    import torch
    from paper_2409_13761_amd import kdn

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        return 3
    kdn.lib()                                   # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    runners = {"8b": workload_8b, "toy": workload_toy, "70b_long": workload_70b, "batched_reuse": workload_batched,
               "host_stream_int8": lambda a, d: workload_host_stream(a, d, "int8"),
               "host_stream_raw": lambda a, d: workload_host_stream(a, d, "raw"),
               "pool_trace": workload_pool_trace, "pool_trace_tiered": workload_pool_trace_tiered,
               "sweep": workload_sweep, "stream_probe": workload_stream_probe}

    def fmt_note(workload):
        f = ("int8" if workload in ("batched_reuse", "host_stream_int8", "pool_trace", "pool_trace_tiered")
             else "raw" if workload == "host_stream_raw" else args.fmt)
        return "bf16 KV, %s stored form, fp32 arithmetic" % {
            "int8": "int8 codes + fp32 row scales", "int4": "int4 codes + fp32 group scales",
            "fp8": "fp8 e4m3 codes + fp32 row scales", "raw": "raw bf16"}[f]

    global ARENA
    arena_error = None
    if args.chunk_memory == "arena" and args.workload not in ("stream_probe", "toy", "host_stream_int8",
                                                              "host_stream_raw"):
        torch.zeros(1, device=dev)
        try:
            ARENA = kdn.kdn_arena_create(int(args.arena_gib * (1 << 30)))
        except kdn.KdnError as e:            # too little free memory, say: the chunks then lie in plain allocations
            print("bench.py: no arena (%s); stored chunks in plain device memory" % e, file=sys.stderr)
            arena_error = str(e)

    res = runners[args.workload](args, dev)

    if args.calibration_copy:
        a = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                              # 1 GiB read, 1 GiB written
        torch.cuda.synchronize()
        del a, b

    body = summarise(res, args.steps, args.warmup, fmt_note(args.workload))
    out = {
        "metric": METRIC,
        "value": body.pop("value"),
        "unit": body.pop("unit"),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": body.pop("ms_per_step"),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": body.pop("dtype"),
        "data": "synthetic N(0,1) bf16 KV, seeded; %s block tables"
                % ("consecutive-block" if args.workload == "8b" and args.tables == "consecutive" else "random disjoint"),
    }
    body.pop("steps")
    body.pop("warmup")
    out.update(body)
    out["library"] = kdn.kdn_version()
    if ARENA is not None:
        out["arena"] = dict(ARENA, what="stored chunks lie in kdn_arena memory: granule i is free granule (i * stride) "
                                        "mod free_granules of the device memory in the driver's order; striped_gbs / "
                                        "packed_gbs: scattered tile writes over 1 GiB of it / of memory in that order")
    elif arena_error is not None:
        out["arena"] = {"error": arena_error, "what": "kdn_arena_create failed: stored chunks lie in plain device memory"}
    if out["roofline"]["traffic"] is not None:
        out["roofline"]["traffic_from"] = COUNTER_TRAFFIC[args.workload]["profile"]
    del res
    gc.collect()                                # chunk buffers go back to the arena, pools to torch
    torch.cuda.empty_cache()

    if args.workload in ("70b_long", "8b") and not args.only:
        ceiling = stream_ceiling(dev, args.pool_gib if not args.pool_blocks else 8)
        torch.cuda.empty_cache()
        # load and compose write through random block tables and store reads through one, so the
        # scattered figures are their yardsticks
        ceiling["frac_of_ceiling"] = {
            n: v["GBps"] / ceiling["store_pattern_scattered_GBps" if n == "store" else "place_pattern_scattered_GBps"]
            for n, v in out["breakdown"].items()}
        ceiling["k_place_frac_of_contiguous_ceiling"] = out["roofline"]["achieved"] / ceiling["place_pattern_contiguous_GBps"]
        out["stream_ceiling"] = ceiling
    if args.workload == "70b_long" and not args.only:
        import copy
        others = {}
        for name in ("8b", "batched_reuse"):
            a2 = copy.copy(args)
            a2.workload, a2.no_cpu_baseline = name, True
            a2.steps, a2.warmup = defaults_of[name]
            r2 = runners[name](a2, dev)
            others[name] = summarise(r2, a2.steps, a2.warmup, fmt_note(name))
            if others[name]["roofline"]["traffic"] is not None:
                others[name]["roofline"]["traffic_from"] = COUNTER_TRAFFIC[name]["profile"]
            del r2
            gc.collect()
            torch.cuda.empty_cache()
        out["other_workloads"] = others
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
