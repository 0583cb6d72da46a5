"""Seeded random parity sweep: shapes, block sizes, formats, ragged token ranges, chunk
views, RoPE variants and patches drawn at random, every result compared with the oracle
bit for bit.  Complements the hand-picked cases of test_gpu_parity.py."""
import numpy as np
import pytest
import torch

from helpers import (FP8, INT4, INT8, RAW, assert_cache_equal, assert_chunk_equal, chunk_to_dev,
                     dev_cache, dev_table, host_cache, to_dev_bf16)
from oracle import kdn_oracle as O
from paper_2409_13761_amd import kdn, synth

pytestmark = pytest.mark.gpu

DIMS = (16, 32, 48, 64, 80, 96, 128, 192, 256)
BLOCKS = (1, 2, 4, 8, 16, 24, 32, 48)


def _case(seed):
    rng = np.random.default_rng(seed)
    L, H = int(rng.integers(1, 4)), int(rng.integers(1, 6))
    D, bs = int(rng.choice(DIMS)), int(rng.choice(BLOCKS))
    fmts = [f for f in (RAW, INT8, INT4, FP8) if f != INT4 or D % 32 == 0]
    tokens_cap = int(rng.integers(40, 200))
    n_tab = (tokens_cap + bs - 1) // bs
    nb = 3 * n_tab + 5
    return rng, L, H, D, bs, fmts, n_tab, nb


@pytest.mark.parametrize("seed", range(40))
def test_random_store_compose_patch(seed):
    rng, L, H, D, bs, fmts, n_tab, nb = _case(1000 + seed)
    cap = n_tab * bs
    print("[case] seed=%d L=%d H=%d D=%d bs=%d cap=%d" % (seed, L, H, D, bs, cap), flush=True)
    src = host_cache(2000 + seed, L, nb, bs, H, D)
    t_a, t_b, dst_bt = synth.disjoint_block_tables(seed, nb, [n_tab, n_tab, n_tab])
    dsrc = dev_cache(src)

    # two stored chunks of random ranges and formats, checked as stored
    hch, dch = [], []
    for tab in (t_a, t_b):
        fmt = int(rng.choice(fmts))
        t0 = int(rng.integers(0, cap // 2))
        T = int(rng.integers(1, cap - t0 + 1))
        h = O.store(src, tab, t0, T, fmt)
        out = kdn.alloc_chunk(dsrc, T, fmt)
        kdn.kdn_store_chunk(dsrc, dev_table(tab), t0, T, out)
        assert_chunk_equal(out, h)
        hch.append(h)
        dch.append(out)

    # random views of them, composed with a random RoPE variant into a third table
    views_h, views_d, offsets, total = [], [], [], 0
    dest = int(rng.integers(0, bs + 1))
    for _ in range(int(rng.integers(1, 6))):
        i = int(rng.integers(0, 2))
        ts = int(rng.integers(0, hch[i].T))
        Tv = int(rng.integers(1, hch[i].T - ts + 1))
        if dest + total + Tv > cap:
            break
        views_h.append(hch[i].slice(ts, Tv))
        views_d.append(dch[i].slice(ts, Tv))
        offsets.append(int(rng.integers(-5000, 5000)) if rng.random() < 0.8 else 0)
        total += Tv
    if not views_h:
        views_h, views_d, offsets = [hch[0].slice(0, 1)], [dch[0].slice(0, 1)], [3]
        dest, total = 0, 1
    rot = int(rng.choice([0] + [r for r in range(16, D + 1, 16)]))
    pairing = int(rng.integers(0, 2))
    base = float(rng.choice([10000.0, 500000.0]))
    inv_freq = None
    if rng.random() < 0.3:
        r = rot or D
        inv_freq = base ** (-2.0 * np.arange(r // 2) / r) * rng.uniform(0.1, 1.0, size=r // 2)
    hd = host_cache(3000 + seed, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.compose_spec(views_h, offsets, hd, dst_bt, base, inv_freq=inv_freq, rot_dim=rot, pairing=pairing, dest=dest)
    kdn.kdn_compose_rope(views_d, offsets, dd, dev_table(dst_bt), kdn.rope_spec(base, inv_freq, rot, pairing),
                         dest_token_start=dest)
    assert_cache_equal(dd, hd)

    # a kept-token store from the composed request, and a patch over a few of its tokens
    n_keep = int(rng.integers(1, dest + total + 1))
    keep = np.sort(rng.choice(dest + total, size=n_keep, replace=False)).astype(np.int32)
    fmt = int(rng.choice(fmts))
    want = O.store_tokens(hd, dst_bt, keep, fmt)
    out = kdn.alloc_chunk(dd, n_keep, fmt)
    kdn.kdn_store_tokens(dd, dev_table(dst_bt), torch.from_numpy(keep).cuda(), out)
    assert_chunk_equal(out, want)
    n_patch = int(rng.integers(1, min(8, cap) + 1))
    tok = rng.choice(cap, size=n_patch, replace=False).astype(np.int32)
    rows = synth.normal_bf16(4000 + seed, (L, 2, n_patch, H, D))
    O.patch_rows(rows, tok, hd, dst_bt)
    kdn.kdn_patch_rows(to_dev_bf16(rows), torch.from_numpy(tok).cuda(), dd, dev_table(dst_bt))
    assert_cache_equal(dd, hd)


@pytest.mark.parametrize("seed", range(16))
def test_random_host_paths(seed):
    """Random shapes, formats, views and stage depths through the host-memory paths: the staged
    store, the staged compose and the kernels addressing pinned host chunks directly."""
    rng, L, H, D, bs, fmts, n_tab, nb = _case(5000 + seed)
    cap = n_tab * bs
    lps = int(rng.integers(1, L + 2))
    print("[case] host seed=%d L=%d H=%d D=%d bs=%d cap=%d lps=%d" % (seed, L, H, D, bs, cap, lps), flush=True)
    src = host_cache(6000 + seed, L, nb, bs, H, D)
    t_a, t_b, dst_bt = synth.disjoint_block_tables(seed, nb, [n_tab, n_tab, n_tab])
    dsrc = dev_cache(src)
    hch, pch = [], []                       # oracle chunks, pinned host chunks written by the library
    for n, tab in enumerate((t_a, t_b)):
        fmt = int(rng.choice(fmts))
        t0 = int(rng.integers(0, cap // 2))
        T = int(rng.integers(1, cap - t0 + 1))
        h = O.store(src, tab, t0, T, fmt)
        out = kdn.alloc_host_chunk(dsrc, T, fmt)
        out.data.fill_(0x5C)
        if n == 0:                          # staged through HBM by the copy engine
            staging = torch.empty(kdn.kdn_store_staging_bytes(dsrc, T, fmt, lps), dtype=torch.uint8, device="cuda")
            kdn.kdn_store_to_host(dsrc, dev_table(tab), t0, T, out, staging, lps)
        else:                               # written across the link by the kernel itself
            kdn.kdn_store_chunk(dsrc, dev_table(tab), t0, T, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.data.numpy(), h.data)
        hch.append(h)
        pch.append(out)
    views_h, views_p, offsets, total = [], [], [], 0
    dest = int(rng.integers(0, bs + 1))
    for _ in range(int(rng.integers(1, 6))):
        i = int(rng.integers(0, 2))
        ts = int(rng.integers(0, hch[i].T))
        Tv = int(rng.integers(1, hch[i].T - ts + 1))
        if dest + total + Tv > cap:
            break
        views_h.append(hch[i].slice(ts, Tv))
        views_p.append(pch[i].slice(ts, Tv))
        offsets.append(int(rng.integers(-5000, 5000)) if rng.random() < 0.8 else 0)
        total += Tv
    if not views_h:
        views_h, views_p, offsets = [hch[0].slice(0, 1)], [pch[0].slice(0, 1)], [3]
        dest = 0
    hd = host_cache(7000 + seed, L, nb, bs, H, D)
    O.compose(views_h, offsets, hd, dst_bt, 10000.0, dest=dest)
    d1, d2 = dev_cache(host_cache(7000 + seed, L, nb, bs, H, D)), dev_cache(host_cache(7000 + seed, L, nb, bs, H, D))
    st = torch.empty(kdn.kdn_staging_bytes(views_p, lps), dtype=torch.uint8, device="cuda")
    kdn.kdn_compose_from_host(views_p, offsets, d1, dev_table(dst_bt), 10000.0, st, lps, dest_token_start=dest)
    kdn.kdn_compose(views_p, offsets, d2, dev_table(dst_bt), 10000.0, dest_token_start=dest)
    assert_cache_equal(d1, hd)
    assert_cache_equal(d2, hd)


@pytest.mark.parametrize("seed", range(24))
def test_random_batches_with_repeated_views(seed):
    """Batched composes in which views recur: the same slice of the same chunk in several
    requests (and twice in one), at destinations that sometimes share the tile grid and
    sometimes do not, with their own offsets.  Whatever the planner chains, every request's
    table must hold what a compose of its own gives; the static entry point must agree too."""
    rng, L, H, D, bs, fmts, n_tab, nb0 = _case(9000 + seed)
    n_req = int(rng.integers(2, 7))
    probe = torch.zeros((L, 2, bs, H, D), dtype=torch.bfloat16)
    G = kdn.kdn_tile_tokens(kdn.PagedCache(probe, torch.zeros_like(probe)))
    cap = n_tab * bs
    req_blocks = -(-(3 * cap + 2 * G) // bs)
    nb = 2 * n_tab + n_req * req_blocks + 3
    print("[case] repeats seed=%d L=%d H=%d D=%d bs=%d cap=%d tile=%d requests=%d" % (seed, L, H, D, bs, cap, G, n_req),
          flush=True)
    src = host_cache(9100 + seed, L, nb, bs, H, D)
    tabs = synth.disjoint_block_tables(seed, nb, [n_tab, n_tab] + [req_blocks] * n_req)
    fmt = int(rng.choice(fmts))                                     # one stored form: one launch, chains possible
    hch = [O.store(src, tabs[i], 0, cap, fmt) for i in range(2)]
    dch = [chunk_to_dev(h) for h in hch]
    seen = []                                                       # (chunk, start, length) of earlier views
    hd = host_cache(9200 + seed, L, nb, bs, H, D)
    dd = dev_cache(hd)
    reqs = []
    for r in range(n_req):
        views, offs = [], []
        dest = int(rng.choice([0, G, 2 * G, int(rng.integers(0, bs + 1))]))
        room = req_blocks * bs - dest
        for _ in range(int(rng.integers(1, 4))):
            if seen and rng.random() < 0.6:
                i, ts, Tv = seen[int(rng.integers(0, len(seen)))]
            else:
                i = int(rng.integers(0, 2))
                ts = int(rng.integers(0, cap))
                Tv = int(rng.integers(1, cap - ts + 1))
            if Tv > room:
                break
            room -= Tv
            seen.append((i, ts, Tv))
            views.append((i, ts, Tv))
            offs.append(int(rng.integers(-3000, 3000)) if rng.random() < 0.8 else 0)
        if not views:
            views, offs = [(0, 0, 1)], [5]
        O.compose([hch[i].slice(ts, Tv) for i, ts, Tv in views], offs, hd, tabs[2 + r], 10000.0, dest=dest)
        reqs.append(([dch[i].slice(ts, Tv) for i, ts, Tv in views], offs, dev_table(tabs[2 + r]), dest))
    plan = kdn.kdn_compose_plan(reqs, dd)
    print("[case] repeats seed=%d: %d views, %d of them chained behind another" %
          (seed, len(plan), sum(p["follows"] >= 0 for p in plan)), flush=True)
    kdn.kdn_compose_batch(reqs, dd, 10000.0)
    assert_cache_equal(dd, hd)
    d2 = dev_cache(host_cache(9200 + seed, L, nb, bs, H, D))
    kdn.kdn_compose_batch_static(reqs, d2, 10000.0)
    assert_cache_equal(d2, hd)
