"""Host logic of the compose from host memory (the delivery module's path from storage to
the GPU, Sec. 3.1), checked without a GPU: the link transfers that kdn_host_stage_plan
reports are carried out with numpy on host buffers, and the staged images must be the
stored chunks of the stage's layers and the spanned token range, in every stored form."""
import numpy as np
import pytest
import torch

from helpers import FP8, INT4, INT8, RAW, host_cache
from oracle import kdn_oracle as O
from paper_2409_13761_amd import kdn, synth

L, NB, BS, H, D = 5, 64, 16, 2, 64


def _binding_chunk(h: O.Chunk) -> kdn.Chunk:
    c = kdn.chunk_from_buffer(torch.from_numpy(h.data), h.fmt, h.L, h.H, h.D, h.Tp)
    return c if (h.tok_start == 0 and h.T == h.Tp) else c.slice(h.tok_start, h.T)


def _views():
    src = host_cache(71, L, NB, BS, H, D)
    t1, t2, t3, t4 = synth.disjoint_block_tables(71, NB, [6, 5, 4, 4])
    a = O.store(src, t1, 0, 90, INT8)
    b = O.store(src, t2, 3, 70, RAW)
    c = O.store(src, t3, 0, 64, INT4)
    d = O.store(src, t4, 1, 50, FP8)
    return [a.slice(10, 75), b, c, a.slice(0, 10), b.slice(20, 31), d.slice(5, 40), c.slice(33, 20)]


def _typed(ch: O.Chunk):
    """(codes, scales) arrays indexed [layer][side][token]…"""
    if ch.fmt == RAW:
        return ch.raw(), None
    if ch.fmt == INT4:
        return ch.packed4(), ch.scales4()
    return ch.codes(), ch.scales()


@pytest.mark.parametrize("lps", [1, 2, 5, 8])
def test_staged_images_are_the_stored_rows(lps):
    views = _views()
    bviews = [_binding_chunk(v) for v in views]
    need = kdn.kdn_staging_bytes(bviews, lps)
    half = need // 2
    # token range spanned by the views of each host buffer
    span = {}
    for v in views:
        lo, hi = span.get(id(v.data), (v.tok_start, v.tok_start + v.T))
        span[id(v.data)] = (min(lo, v.tok_start), max(hi, v.tok_start + v.T))
    n_stages = -(-L // lps)
    for stage in range(n_stages):
        l0, lg = stage * lps, min(lps, L - stage * lps)
        copies, view_off = kdn.kdn_host_stage_plan(bviews, lps, stage)
        staging = np.full(half, 0xA5, dtype=np.uint8)
        written = np.zeros(half, dtype=bool)
        for c in copies:
            srcbuf = views[c["chunk"]].data
            for r in range(c["rows"]):
                s = c["src_offset"] + r * c["src_pitch"]
                t = c["dst_offset"] + r * c["width"]
                assert s + c["width"] <= srcbuf.nbytes and t + c["width"] <= half
                assert not written[t:t + c["width"]].any()          # no two copies overlap
                staging[t:t + c["width"]] = srcbuf[s:s + c["width"]]
                written[t:t + c["width"]] = True
        for v, off in zip(views, view_off):
            lo, hi = span[id(v.data)]
            n = O.chunk_bytes(lg, H, D, hi - lo, v.fmt)
            assert off % 256 == 0 and written[off:off + n].all()
            image = O.Chunk(np.ascontiguousarray(staging[off:off + n]), v.fmt, lg, H, D, hi - lo)
            got_c, got_s = _typed(image)
            want_c, want_s = _typed(O.Chunk(v.data, v.fmt, L, H, D, v.Tp))
            assert np.array_equal(got_c, want_c[l0:l0 + lg, :, lo:hi])
            if want_s is not None:
                assert np.array_equal(got_s.view(np.uint32), want_s[l0:l0 + lg, :, lo:hi].view(np.uint32))
    with pytest.raises(kdn.KdnError) as e:
        kdn.kdn_host_stage_plan(bviews, lps, n_stages)
    assert e.value.status == kdn.ERANGE


def test_link_bytes_are_the_compact_rows_once_per_host_buffer():
    views = _views()
    bviews = [_binding_chunk(v) for v in views]
    moved = sum(c["rows"] * c["width"] for s in range(L) for c in kdn.kdn_host_stage_plan(bviews, 1, s)[0])
    # a: tokens 0..84 of 90, b: 0..69, c: 0..63, d: 5..44
    want = (O.chunk_bytes(L, H, D, 85, INT8) + O.chunk_bytes(L, H, D, 70, RAW)
            + O.chunk_bytes(L, H, D, 64, INT4) + O.chunk_bytes(L, H, D, 40, FP8))
    assert moved == want


def test_plan_refuses_a_chunk_whose_bytes_do_not_cover_its_layout():
    v = _views()[2]
    good = _binding_chunk(v)
    short = kdn.Chunk(good.data, kdn.ChunkDesc.from_buffer_copy(good.desc))
    short.desc.bytes -= 1
    with pytest.raises(kdn.KdnError) as e:
        kdn.kdn_host_stage_plan([short], 2, 0)
    assert e.value.status == kdn.ESIZE


@pytest.mark.parametrize("seed", range(24))
def test_random_plans_stage_the_stored_rows(seed):
    """Random shapes, forms, views and stage depths: carrying the planned copies out always
    yields, per view, the stored chunk of the stage's layers over the spanned tokens."""
    rng = np.random.default_rng(900 + seed)
    l_, h_ = int(rng.integers(1, 7)), int(rng.integers(1, 5))
    d_ = int(rng.choice([16, 32, 64, 96, 128, 256]))
    lps = int(rng.integers(1, l_ + 2))
    parents = []
    for _ in range(int(rng.integers(1, 4))):
        fmt = int(rng.choice([f for f in (RAW, INT8, INT4, FP8) if f != INT4 or d_ % 32 == 0]))
        tp = int(rng.integers(1, 70))
        data = rng.integers(0, 256, size=O.chunk_bytes(l_, h_, d_, tp, fmt), dtype=np.uint8)
        parents.append(O.Chunk(data, fmt, l_, h_, d_, tp))
    views = []
    for _ in range(int(rng.integers(1, 7))):
        p = parents[int(rng.integers(0, len(parents)))]
        ts = int(rng.integers(0, p.Tp))
        views.append(p.slice(ts, int(rng.integers(1, p.Tp - ts + 1))))
    bviews = [_binding_chunk(v) for v in views]
    half = kdn.kdn_staging_bytes(bviews, lps) // 2
    span = {}
    for v in views:
        lo, hi = span.get(id(v.data), (v.tok_start, v.tok_start + v.T))
        span[id(v.data)] = (min(lo, v.tok_start), max(hi, v.tok_start + v.T))
    for stage in range(-(-l_ // lps)):
        l0, lg = stage * lps, min(lps, l_ - stage * lps)
        copies, view_off = kdn.kdn_host_stage_plan(bviews, lps, stage)
        staging = np.zeros(half, dtype=np.uint8)
        for c in copies:
            srcbuf = views[c["chunk"]].data
            for r in range(c["rows"]):
                s, t = c["src_offset"] + r * c["src_pitch"], c["dst_offset"] + r * c["width"]
                assert s + c["width"] <= srcbuf.nbytes and t + c["width"] <= half
                staging[t:t + c["width"]] = srcbuf[s:s + c["width"]]
        for v, off in zip(views, view_off):
            lo, hi = span[id(v.data)]
            n = O.chunk_bytes(lg, h_, d_, hi - lo, v.fmt)
            image = O.Chunk(np.ascontiguousarray(staging[off:off + n]), v.fmt, lg, h_, d_, hi - lo)
            got_c, got_s = _typed(image)
            want_c, want_s = _typed(O.Chunk(v.data, v.fmt, l_, h_, d_, v.Tp))
            assert np.array_equal(got_c, want_c[l0:l0 + lg, :, lo:hi])
            if want_s is not None:
                assert np.array_equal(got_s.view(np.uint32), want_s[l0:l0 + lg, :, lo:hi].view(np.uint32))
