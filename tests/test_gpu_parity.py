"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element, on the same seeded inputs.  Sizes span several tiles and ragged tails.

Bars: stored codes, scales, raw copies, placement and all V outputs bit-exact;
RoPE-shifted K within 1e-2 absolute for N(0,1) inputs (and, as the design
target, without a differing bit)."""
import numpy as np
import pytest
import torch

from helpers import (FP8, INT4, INT8, RAW, assert_cache_equal, assert_chunk_equal, bits_of, chunk_to_dev,
                     dev_cache, dev_table, host_cache, to_dev_bf16)
from oracle import kdn_oracle as O
from paper_2409_13761_amd import kdn, synth

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)


# ------------------------------------------------------------------ store
@pytest.mark.parametrize("fmt", [RAW, INT8, INT4, FP8])
@pytest.mark.parametrize("shape", [
    # L, nb, bs, H, D, t0, T
    (2, 24, 16, 4, 64, 0, 128),        # block aligned, several tiles
    (2, 24, 16, 4, 64, 5, 150),        # starts and ends inside a block
    (3, 40, 16, 8, 128, 17, 301),      # 8B-like rows, ragged
    (1, 64, 1, 2, 128, 3, 50),         # block of one token
    (2, 12, 32, 2, 64, 9, 300),        # block larger than the token group
    (2, 12, 24, 3, 32, 7, 200),        # block size not a multiple of 16
    (1, 20, 16, 1, 16, 0, 97),         # smallest head_dim
    (1, 20, 8, 2, 96, 3, 100),         # head_dim whose lane group is padded
    (1, 10, 16, 2, 256, 1, 77),
    (1, 6, 16, 1, 512, 0, 40),         # largest head_dim
    (2, 30, 3, 2, 64, 4, 70),          # blocks of 3 tokens: rows look their own block up
    (2, 64, 2, 3, 128, 1, 90),         # blocks of 2 tokens
    (3, 40, 16, 1, 128, 5, 300),       # one head: small tiles, workgroups of one wavefront
    (2, 12, 128, 1, 128, 9, 700),      # one head, large blocks
    (2, 40, 16, 2, 64, 3, 333),        # two short heads
])
def test_store_matches_oracle(fmt, shape):
    L, nb, bs, H, D, t0, T = shape
    if fmt == INT4 and D % 32:
        pytest.skip("int4 groups need head_dim % 32 == 0")
    _say("store fmt=%d shape=%s" % (fmt, shape))
    hc = host_cache(100 + D + bs, L, nb, bs, H, D)
    n_tab = (t0 + T + bs - 1) // bs
    bt = synth.disjoint_block_tables(3, nb, [n_tab])[0]
    want = O.store(hc, bt, t0, T, fmt)
    dc = dev_cache(hc)
    out = kdn.alloc_chunk(dc, T, fmt)
    out.data.fill_(0xAB)
    kdn.kdn_store_chunk(dc, dev_table(bt), t0, T, out)
    assert_chunk_equal(out, want)
    assert (out.desc.parent_tokens, out.desc.token_start, out.desc.num_tokens) == (T, 0, T)


def test_store_special_rows():
    """Zero rows, -0, rows under the 2^-121 threshold, fp32-denormal scales, huge rows,
    exact ties; and every positive finite bf16 as a row's amax."""
    L, nb, bs, H, D = 1, 2100, 16, 1, 16
    k = np.zeros((L, nb, bs, H, D), dtype=np.uint16)
    rows = k.reshape(-1, D)
    # every positive finite bf16 once as amax, with companions at fixed ratios
    amax_bits = np.arange(1, 0x7F80, dtype=np.uint16)
    n = amax_bits.size
    rows[:n, 0] = amax_bits
    f = (amax_bits.astype(np.uint32) << 16).view(np.float32)
    for j, ratio in enumerate((0.5, -0.25, 0.75, -0.999, 0.0039, 0.3333, -0.0117), start=1):
        rows[:n, j] = bits_of(torch.from_numpy((f * np.float32(ratio)).astype(np.float32)).to(torch.bfloat16))
    rows[n, 3] = 0x8000                                   # row of zeros with one -0
    rows[n + 1, :] = 0x02FF                               # under the threshold everywhere
    rows[n + 2, :4] = [0x0300, 0x8300, 0x0280, 0x0001]    # exactly 2^-121
    ties = torch.tensor([127.0, 63.5, -63.5, 0.5, -0.5, 1.5, 2.5, -2.5, 126.5, -126.5, 3.5, 0, 0, 0, 0, 0])
    rows[n + 3] = bits_of(ties.to(torch.bfloat16))
    v = synth.normal_bf16(5, k.shape)
    hc = O.PagedCache(k, v)
    T = nb * bs
    bt = np.arange(nb, dtype=np.int32)
    want = O.store(hc, bt, 0, T, INT8)
    dc = dev_cache(hc)
    out = kdn.alloc_chunk(dc, T, INT8)
    kdn.kdn_store_chunk(dc, dev_table(bt), 0, T, out)
    assert_chunk_equal(out, want)
    sc = out.scales().cpu().numpy()[0, 0, :, 0]
    assert sc[n] == 0 and sc[n + 1] == 0 and sc[n + 2] > 0
    # and the special rows load back bit-exactly as the oracle says
    hd = O.PagedCache(np.zeros_like(k), np.zeros_like(v))
    O.load(want, hd, bt, 0)
    dd = dev_cache(O.PagedCache(np.zeros_like(k), np.zeros_like(v)))
    kdn.kdn_load_chunk(out, dd, dev_table(bt), 0)
    assert_cache_equal(dd, hd)


def test_store_strided_cache():
    """Paged memory with padded token and head strides (a view of a larger tensor)."""
    L, nb, bs, H, D = 2, 10, 16, 3, 64
    hc = host_cache(7, L, nb, bs, H, D)
    bt = synth.disjoint_block_tables(7, nb, [6])[0]
    want = O.store(hc, bt, 3, 80, INT8)
    big_k = torch.zeros((L, nb, bs, H + 2, D + 16), dtype=torch.bfloat16, device="cuda")
    big_v = torch.zeros_like(big_k)
    big_k[:, :, :, :H, :D] = to_dev_bf16(hc.k)
    big_v[:, :, :, :H, :D] = to_dev_bf16(hc.v)
    dc = kdn.PagedCache(big_k[:, :, :, :H, :D], big_v[:, :, :, :H, :D])
    out = kdn.alloc_chunk(dc, 80, INT8)
    kdn.kdn_store_chunk(dc, dev_table(bt), 3, 80, out)
    assert_chunk_equal(out, want)
    # and the way back into the padded layout touches no padding
    dst_bt = synth.disjoint_block_tables(8, nb, [6])[0]
    hd = host_cache(9, L, nb, bs, H, D)
    O.compose([want], [40], hd, dst_bt, 10000.0, dest=5)
    big_k.fill_(0), big_v.fill_(0)
    hd0 = host_cache(9, L, nb, bs, H, D)
    big_k[:, :, :, :H, :D] = to_dev_bf16(hd0.k)
    big_v[:, :, :, :H, :D] = to_dev_bf16(hd0.v)
    kdn.kdn_compose([out], [40], dc, dev_table(dst_bt), 10000.0, dest_token_start=5)
    assert_cache_equal(kdn.PagedCache(big_k[:, :, :, :H, :D].contiguous(), big_v[:, :, :, :H, :D].contiguous()), hd)
    assert float(big_k[:, :, :, H:, :].abs().max()) == 0 and float(big_k[..., D:].abs().max()) == 0


# ------------------------------------------------------------------ load / compose
@pytest.mark.parametrize("fmt", [RAW, INT8, INT4, FP8])
@pytest.mark.parametrize("shape", [
    # L, nb, bs, H, D, dest, T
    (2, 24, 16, 4, 64, 0, 128),
    (2, 24, 16, 4, 64, 7, 150),
    (3, 40, 16, 8, 128, 21, 301),
    (1, 64, 1, 2, 128, 3, 50),
    (2, 12, 32, 2, 64, 9, 300),
    (2, 12, 24, 3, 32, 7, 200),
    (1, 20, 16, 1, 16, 0, 97),
    (1, 20, 8, 2, 96, 3, 100),
    (1, 10, 16, 2, 256, 1, 77),
    (1, 6, 16, 1, 512, 0, 40),
    (2, 30, 3, 2, 64, 4, 70),
    (2, 64, 2, 3, 128, 1, 90),
    (3, 40, 16, 1, 128, 5, 300),
    (2, 12, 128, 1, 128, 9, 700),
    (2, 40, 16, 2, 64, 3, 333),
])
def test_load_matches_oracle_and_touches_nothing_else(fmt, shape):
    L, nb, bs, H, D, dest, T = shape
    if fmt == INT4 and D % 32:
        pytest.skip("int4 groups need head_dim % 32 == 0")
    _say("load fmt=%d shape=%s" % (fmt, shape))
    src = host_cache(200 + D, L, nb, bs, H, D)
    n_src = (T + bs - 1) // bs
    n_dst = (dest + T + bs - 1) // bs
    if n_src + n_dst > nb:
        src_bt = synth.disjoint_block_tables(4, nb, [n_src])[0]
        dst_bt = synth.disjoint_block_tables(5, nb, [n_dst])[0]
    else:
        src_bt, dst_bt = synth.disjoint_block_tables(4, nb, [n_src, n_dst])
    ch = O.store(src, src_bt, 0, T, fmt)
    hd = host_cache(300 + D, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.load(ch, hd, dst_bt, dest)
    kdn.kdn_load_chunk(chunk_to_dev(ch), dd, dev_table(dst_bt), dest)
    assert_cache_equal(dd, hd)


@pytest.mark.parametrize("fmt", [RAW, INT8, INT4, FP8])
@pytest.mark.parametrize("D,base", [(64, 10000.0), (128, 500000.0), (96, 10000.0), (16, 10000.0), (256, 1e6),
                                    (32, 10000.0), (512, 10000.0)])
def test_compose_ragged_chunks_with_offsets(fmt, D, base):
    L, nb, bs, H = 2, 64, 16, 2
    if fmt == INT4 and D % 32:
        pytest.skip("int4 groups need head_dim % 32 == 0")
    _say("compose fmt=%d D=%d" % (fmt, D))
    src = host_cache(400 + D, L, nb, bs, H, D)
    t1, t2, t3, t4, dst_bt = synth.disjoint_block_tables(11, nb, [4, 3, 5, 2, 16])
    chunks = [O.store(src, t1, 0, 61, fmt), O.store(src, t2, 2, 40, fmt),
              O.store(src, t3, 5, 70, fmt), O.store(src, t4, 0, 17, fmt)]
    offsets = [0, 61, -33, 100000]
    hd = host_cache(500 + D, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.compose(chunks, offsets, hd, dst_bt, base, dest=9)
    kdn.kdn_compose([chunk_to_dev(c) for c in chunks], offsets, dd, dev_table(dst_bt), base,
                    dest_token_start=9)
    assert_cache_equal(dd, hd)


def test_compose_mixed_formats_and_slices():
    L, nb, bs, H, D = 2, 48, 16, 4, 64
    src = host_cache(21, L, nb, bs, H, D)
    a, b, dst_bt = synth.disjoint_block_tables(21, nb, [10, 6, 18])
    whole = O.store(src, a, 0, 160, INT8)
    rawc = O.store(src, b, 3, 90, RAW)
    four = O.store(src, a, 16, 70, INT4)
    eight = O.store(src, b, 0, 40, FP8)
    chunks = [whole.slice(100, 50), rawc.slice(10, 33), whole.slice(0, 64), rawc.slice(0, 10), four.slice(5, 60),
              eight.slice(3, 30)]
    offsets = [7, 0, 50, -90, 33, -5]
    hd = host_cache(22, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.compose(chunks, offsets, hd, dst_bt, 10000.0, dest=1)
    dw, dr, d4, d8 = chunk_to_dev(whole), chunk_to_dev(rawc), chunk_to_dev(four), chunk_to_dev(eight)
    dchunks = [dw.slice(100, 50), dr.slice(10, 33), dw.slice(0, 64), dr.slice(0, 10), d4.slice(5, 60),
               d8.slice(3, 30)]
    kdn.kdn_compose(dchunks, offsets, dd, dev_table(dst_bt), 10000.0, dest_token_start=1)
    assert_cache_equal(dd, hd)


def test_fp8_special_rows_and_every_amax():
    """Every positive finite bf16 as a row's amax with companions at ratios that land on
    and next to e4m3 ties and in its subnormal range; zero and under-threshold rows."""
    L, nb, bs, H, D = 1, 2100, 16, 1, 32
    k = np.zeros((L, nb, bs, H, D), dtype=np.uint16)
    rows = k.reshape(-1, D)
    amax_bits = np.arange(1, 0x7F80, dtype=np.uint16)
    n = amax_bits.size
    rows[:n, 0] = amax_bits
    f = (amax_bits.astype(np.uint32) << 16).view(np.float32)
    ratios = (0.5, -0.25, 0.96875, -0.9375, 0.53125, 0.03515625, -0.001953125, 0.0009765625, 0.00048828125,
              0.000244140625, -0.0001, 0.3333, -0.0117, 0.99, 0.0021, -0.0033, 0.07, 0.6, -0.8, 0.15)
    for j, ratio in enumerate(ratios, start=1):
        rows[:n, j] = bits_of(torch.from_numpy((f * np.float32(ratio)).astype(np.float32)).to(torch.bfloat16))
    rows[n, 3] = 0x8000
    rows[n + 1, :] = 0x03FF                               # under 2^-119 everywhere
    rows[n + 2, :4] = [0x0400, 0x8400, 0x0380, 0x0001]    # exactly 2^-119
    hc = O.PagedCache(k, synth.normal_bf16(8, k.shape))
    T = nb * bs
    bt = np.arange(nb, dtype=np.int32)
    want = O.store(hc, bt, 0, T, FP8)
    dc = dev_cache(hc)
    out = kdn.alloc_chunk(dc, T, FP8)
    kdn.kdn_store_chunk(dc, dev_table(bt), 0, T, out)
    assert_chunk_equal(out, want)
    hd = O.PagedCache(np.zeros_like(hc.k), np.zeros_like(hc.v))
    O.load(want, hd, bt, 0)
    dd = dev_cache(O.PagedCache(np.zeros_like(hc.k), np.zeros_like(hc.v)))
    kdn.kdn_load_chunk(out, dd, dev_table(bt), 0)
    assert_cache_equal(dd, hd)
    # every e4m3 code decodes on the device as the oracle says
    codes = np.tile(np.arange(256, dtype=np.uint8), 4)                      # one row of 1024... as 32 rows of 32
    codes[codes == 0x7F] = 0
    codes[codes == 0xFF] = 0x80
    chunk = O.Chunk(np.zeros(O.chunk_bytes(1, 1, 32, 32, FP8), dtype=np.uint8), FP8, 1, 1, 32, 32)
    chunk.codes()[0, 0] = codes.reshape(32, 1, 32)
    chunk.codes()[0, 1] = codes.reshape(32, 1, 32)
    chunk.scales()[:] = np.float32(0.37)
    hd2 = O.PagedCache(np.zeros((1, 2, 16, 1, 32), dtype=np.uint16), np.zeros((1, 2, 16, 1, 32), dtype=np.uint16))
    O.load(chunk, hd2, np.array([1, 0], dtype=np.int32), 0)
    dd2 = dev_cache(O.PagedCache(np.zeros_like(hd2.k), np.zeros_like(hd2.v)))
    kdn.kdn_load_chunk(chunk_to_dev(chunk), dd2, dev_table(np.array([1, 0], dtype=np.int32)), 0)
    assert_cache_equal(dd2, hd2)


def test_int4_special_groups():
    """Zero groups, groups under the 2^-121 threshold, ties, and every positive finite
    bf16 as a group's amax."""
    L, nb, bs, H, D = 1, 2100, 16, 1, 32
    k = np.zeros((L, nb, bs, H, D), dtype=np.uint16)
    rows = k.reshape(-1, D)
    amax_bits = np.arange(1, 0x7F80, dtype=np.uint16)
    n = amax_bits.size
    rows[:n, 0] = amax_bits
    f = (amax_bits.astype(np.uint32) << 16).view(np.float32)
    for j, ratio in enumerate((0.5, -0.25, 0.75, -0.999, 0.0714, 0.2143, -0.3571, 0.6429, -0.9286), start=1):
        rows[:n, j] = bits_of(torch.from_numpy((f * np.float32(ratio)).astype(np.float32)).to(torch.bfloat16))
    rows[n, 3] = 0x8000
    rows[n + 1, :] = 0x02FF
    rows[n + 2, :4] = [0x0300, 0x8300, 0x0280, 0x0001]
    ties = torch.zeros(32)
    ties[:11] = torch.tensor([7.0, 3.5, -3.5, 0.5, -0.5, 1.5, 2.5, -2.5, 6.5, -6.5, 4.5])
    rows[n + 3] = bits_of(ties.to(torch.bfloat16))
    hc = O.PagedCache(k, synth.normal_bf16(6, k.shape))
    T = nb * bs
    bt = np.arange(nb, dtype=np.int32)
    want = O.store(hc, bt, 0, T, INT4)
    dc = dev_cache(hc)
    out = kdn.alloc_chunk(dc, T, INT4)
    kdn.kdn_store_chunk(dc, dev_table(bt), 0, T, out)
    assert_chunk_equal(out, want)
    hd = O.PagedCache(np.zeros_like(hc.k), np.zeros_like(hc.v))
    O.load(want, hd, bt, 0)
    dd = dev_cache(O.PagedCache(np.zeros_like(hc.k), np.zeros_like(hc.v)))
    kdn.kdn_load_chunk(out, dd, dev_table(bt), 0)
    assert_cache_equal(dd, hd)


def test_zero_offset_compose_is_bitwise_the_loads():
    """Raw chunks holding -0.0 and NaN-free extreme patterns survive store -> compose(0)."""
    L, nb, bs, H, D = 1, 16, 16, 2, 64
    k = synth.normal_bf16(31, (L, nb, bs, H, D))
    k[0, :, :, 0, ::7] = 0x8000
    k[0, :, :, 1, ::5] = 0x0001
    k[0, :, :, 1, 1::5] = 0x7F7F
    hc = O.PagedCache(k, synth.normal_bf16(32, (L, nb, bs, H, D)))
    a, b = synth.disjoint_block_tables(31, nb, [6, 6])
    dc = dev_cache(hc)
    out = kdn.alloc_chunk(dc, 96, RAW)
    kdn.kdn_store_chunk(dc, dev_table(a), 0, 96, out)
    kdn.kdn_compose([out.slice(0, 40), out.slice(40, 56)], [0, 0], dc, dev_table(b), 10000.0)
    torch.cuda.synchronize()
    gk, gv = bits_of(dc.k), bits_of(dc.v)
    assert np.array_equal(gk[:, b], hc.k[:, a]) and np.array_equal(gv[:, b], hc.v[:, a])


def test_many_chunks_go_through_the_device_segment_table():
    """More chunks than fit in the kernel arguments."""
    L, nb, bs, H, D = 1, 128, 16, 2, 64
    src = host_cache(41, L, nb, bs, H, D)
    a, dst_bt = synth.disjoint_block_tables(41, nb, [60, 60])
    whole = O.store(src, a, 0, 960, INT8)
    n = 100
    cuts = np.sort(synth._rng(41, 9).choice(np.arange(1, 900), size=n - 1, replace=False))
    cuts = np.concatenate([[0], cuts, [900]])
    order = synth.permutation(41, n)
    chunks = [whole.slice(int(cuts[i]), int(cuts[i + 1] - cuts[i])) for i in order]
    offsets = [int((i * 37) % 11 - 5) for i in range(n)]
    hd = host_cache(42, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.compose(chunks, offsets, hd, dst_bt, 10000.0, dest=3)
    dw = chunk_to_dev(whole)
    dchunks = [dw.slice(int(cuts[i]), int(cuts[i + 1] - cuts[i])) for i in order]
    for _ in range(3):       # the ring of device tables is reused
        kdn.kdn_compose(dchunks, offsets, dd, dev_table(dst_bt), 10000.0, dest_token_start=3)
    assert_cache_equal(dd, hd)


@pytest.mark.parametrize("D,fmt", [(128, INT8), (64, INT8), (96, FP8), (64, INT4), (256, RAW)])
def test_batched_compose_matches_independent_oracle_composes(D, fmt):
    """Requests that share chunks (the cached-load flavour of both place kernels)."""
    L, nb, bs, H = 2, 200, 16, 2
    _say("compose_batch D=%d fmt=%d" % (D, fmt))
    src = host_cache(51, L, nb, bs, H, D)
    tabs = synth.disjoint_block_tables(51, nb, [8] * 6 + [18] * 8)
    pool = [O.store(src, tabs[i], 0, 128 - 3 * i, fmt) for i in range(6)]
    dpool = [chunk_to_dev(c) for c in pool]
    draws = synth.zipf_distinct_draws(51, 8, 2, 6)
    hd = host_cache(52, L, nb, bs, H, D)
    dd = dev_cache(hd)
    reqs = []
    for r in range(8):
        ids = [int(x) for x in draws[r]]
        offs = [0, pool[ids[0]].T]
        O.compose([pool[i] for i in ids], offs, hd, tabs[6 + r], 500000.0, dest=r % 3)
        reqs.append(([dpool[i] for i in ids], offs, dev_table(tabs[6 + r]), r % 3))
    kdn.kdn_compose_batch(reqs, dd, 500000.0)
    assert_cache_equal(dd, hd)


@pytest.mark.parametrize("shape", [(16, 2, 128), (16, 8, 128), (32, 2, 64), (24, 2, 64), (2, 2, 128), (16, 1, 256),
                                   (16, 2, 96)])
@pytest.mark.parametrize("fmt", [INT8, RAW, INT4, FP8])
def test_views_read_once_for_many_destinations_equal_the_oracle(shape, fmt):
    """The same stored rows going to several destinations in one call: chained onto one set of
    workgroups where the tiles cut them the same way (same view, destinations congruent modulo
    the tile's token count), separate workgroups otherwise; every destination must hold what a
    compose of its own would have put there, with its own rotation."""
    bs, H, D = shape
    L, T = 2, 96
    probe = torch.zeros((L, 4, bs, H, D), dtype=torch.bfloat16)
    G = kdn.kdn_tile_tokens(kdn.PagedCache(probe, torch.zeros_like(probe)))
    span = 3 * G + 2 * T                                            # tokens a request's table covers
    need = [-(-span // bs)] * 7
    nb = sum(need) + -(-T // bs) + -(-5 // bs) + 3
    _say("chained views bs=%d H=%d D=%d fmt=%d (tile of %d tokens)" % (bs, H, D, fmt, G))
    src = host_cache(61, L, nb, bs, H, D)
    tabs = synth.disjoint_block_tables(61, nb, [-(-T // bs), -(-5 // bs)] + need)
    a = O.store(src, tabs[0], 0, T, fmt)
    b = O.store(src, tabs[1], 0, 5, fmt)
    da, db = chunk_to_dev(a), chunk_to_dev(b)
    hd = host_cache(62, L, nb, bs, H, D)
    dd = dev_cache(hd)
    sl = lambda t0, n: (a.slice(t0, n), da.slice(t0, n))
    # (views, offsets, destination start)
    cases = [([(a, da)], [0], 0), ([(a, da)], [T], G),                            # the chunk, a whole tile further on
             ([sl(16, 64)], [7], 32), ([sl(16, 64)], [-9], 32 + 2 * G),           # a slice, two tiles further on
             ([sl(16, 64)], [1000], 8),                                           # off that grid
             ([(b, db), (a, da), (a, da)], [3, 5, 0], 0),                         # the chunk, 5 tokens in, and right behind
             ([sl(17, 64), sl(16, 63)], [2, 4], 0)]                               # other slices of the buffer
    reqs = []
    for i, (views, offs, dest) in enumerate(cases):
        O.compose([h for h, _ in views], offs, hd, tabs[2 + i], 10000.0, dest=dest)
        reqs.append(([d for _, d in views], offs, dev_table(tabs[2 + i]), dest))
    plan = kdn.kdn_compose_plan(reqs, dd)
    assert sum(p["follows"] >= 0 for p in plan) >= 2, plan           # the case is about chains: there are some
    kdn.kdn_compose_batch(reqs, dd, 10000.0)
    assert_cache_equal(dd, hd)
    # one request that holds the chunk twice a tile apart, through a capped launch (workgroups stride
    # over tiles, each walking its chain)
    hd2 = host_cache(63, L, nb, bs, H, D)
    dd2 = dev_cache(hd2)
    pad = -T % G                                                    # tokens up to the next tile boundary
    views = [(a, da)] + ([sl(0, pad)] if pad else []) + [(a, da)]
    offs = list(range(len(views)))
    O.compose([h for h, _ in views], offs, hd2, tabs[2], 10000.0, dest=0)
    kdn.kdn_compose([d for _, d in views], offs, dd2, dev_table(tabs[2]), 10000.0, 0, max_workgroups=3)
    assert_cache_equal(dd2, hd2)
    assert [p["follows"] for p in kdn.kdn_compose_plan([([d for _, d in views], offs, dev_table(tabs[2]), 0)], dd2)] \
        == [-1] * (len(views) - 1) + [0]


# ------------------------------------------------------------------ utilities
@pytest.mark.timeout(600)
def test_f32_to_bf16_every_input_pattern():
    """All 2^32 fp32 inputs, in 64 slabs, against the oracle's conversion."""
    lo = torch.arange(0, 1 << 26, dtype=torch.int64, device="cuda")
    for slab in range(64):
        u = (lo + (slab << 26)).to(torch.int32) if slab < 32 else (lo + (slab << 26) - (1 << 32)).to(torch.int32)
        x = u.view(torch.float32)
        got = bits_of(kdn.kdn_f32_to_bf16(x))
        xh = x.cpu().numpy()
        want = O.f32_to_bf16(xh)
        nan = np.isnan(xh)
        if slab % 8 == 0:
            print("[bf16] slab %d" % slab, flush=True)
        assert np.array_equal(got[~nan], want[~nan]), "slab %d" % slab
        assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x7F) != 0)


def test_validate_block_table():
    ok = dev_table(np.array([5, 1, 7, 0], dtype=np.int32))
    assert kdn.kdn_validate_block_table(ok, 8) == kdn.OK
    assert kdn.kdn_validate_block_table(ok, 7) == kdn.ERANGE
    assert kdn.kdn_validate_block_table(dev_table(np.array([5, 1, 5], dtype=np.int32)), 8) == kdn.ERANGE
    assert kdn.kdn_validate_block_table(dev_table(np.array([-1, 2], dtype=np.int32)), 8) == kdn.ERANGE


def test_rope_prepare_then_compose_and_shutdown_are_repeatable():
    L, nb, bs, H, D = 1, 16, 16, 1, 64
    src = host_cache(61, L, nb, bs, H, D)
    a, b = synth.disjoint_block_tables(61, nb, [4, 4])
    ch = O.store(src, a, 0, 64, INT8)
    kdn.kdn_rope_prepare(10000.0, D, [5, 6, 7])
    for _ in range(2):
        hd = host_cache(62, L, nb, bs, H, D)
        dd = dev_cache(hd)
        O.compose([ch], [6], hd, b, 10000.0)
        kdn.kdn_compose([chunk_to_dev(ch)], [6], dd, dev_table(b), 10000.0)
        assert_cache_equal(dd, hd)
        torch.cuda.synchronize()
        kdn.kdn_shutdown()


# ------------------------------------------------------------------ chunks streamed from host memory
@pytest.mark.parametrize("layers_per_stage", [1, 2, 3, 8])
def test_compose_from_pinned_host_chunks_equals_compose(layers_per_stage):
    """Stored chunks (every format, whole and sliced) that live in pinned host memory are
    streamed in stages of layers; the result is the oracle's compose."""
    L, nb, bs, H, D = 5, 64, 16, 2, 64
    _say("compose_from_host layers_per_stage=%d" % layers_per_stage)
    src = host_cache(71, L, nb, bs, H, D)
    t1, t2, t3, t4, dst_bt = synth.disjoint_block_tables(71, nb, [6, 5, 4, 4, 24])
    a = O.store(src, t1, 0, 90, INT8)
    b = O.store(src, t2, 3, 70, RAW)
    c = O.store(src, t3, 0, 64, INT4)
    d = O.store(src, t4, 1, 50, FP8)
    chunks = [a.slice(10, 75), b, c, a.slice(0, 10), b.slice(20, 31), d.slice(5, 40), c.slice(33, 20)]
    offsets = [0, 75, -12, 300, 7, 1000, 55]
    hd = host_cache(72, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.compose(chunks, offsets, hd, dst_bt, 10000.0, dest=5)
    ha, hb, hc, hdd = (kdn.pinned_host_copy(chunk_to_dev(x)) for x in (a, b, c, d))
    hchunks = [ha.slice(10, 75), hb, hc, ha.slice(0, 10), hb.slice(20, 31), hdd.slice(5, 40), hc.slice(33, 20)]
    need = kdn.kdn_staging_bytes(hchunks, layers_per_stage)
    assert need > 0
    staging = torch.empty(need, dtype=torch.uint8, device="cuda")
    for _ in range(2):          # a second call reuses the staging halves
        kdn.kdn_compose_from_host(hchunks, offsets, dd, dev_table(dst_bt), 10000.0, staging,
                                  layers_per_stage, dest_token_start=5)
    assert_cache_equal(dd, hd)
    # the same staging memory cut into halves of another size, with the previous call still in flight
    other = 3 if layers_per_stage != 3 else 2
    big = torch.empty(max(need, kdn.kdn_staging_bytes(hchunks, other)), dtype=torch.uint8, device="cuda")
    dd2 = dev_cache(host_cache(72, L, nb, bs, H, D))
    kdn.kdn_compose_from_host(hchunks, offsets, dd2, dev_table(dst_bt), 10000.0, big[:need], layers_per_stage, dest_token_start=5)
    kdn.kdn_compose_from_host(hchunks, offsets, dd, dev_table(dst_bt), 10000.0, big, other, dest_token_start=5)
    assert_cache_equal(dd, hd)
    assert_cache_equal(dd2, hd)
    small = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(kdn.KdnError) as e:
        kdn.kdn_compose_from_host(hchunks, offsets, dd, dev_table(dst_bt), 10000.0, small, layers_per_stage)
    assert e.value.status == kdn.ESIZE
    with pytest.raises(kdn.KdnError) as e:       # device-resident chunks are refused here
        kdn.kdn_compose_from_host([chunk_to_dev(c)], [0], dd, dev_table(dst_bt), 10000.0, staging, layers_per_stage)
    assert e.value.status == kdn.EINVAL


def test_compose_from_host_stage_events_release_layers_in_order():
    """A second stream waits for the event of each stage and snapshots that stage's layers
    while later stages are still being streamed: every snapshot already holds the oracle's
    final values."""
    L, nb, bs, H, D = 6, 64, 16, 2, 128
    lps = 2
    _say("compose_from_host_staged")
    src = host_cache(81, L, nb, bs, H, D)
    t1, t2, dst_bt = synth.disjoint_block_tables(81, nb, [8, 8, 20])
    a, b = O.store(src, t1, 0, 128, INT8), O.store(src, t2, 0, 120, FP8)
    views, offsets = [a.slice(5, 100), b, a.slice(0, 60)], [17, 0, 2000]
    hd = host_cache(82, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.compose(views, offsets, hd, dst_bt, 500000.0, dest=3)
    ha, hb = kdn.pinned_host_copy(chunk_to_dev(a)), kdn.pinned_host_copy(chunk_to_dev(b))
    hviews = [ha.slice(5, 100), hb, ha.slice(0, 60)]
    staging = torch.empty(kdn.kdn_staging_bytes(hviews, lps), dtype=torch.uint8, device="cuda")
    events = [torch.cuda.Event() for _ in range(L // lps)]
    for e in events:
        e.record()
    side = torch.cuda.Stream()
    snaps = []
    kdn.kdn_compose_from_host(hviews, offsets, dd, dev_table(dst_bt), 500000.0, staging, lps,
                              dest_token_start=3, stage_events=events)
    with torch.cuda.stream(side):
        for s, e in enumerate(events):
            side.wait_event(e)
            snaps.append((dd.k[s * lps:(s + 1) * lps].clone(), dd.v[s * lps:(s + 1) * lps].clone()))
    torch.cuda.synchronize()
    for s, (ks, vs) in enumerate(snaps):
        assert np.array_equal(bits_of(ks), hd.k[s * lps:(s + 1) * lps]), "K of stage %d" % s
        assert np.array_equal(bits_of(vs), hd.v[s * lps:(s + 1) * lps]), "V of stage %d" % s
    assert_cache_equal(dd, hd)
    with pytest.raises(kdn.KdnError) as e:                      # one event per stage, no fewer
        kdn.kdn_compose_from_host(hviews, offsets, dd, dev_table(dst_bt), 500000.0, staging, lps,
                                  dest_token_start=3, stage_events=events[:2])
    assert e.value.status == kdn.EINVAL


# ------------------------------------------------------------------ RoPE variants, patching
@pytest.mark.parametrize("fmt", [RAW, INT8, INT4, FP8])
@pytest.mark.parametrize("variant", [
    # D, rot_dim, pairing, explicit frequencies?
    (128, 0, 1, False),        # interleaved pairs, whole row
    (128, 64, 0, False),       # partial rotary, half-split
    (128, 64, 1, False),       # partial rotary, interleaved
    (64, 32, 0, True),         # explicit (rescaled) frequencies, partial
    (128, 0, 0, True),         # explicit frequencies, plain pairing
    (256, 16, 1, False),       # smallest rotary part
    (96, 32, 0, False),        # head_dim whose lane group is padded
])
def test_compose_rope_variants(fmt, variant):
    D, rot, pairing, explicit = variant
    _say("compose_rope fmt=%d variant=%s" % (fmt, variant))
    L, nb, bs, H = 2, 64, 16, 2
    base = 500000.0
    r = rot or D
    inv_freq = None
    if explicit:
        j = np.arange(r // 2, dtype=np.float64)
        inv_freq = base ** (-2.0 * j / r) / np.where(j >= r // 4, 8.0, 1.0)
    src = host_cache(600 + D, L, nb, bs, H, D)
    t1, t2, t3, dst_bt = synth.disjoint_block_tables(13, nb, [4, 3, 5, 16])
    chunks = [O.store(src, t1, 0, 61, fmt), O.store(src, t2, 2, 40, fmt), O.store(src, t3, 5, 70, fmt)]
    offsets = [0, 61, -1000]
    hd = host_cache(700 + D, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.compose_spec(chunks, offsets, hd, dst_bt, base, inv_freq=inv_freq, rot_dim=rot, pairing=pairing, dest=9)
    spec = kdn.rope_spec(base, inv_freq, rot, pairing)
    kdn.kdn_compose_rope([chunk_to_dev(c) for c in chunks], offsets, dd, dev_table(dst_bt), spec,
                         dest_token_start=9)
    assert_cache_equal(dd, hd)


def test_compose_rope_default_spec_is_compose():
    L, nb, bs, H, D = 2, 32, 16, 2, 64
    src = host_cache(81, L, nb, bs, H, D)
    a, b = synth.disjoint_block_tables(81, nb, [5, 8])
    ch = O.store(src, a, 0, 77, INT8)
    hd = host_cache(82, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.compose([ch], [33], hd, b, 10000.0, dest=4)
    kdn.kdn_compose_rope([chunk_to_dev(ch)], [33], dd, dev_table(b), kdn.rope_spec(10000.0), dest_token_start=4)
    assert_cache_equal(dd, hd)
    kdn.kdn_rope_prepare_spec(kdn.rope_spec(10000.0, None, 32, 1), D, [1, 2, 3])
    bad = kdn.rope_spec(10000.0, None, 24, 0)                 # rot_dim not a multiple of 16
    with pytest.raises(kdn.KdnError) as e:
        kdn.kdn_compose_rope([chunk_to_dev(ch)], [33], dd, dev_table(b), bad)
    assert e.value.status == kdn.EUNSUPPORTED
    bad = kdn.rope_spec(10000.0, None, 0, 5)
    with pytest.raises(kdn.KdnError) as e:
        kdn.kdn_compose_rope([chunk_to_dev(ch)], [33], dd, dev_table(b), bad)
    assert e.value.status == kdn.EINVAL


def test_batched_compose_with_a_variant():
    L, nb, bs, H, D = 2, 96, 16, 2, 128
    src = host_cache(83, L, nb, bs, H, D)
    tabs = synth.disjoint_block_tables(83, nb, [6] * 4 + [12] * 5)
    pool = [O.store(src, tabs[i], 0, 90 - i, INT8) for i in range(4)]
    dpool = [chunk_to_dev(c) for c in pool]
    hd = host_cache(84, L, nb, bs, H, D)
    dd = dev_cache(hd)
    reqs = []
    for r in range(5):
        ids = [r % 4, (r + 1) % 4]
        offs = [5 * r, -pool[ids[0]].T]
        O.compose_spec([pool[i] for i in ids], offs, hd, tabs[4 + r], 10000.0, rot_dim=64, pairing=1, dest=r)
        reqs.append(([dpool[i] for i in ids], offs, dev_table(tabs[4 + r]), r))
    kdn.kdn_compose_batch_rope(reqs, dd, kdn.rope_spec(10000.0, None, 64, 1))
    assert_cache_equal(dd, hd)


@pytest.mark.parametrize("shape", [(2, 24, 16, 4, 64), (3, 40, 16, 8, 128), (1, 30, 8, 3, 96), (1, 64, 1, 2, 32)])
def test_patch_rows_matches_oracle(shape):
    L, nb, bs, H, D = shape
    hc = host_cache(85 + D, L, nb, bs, H, D)
    dc = dev_cache(hc)
    n_tab = min(nb - 2, 12)
    bt = synth.disjoint_block_tables(85, nb, [n_tab])[0]
    cap = n_tab * bs
    tokens = synth.permutation(86, cap)[:min(cap, 37)].astype(np.int32)
    rows = synth.normal_bf16(87, (L, 2, len(tokens), H, D))
    O.patch_rows(rows, tokens, hc, bt)
    kdn.kdn_patch_rows(to_dev_bf16(rows), torch.from_numpy(tokens).cuda(), dc, dev_table(bt))
    assert_cache_equal(dc, hc)
    # a token outside the table is skipped, the others still land
    tok2 = tokens.copy()
    tok2[0] = cap + 5
    rows2 = synth.normal_bf16(88, rows.shape)
    O.patch_rows(rows2[:, :, 1:], tok2[1:], hc, bt)
    kdn.kdn_patch_rows(to_dev_bf16(rows2), torch.from_numpy(tok2).cuda(), dc, dev_table(bt))
    assert_cache_equal(dc, hc)


# ------------------------------------------------------------------ HIP graph capture
def test_capped_store_to_and_compose_from_host_memory_replay_inside_a_hip_graph():
    """Chunks in pinned host memory, capped launches, kernels only: the store into host
    memory and the compose back from it are captured once and replayed with fresh data."""
    L, nb, bs, H, D = 2, 48, 16, 2, 64
    a, c = synth.disjoint_block_tables(93, nb, [8, 12])
    offsets = [40, 0]
    base = 10000.0
    hc = host_cache(94, L, nb, bs, H, D)
    dc = dev_cache(hc)
    ta, tc = dev_table(a), dev_table(c)
    out = kdn.alloc_host_chunk(dc, 120, FP8)
    kdn.kdn_rope_prepare(base, D, offsets)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        kdn.kdn_store_chunk(dc, ta, 2, 120, out, max_workgroups=8)       # warm-up outside the capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            kdn.kdn_store_chunk(dc, ta, 2, 120, out, max_workgroups=8)
            kdn.kdn_compose([out.slice(60, 60), out.slice(0, 60)], offsets, dc, tc, base, dest_token_start=1,
                            max_workgroups=8)
    torch.cuda.synchronize()
    for rep in range(3):
        fresh = host_cache(110 + rep, L, nb, bs, H, D)
        dc.k.copy_(to_dev_bf16(fresh.k))
        dc.v.copy_(to_dev_bf16(fresh.v))
        out.data.fill_(0x11 * rep)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        h = O.store(fresh, a, 2, 120, FP8)
        O.compose([h.slice(60, 60), h.slice(0, 60)], offsets, fresh, c, base, dest=1)
        assert np.array_equal(out.data.numpy(), h.data)
        assert_cache_equal(dc, fresh)
        _ = (dc.k.float().sum() + dc.v.float().sum()).item()   # unrelated eager work between replays


def test_store_and_compose_replay_inside_a_hip_graph():
    """With the cos/sin rows resident, store / load / compose enqueue kernels only, so a
    captured sequence can be replayed: every replay is checked against the oracle with
    fresh source data, with eager work and synchronisation between the replays."""
    L, nb, bs, H, D = 2, 48, 16, 2, 128
    a, b, c = synth.disjoint_block_tables(91, nb, [6, 6, 12])
    offsets = [0, 96]
    base = 500000.0
    hc = host_cache(92, L, nb, bs, H, D)
    dc = dev_cache(hc)
    ta, tb, tc = dev_table(a), dev_table(b), dev_table(c)
    out1 = kdn.alloc_chunk(dc, 96, INT8)
    out2 = kdn.alloc_chunk(dc, 96, INT4)
    kdn.kdn_rope_prepare(base, D, offsets)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        kdn.kdn_store_chunk(dc, ta, 0, 96, out1)            # warm-up outside the capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            kdn.kdn_store_chunk(dc, ta, 0, 96, out1)
            kdn.kdn_store_chunk(dc, tb, 0, 96, out2)
            kdn.kdn_compose([out1, out2], offsets, dc, tc, base)
    torch.cuda.synchronize()
    for rep in range(3):
        fresh = host_cache(100 + rep, L, nb, bs, H, D)
        dc.k.copy_(to_dev_bf16(fresh.k))
        dc.v.copy_(to_dev_bf16(fresh.v))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        h1 = O.store(fresh, a, 0, 96, INT8)
        h2 = O.store(fresh, b, 0, 96, INT4)
        O.compose([h1, h2], offsets, fresh, c, base)
        assert_chunk_equal(out1, h1)
        assert_chunk_equal(out2, h2)
        assert_cache_equal(dc, fresh)
        _ = (dc.k.float().sum() + dc.v.float().sum()).item()   # unrelated eager work between replays


# ------------------------------------------------------------------ token-list store
@pytest.mark.parametrize("fmt", [RAW, INT8, INT4, FP8])
@pytest.mark.parametrize("shape", [(2, 24, 16, 4, 64), (3, 40, 16, 8, 128), (1, 30, 8, 3, 96), (1, 64, 1, 2, 32)])
def test_store_tokens_matches_oracle(fmt, shape):
    L, nb, bs, H, D = shape
    _say("store_tokens fmt=%d shape=%s" % (fmt, shape))
    hc = host_cache(95 + D, L, nb, bs, H, D)
    n_tab = min(nb - 2, 14)
    bt = synth.disjoint_block_tables(95, nb, [n_tab])[0]
    cap = n_tab * bs
    tokens = np.sort(synth.permutation(96, cap)[:max(1, (cap * 2) // 3)]).astype(np.int32)   # a kept subset
    want = O.store_tokens(hc, bt, tokens, fmt)
    dc = dev_cache(hc)
    out = kdn.alloc_chunk(dc, len(tokens), fmt)
    out.data.fill_(0xCD)
    kdn.kdn_store_tokens(dc, dev_table(bt), torch.from_numpy(tokens).cuda(), out)
    assert_chunk_equal(out, want)
    # the thinned chunk composes like any other
    dst_bt = synth.disjoint_block_tables(97, nb, [n_tab])[0]
    hd = host_cache(98, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.compose([want], [11], hd, dst_bt, 10000.0)
    kdn.kdn_compose([out], [11], dd, dev_table(dst_bt), 10000.0)
    assert_cache_equal(dd, hd)


# ------------------------------------------------------------------ planner state under load
def test_cos_sin_table_recycles_transient_rows_and_keeps_pinned_ones():
    """More distinct offsets than the resident table holds.  Rows that composes bring in by
    themselves are dropped when the table is full and composes before and after still match
    the oracle; rows that kdn_rope_prepare pinned keep their place, so a graph captured
    before the table overflowed replays with the right cos/sin values afterwards."""
    L, nb, bs, H, D = 1, 24, 16, 1, 32
    src = host_cache(111, L, nb, bs, H, D)
    a, b, c = synth.disjoint_block_tables(111, nb, [2, 4, 8])
    ch = O.store(src, a, 0, 32, INT8)
    dch = chunk_to_dev(ch)
    base = 12345.0                                 # a table of its own
    pinned = [777, -4242]
    kdn.kdn_rope_prepare(base, D, pinned)
    dd = dev_cache(host_cache(112, L, nb, bs, H, D))
    tb, tc = dev_table(b), dev_table(c)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        kdn.kdn_compose([dch, dch], pinned, dd, tb, base)       # warm-up outside the capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            kdn.kdn_compose([dch, dch], pinned, dd, tb, base)
    torch.cuda.synchronize()
    views = [dch.slice(i % 32, 1) for i in range(64)]
    hviews = [ch.slice(i % 32, 1) for i in range(64)]
    n_calls = 0
    for start in range(1, 6000, 64):               # 94 composes of 64 new offsets each: capacity is 4096
        offs = list(range(start, start + 64))
        kdn.kdn_compose(views, offs, dd, tc, base)
        n_calls += 1
        if start in (1, 1985, 4033, 4097, 5953):   # before, around and after the table fills up
            hd = host_cache(113, L, nb, bs, H, D)
            d2 = dev_cache(hd)
            O.compose(hviews, offs, hd, c, base)
            kdn.kdn_compose(views, offs, d2, tc, base)
            assert_cache_equal(d2, hd)
    assert n_calls * 64 > 4096 + 64
    # the captured compose still reads its own rows
    for rep in range(2):
        hd = host_cache(114 + rep, L, nb, bs, H, D)
        dd.k.copy_(to_dev_bf16(hd.k))
        dd.v.copy_(to_dev_bf16(hd.v))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        O.compose([ch, ch], pinned, hd, b, base)
        assert_cache_equal(dd, hd)
        _ = (dd.k.float().sum()).item()             # unrelated eager work between replays
    # pinning more rows than the table holds is refused and changes nothing
    kdn.kdn_rope_prepare(base, D, list(range(10000, 14000)))
    with pytest.raises(kdn.KdnError) as e:
        kdn.kdn_rope_prepare(base, D, list(range(20000, 20200)))
    assert e.value.status == kdn.EFULL
    with pytest.raises(kdn.KdnError) as e:          # more distinct offsets in ONE call than the table holds
        kdn.kdn_rope_prepare(base, D, list(range(1, 5000)))
    assert e.value.status == kdn.ESIZE
    with pytest.raises(kdn.KdnError) as e:          # a compose whose transient rows do not fit beside the pinned ones
        kdn.kdn_compose(views + views, list(range(30000, 30128)), dd, tc, base)
    assert e.value.status == kdn.EFULL
    hd = host_cache(116, L, nb, bs, H, D)
    d3 = dev_cache(hd)
    O.compose([ch, ch], pinned, hd, b, base)
    kdn.kdn_compose([dch, dch], pinned, d3, tb, base)
    assert_cache_equal(d3, hd)
    # after a release everything can be prepared again (graphs captured before must not be replayed)
    kdn.kdn_rope_release()
    kdn.kdn_rope_prepare(base, D, list(range(20000, 20200)))
    hd = host_cache(117, L, nb, bs, H, D)
    d4 = dev_cache(hd)
    O.compose([ch, ch], [20100, 777], hd, b, base)
    kdn.kdn_compose([dch, dch], [20100, 777], d4, tb, base)
    assert_cache_equal(d4, hd)
    kdn.kdn_rope_release()


def test_store_to_host_then_compose_from_host_on_one_stream_without_a_host_sync():
    """Both staged calls are ordered on the caller's stream: a compose from a host chunk
    that the preceding call on the same stream is still storing, through a staging tensor
    that kernels of that stream used just before, sees the finished chunk."""
    L, nb, bs, H, D = 8, 96, 16, 4, 128
    src = host_cache(141, L, nb, bs, H, D)
    a, b = synth.disjoint_block_tables(141, nb, [32, 32])
    T = 500
    want = O.store(src, a, 3, T, INT8)
    hd = host_cache(142, L, nb, bs, H, D)
    O.compose([want.slice(100, 400), want.slice(0, 100)], [64, -9], hd, b, 10000.0, dest=2)
    dc = dev_cache(src)
    dd = dev_cache(host_cache(142, L, nb, bs, H, D))
    ta, tb = dev_table(a), dev_table(b)
    out = kdn.alloc_host_chunk(dc, T, INT8)
    views = [out.slice(100, 400), out.slice(0, 100)]
    lps = 2
    n = max(kdn.kdn_store_staging_bytes(dc, T, INT8, lps), kdn.kdn_staging_bytes(views, lps))
    staging = torch.empty(n, dtype=torch.uint8, device="cuda")
    kdn.kdn_rope_prepare(10000.0, D, [64, -9])
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        for rep in range(3):
            out.data.fill_(0xEE)                     # host-side fill: the stream is idle here
            staging.fill_(0x5A)                      # a kernel of this stream writes the staging memory
            kdn.kdn_store_to_host(dc, ta, 3, T, out, staging, lps, stream=s)
            kdn.kdn_compose_from_host(views, [64, -9], dd, tb, 10000.0, staging, lps, dest_token_start=2, stream=s)
            s.synchronize()
            assert np.array_equal(out.data.numpy(), want.data), "host chunk, round %d" % rep
            assert_cache_equal(dd, hd)
            dd.k.zero_()
            dd.v.zero_()
            hd0 = host_cache(142, L, nb, bs, H, D)
            dd.k.copy_(to_dev_bf16(hd0.k))
            dd.v.copy_(to_dev_bf16(hd0.v))
            s.synchronize()


def test_two_streams_and_two_host_threads():
    """Independent composes issued from two host threads on two streams into disjoint
    tables of one cache."""
    import threading
    L, nb, bs, H, D = 2, 96, 16, 2, 128
    src = host_cache(121, L, nb, bs, H, D)
    tabs = synth.disjoint_block_tables(121, nb, [6, 6, 20, 20])
    c1, c2 = O.store(src, tabs[0], 0, 96, INT8), O.store(src, tabs[1], 0, 96, INT4)
    d1, d2 = chunk_to_dev(c1), chunk_to_dev(c2)
    hd = host_cache(122, L, nb, bs, H, D)
    dd = dev_cache(hd)
    bt = [dev_table(tabs[2]), dev_table(tabs[3])]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    errors = []

    def worker(i):
        try:
            with torch.cuda.stream(streams[i]):
                for rep in range(20):
                    kdn.kdn_compose([d1, d2, d1], [rep + 1, -(rep + 1), 100 * i], dd, bt[i], 500000.0,
                                    stream=streams[i])
                    kdn.kdn_load_chunk(d2, dd, bt[i], 220, stream=streams[i])
        except Exception as exc:                    # surfaced in the main thread
            errors.append(exc)

    th = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in th:
        t.start()
    for t in th:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i in range(2):
        O.compose([c1, c2, c1], [20, -20, 100 * i], hd, tabs[2 + i], 500000.0)
        O.load(c2, hd, tabs[2 + i], 220)
    assert_cache_equal(dd, hd)


@pytest.mark.parametrize("fmt", [RAW, INT8, INT4, FP8])
@pytest.mark.parametrize("layers_per_stage", [1, 2, 5])
def test_store_to_pinned_host_memory_and_back(fmt, layers_per_stage):
    """The staged store lands the oracle's chunk bytes in host memory; streamed back through
    kdn_compose_from_host they give the oracle's compose."""
    L, nb, bs, H, D = 5, 48, 16, 2, 64
    _say("store_to_host fmt=%d layers_per_stage=%d" % (fmt, layers_per_stage))
    src = host_cache(131, L, nb, bs, H, D)
    a, b = synth.disjoint_block_tables(131, nb, [8, 10])
    want = O.store(src, a, 5, 110, fmt)
    dc = dev_cache(src)
    out = kdn.alloc_host_chunk(dc, 110, fmt)
    out.data.fill_(0xEE)
    staging = torch.empty(kdn.kdn_store_staging_bytes(dc, 110, fmt, layers_per_stage), dtype=torch.uint8, device="cuda")
    for _ in range(2):
        kdn.kdn_store_to_host(dc, dev_table(a), 5, 110, out, staging, layers_per_stage)
    torch.cuda.synchronize()
    assert np.array_equal(out.data.numpy(), want.data)
    assert (out.desc.parent_tokens, out.desc.num_tokens) == (110, 110)
    hd = host_cache(132, L, nb, bs, H, D)
    dd = dev_cache(hd)
    O.compose([want.slice(10, 90)], [64], hd, b, 10000.0, dest=3)
    view = out.slice(10, 90)
    st2 = torch.empty(kdn.kdn_staging_bytes([view], layers_per_stage), dtype=torch.uint8, device="cuda")
    kdn.kdn_compose_from_host([view], [64], dd, dev_table(b), 10000.0, st2, layers_per_stage, dest_token_start=3)
    assert_cache_equal(dd, hd)
    with pytest.raises(kdn.KdnError) as e:                      # a device buffer is not a host destination
        lib_store_to_host_with_device_chunk(dc, a, fmt, staging, layers_per_stage)
    assert e.value.status == kdn.EINVAL


@pytest.mark.parametrize("fmt", [RAW, INT8, INT4, FP8])
def test_kernels_on_chunks_in_pinned_host_memory(fmt):
    """Store, load and compose with the chunk itself in pinned host memory (no staging, the
    kernels cross the link): the oracle's bytes land in host memory, and views of the host
    chunk compose to the oracle's result."""
    L, nb, bs, H, D = 3, 64, 16, 2, 128
    _say("direct host chunk fmt=%d" % fmt)
    src = host_cache(141, L, nb, bs, H, D)
    a, b, c = synth.disjoint_block_tables(141, nb, [9, 12, 8])
    want = O.store(src, a, 7, 130, fmt)
    dc = dev_cache(src)
    out = kdn.alloc_host_chunk(dc, 130, fmt)
    out.data.fill_(0xEE)
    kdn.kdn_store_chunk(dc, dev_table(a), 7, 130, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.data.numpy(), want.data)
    keep = synth.permutation(141, 130)[:40].astype(np.int32) + 7
    want_t = O.store_tokens(src, a, keep, fmt)
    out_t = kdn.alloc_host_chunk(dc, 40, fmt)
    kdn.kdn_store_tokens(dc, dev_table(a), torch.from_numpy(keep).cuda(), out_t)
    torch.cuda.synchronize()
    assert np.array_equal(out_t.data.numpy(), want_t.data)
    hd = host_cache(142, L, nb, bs, H, D)
    dd = dev_cache(hd)
    views = [want.slice(100, 30), want_t, want.slice(0, 64), want.slice(50, 37)]
    offsets = [0, 30, -20, 4000]
    O.compose(views, offsets, hd, b, 500000.0, dest=9)
    O.load(want.slice(3, 100), hd, c, 11)
    # host- and device-resident chunks side by side in one call
    on_dev = chunk_to_dev(want)
    hviews = [out.slice(100, 30), out_t, on_dev.slice(0, 64), out.slice(50, 37)]
    kdn.kdn_compose(hviews, offsets, dd, dev_table(b), 500000.0, dest_token_start=9)
    kdn.kdn_load_chunk(out.slice(3, 100), dd, dev_table(c), 11)
    assert_cache_equal(dd, hd)


@pytest.mark.parametrize("cap", [1, 7, 64, 100000])
@pytest.mark.parametrize("D,fmt", [(128, INT8), (64, INT4), (96, RAW), (128, FP8)])
def test_capped_launch_gives_the_same_result(cap, D, fmt):
    """A launch with fewer workgroups than tiles strides over them: same stored bytes, same
    composed cache, for both place kernels, device- and host-resident chunks, a RoPE variant."""
    L, nb, bs, H = 3, 64, 16, 2
    _say("capped launch cap=%d D=%d fmt=%d" % (cap, D, fmt))
    src = host_cache(151, L, nb, bs, H, D)
    a, b, dst_bt = synth.disjoint_block_tables(151, nb, [10, 8, 22])
    want_a, want_b = O.store(src, a, 3, 150, fmt), O.store(src, b, 0, 100, fmt)
    dc = dev_cache(src)
    out_a = kdn.alloc_chunk(dc, 150, fmt)
    out_b = kdn.alloc_host_chunk(dc, 100, fmt)
    kdn.kdn_store_chunk(dc, dev_table(a), 3, 150, out_a, max_workgroups=cap)
    kdn.kdn_store_chunk(dc, dev_table(b), 0, 100, out_b, max_workgroups=cap)
    assert_chunk_equal(out_a, want_a)
    assert np.array_equal(out_b.data.numpy(), want_b.data)
    views_h = [want_a.slice(20, 100), want_b, want_a.slice(0, 33), want_b.slice(50, 50)]
    views_d = [out_a.slice(20, 100), out_b, out_a.slice(0, 33), out_b.slice(50, 50)]
    offsets = [0, 100, -7, 2048]
    for spec in (None, kdn.rope_spec(10000.0, None, 32, kdn.ROPE_INTERLEAVED)):
        hd = host_cache(152, L, nb, bs, H, D)
        dd = dev_cache(hd)
        if spec is None:
            O.compose(views_h, offsets, hd, dst_bt, 10000.0, dest=5)
        else:
            O.compose_spec(views_h, offsets, hd, dst_bt, 10000.0, rot_dim=32, pairing=1, dest=5)
        kdn.kdn_compose(views_d, offsets, dd, dev_table(dst_bt), 10000.0, dest_token_start=5,
                        max_workgroups=cap, spec=spec)
        assert_cache_equal(dd, hd)


def test_host_path_argument_errors():
    """Pageable host memory, short or misaligned staging memory and a negative cap come back
    as status codes with nothing enqueued."""
    import ctypes as C
    L, nb, bs, H, D = 2, 16, 16, 2, 64
    hc = host_cache(161, L, nb, bs, H, D)
    dc = dev_cache(hc)
    bt = dev_table(np.arange(8, dtype=np.int32))
    cd = dc.desc()
    need = kdn.kdn_store_staging_bytes(dc, 100, INT8, 1)
    staging = torch.empty(need + 16, dtype=torch.uint8, device="cuda")
    pageable = kdn.chunk_from_buffer(torch.empty(kdn.kdn_chunk_bytes(L, H, D, 100, INT8), dtype=torch.uint8),
                                     INT8, L, H, D, 100)
    pinned = kdn.alloc_host_chunk(dc, 100, INT8)

    def store_to_host(chunk, ptr, nbytes, lps=1):
        return kdn.lib().kdn_store_to_host(C.byref(cd), bt.data_ptr(), bt.numel(), 0, 100, C.byref(chunk.desc),
                                           ptr, nbytes, lps, None)
    assert store_to_host(pageable, staging.data_ptr(), need) == kdn.EINVAL
    assert store_to_host(pinned, staging.data_ptr(), need - 1) == kdn.ESIZE
    assert store_to_host(pinned, staging.data_ptr() + 8, need) == kdn.EALIGN
    assert store_to_host(pinned, staging.data_ptr(), need, lps=0) == kdn.EINVAL
    assert store_to_host(pinned, staging.data_ptr(), need) == kdn.OK
    torch.cuda.synchronize()
    assert np.array_equal(pinned.data.numpy(), O.store(hc, np.arange(8, dtype=np.int32), 0, 100, INT8).data)
    with pytest.raises(kdn.KdnError) as e:
        kdn.kdn_compose_from_host([pageable], [0], dc, bt, 10000.0, staging, 1)
    assert e.value.status == kdn.EINVAL
    opts = kdn.LaunchOpts(-1)
    out = kdn.alloc_chunk(dc, 100, INT8)
    assert kdn.lib().kdn_store_chunk_opts(C.byref(cd), bt.data_ptr(), bt.numel(), 0, 100, C.byref(out.desc),
                                          C.byref(opts), None) == kdn.EINVAL


def lib_store_to_host_with_device_chunk(dc, a, fmt, staging, layers_per_stage):
    import ctypes as C
    dev_chunk = kdn.alloc_chunk(dc, 110, fmt)
    cd = dc.desc()
    bt = dev_table(a)
    st = kdn.lib().kdn_store_to_host(C.byref(cd), bt.data_ptr(), bt.numel(), 5, 110, C.byref(dev_chunk.desc),
                                     staging.data_ptr(), staging.numel(), layers_per_stage, None)
    if st != kdn.OK:
        raise kdn.KdnError(st, "kdn_store_to_host")


# ------------------------------------------------------------------ the streaming yardstick
@pytest.mark.parametrize("tile_kib,cap", [(4, 0), (4, 7), (8, 0), (32, 0), (32, 5), (72, 3), (256, 0)])
def test_probe_stream_moves_the_bytes_it_is_timed_for(tile_kib, cap):
    """The yardstick kernel is only worth timing if it moves what it says: every tile of the
    small buffer lands in the tile of the big one that the id names (each run of 4 KiB, 2 KiB
    for the 4 KiB tile, twice, the second copy with one bit pattern flipped per 16 bytes),
    nothing else is written, the reverse direction folds the two copies back, the write-only
    direction fills exactly the named tiles and the read-only one changes nothing."""
    tiles = 37
    run = 2048 if tile_kib == 4 else 4096                          # bytes of one run of the small buffer
    runs = tile_kib * 512 // run                                   # runs per small tile
    rng = np.random.default_rng(500 + tile_kib)
    ids_h = rng.permutation(64)[:tiles].astype(np.int32)
    small_h = rng.integers(0, 256, size=tiles * tile_kib * 512, dtype=np.uint8)
    small = torch.from_numpy(small_h).cuda()
    big = torch.full((64 * tile_kib * 1024,), 0xA5, dtype=torch.uint8, device="cuda")
    ids = torch.from_numpy(ids_h).cuda()
    kdn.kdn_probe_stream(small, big, tiles, ids, tile_kib, 0, cap)
    torch.cuda.synchronize()
    got = big.cpu().numpy().reshape(64, runs, 2, run)
    src = small_h.reshape(tiles, runs, run)
    flipped = src.copy().view(np.uint32).reshape(tiles, runs, run // 16, 4)
    flipped[..., 0] ^= np.uint32(0x80008000)
    flipped = flipped.view(np.uint8).reshape(tiles, runs, run)
    assert np.array_equal(got[ids_h, :, 0], src) and np.array_equal(got[ids_h, :, 1], flipped)
    untouched = np.setdiff1d(np.arange(64), ids_h)
    assert np.all(got[untouched] == 0xA5)
    back = torch.zeros_like(small)
    kdn.kdn_probe_stream(back, big, tiles, ids, tile_kib, 1, cap)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy().reshape(src.shape), src ^ flipped)
    # without ids tile i goes to tile i
    big.fill_(0)
    kdn.kdn_probe_stream(small, big, tiles, None, tile_kib, 0, cap)
    torch.cuda.synchronize()
    assert np.array_equal(big.cpu().numpy().reshape(64, runs, 2, run)[:tiles, :, 0], src)
    # write only: every named tile holds (tile, run, lane, mark) per 16 bytes, the others are untouched
    big.fill_(0xA5)
    keep = small.clone()
    kdn.kdn_probe_stream(small, big, tiles, ids, tile_kib, 2, cap)
    torch.cuda.synchronize()
    got = big.cpu().numpy().reshape(64, 2 * runs, run // 16, 16)
    want = np.empty((tiles, 2 * runs, run // 16, 4), dtype=np.uint32)
    want[..., 0] = ids_h[:, None, None]
    want[..., 1] = np.arange(2 * runs)[None, :, None]
    want[..., 2] = np.arange(run // 16)[None, None, :]
    want[..., 3] = 0x4B444E21
    assert np.array_equal(got[ids_h].view(np.uint32).reshape(want.shape), want)
    assert np.all(got[untouched] == 0xA5) and torch.equal(small, keep)
    # read only: nothing changes anywhere
    before = big.clone()
    kdn.kdn_probe_stream(small, big, tiles, ids, tile_kib, 3, cap)
    torch.cuda.synchronize()
    assert torch.equal(big, before) and torch.equal(small, keep)
    for bad_tile, bad_dir in ((2, 0), (tile_kib, 4), (tile_kib, -1)):   # below the smallest tile; no such direction
        with pytest.raises(kdn.KdnError) as e:
            kdn.kdn_probe_stream(small, big, tiles, ids, bad_tile, bad_dir, 0)
        assert e.value.status == kdn.EINVAL
