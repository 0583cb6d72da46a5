"""Pins of the CPU oracle against things other than itself (no GPU needed).

The paper prints no value for the store/load/compose path, so the oracle is
pinned by brute force on tagged inputs, float64 mathematics, closed forms and
invariants.  Each test names the part of the oracle a mistake would break.
"""
import os

import numpy as np
import pytest
import torch

from paper_2409_13761_amd import synth

RAW, INT8, INT4, FP8 = 0, 1, 2, 3


def bf16_bits_to_f64(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bf16_bits_to_f32(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def make_cache(oracle, seed, L, nb, bs, H, D):
    k = synth.normal_bf16(seed, (L, nb, bs, H, D), stream=10)
    v = synth.normal_bf16(seed, (L, nb, bs, H, D), stream=11)
    return oracle.PagedCache(k, v)


# --------------------------------------------------------------------------- bf16
def test_bf16_widen_is_exact_shift(oracle):
    bits = np.arange(0, 65536, dtype=np.uint32)
    finite = ((bits & 0x7F80) != 0x7F80)
    got = np.array([oracle.lib().kdno_bf16_to_f32(int(b)) for b in bits[finite][::37]], dtype=np.float32)
    want = (bits[finite][::37] << 16).view(np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_bf16_round_nearest_even_against_float64_grid(oracle):
    """Narrowing must pick the nearest point of the bf16 grid, ties to the even
    significand.  Reference: scale to the grid in float64 and use rint there.
    Inputs: every upper half-word with a set of lower half-words that covers
    both sides of, and exactly, the tie."""
    hi = np.arange(0, 65536, dtype=np.uint32)
    hi = hi[(hi & 0x7F80) != 0x7F80]                     # finite
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x4000, 0xC000,
                     0x1234, 0x8ACE, 0x7F00, 0x80FF], dtype=np.uint32)
    rng = np.random.default_rng(7)
    lows = np.concatenate([lows, rng.integers(0, 65536, size=52).astype(np.uint32)])
    u = (hi[:, None] << 16 | lows[None, :]).ravel()
    x32 = u.view(np.float32)
    got = bf16_bits_to_f64(oracle.f32_to_bf16(x32))

    x = x32.astype(np.float64)
    _, e = np.frexp(x)                                   # |x| = m * 2^e, m in [0.5, 1)
    e = np.maximum(e - 1, -126)                          # binade of a normal; denormals share -126
    ulp = np.ldexp(1.0, e - 7)                           # bf16 keeps 7 explicit significand bits
    want = np.rint(x / ulp) * ulp                        # np.rint is half-to-even
    want = np.where(np.abs(want) >= 2.0 ** 128, np.sign(x) * np.inf, want)
    assert np.array_equal(got, want)
    assert np.array_equal(np.signbit(got), np.signbit(x))


def test_bf16_matches_torch_cast_on_random_values(oracle):
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32),
                        (rng.standard_normal(1000) * 1e-39).astype(np.float32),
                        (rng.standard_normal(1000) * 1e38).astype(np.float32)])
    got = oracle.f32_to_bf16(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)


def test_bf16_nan_stays_nan(oracle):
    x = np.array([np.nan, -np.nan], dtype=np.float32)
    out = oracle.f32_to_bf16(x)
    assert np.all((out & 0x7F80) == 0x7F80) and np.all((out & 0x007F) != 0)


# ------------------------------------------------------- addressing / gather / scatter
def _tagged_cache(oracle, L, nb, bs, H, D, hi_pass):
    n = L * nb * bs * H * D
    idx = np.arange(n, dtype=np.int64)
    tags = ((idx >> 16) if hi_pass else (idx & 0xFFFF)).astype(np.uint16)
    k = tags.reshape(L, nb, bs, H, D).copy()
    v = (tags ^ np.uint16(0x5555)).reshape(L, nb, bs, H, D).copy()
    return oracle.PagedCache(k, v)


@pytest.mark.parametrize("hi_pass", [False, True])
def test_store_raw_gathers_the_addressed_rows(oracle, hi_pass):
    """Brute force over a tagged cache: tag = the element's own linear index."""
    L, nb, bs, H, D = 2, 40, 4, 3, 8
    cache = _tagged_cache(oracle, L, nb, bs, H, D, hi_pass)
    bt = synth.disjoint_block_tables(5, nb, [9])[0]
    t0, T = 6, 25                                        # starts and ends inside a block
    ch = oracle.store(cache, bt, t0, T, RAW)
    raw = ch.raw()
    for l in range(L):
        for side, base in enumerate((cache.k, cache.v)):
            for t in range(T):
                tok = t0 + t
                blk, slot = int(bt[tok // bs]), tok % bs
                for h in range(H):
                    for j in range(D):
                        assert raw[l, side, t, h, j] == base[l, blk, slot, h, j]


def test_load_raw_writes_each_destination_once_and_nothing_else(oracle):
    L, nb, bs, H, D = 2, 32, 4, 2, 8
    src = make_cache(oracle, 21, L, nb, bs, H, D)
    src_bt, dst_bt = synth.disjoint_block_tables(6, nb, [8, 7])
    T = 23
    ch = oracle.store(src, src_bt, 3, T, RAW)
    sentinel = np.uint16(0x7FC1)                          # a NaN pattern N(0,1) never yields
    dst = oracle.PagedCache(np.full_like(src.k, sentinel), np.full_like(src.v, sentinel))
    dest = 2
    oracle.load(ch, dst, dst_bt, dest)
    written = np.zeros((L, 2, nb, bs), dtype=bool)
    for side, (sb, db) in enumerate(((src.k, dst.k), (src.v, dst.v))):
        for l in range(L):
            for t in range(T):
                s_blk, s_slot = int(src_bt[(3 + t) // bs]), (3 + t) % bs
                d_blk, d_slot = int(dst_bt[(dest + t) // bs]), (dest + t) % bs
                assert np.array_equal(db[l, d_blk, d_slot], sb[l, s_blk, s_slot])
                assert not written[l, side, d_blk, d_slot]
                written[l, side, d_blk, d_slot] = True
    for side, db in enumerate((dst.k, dst.v)):
        untouched = db[~written[:, side]]
        assert np.all(untouched == sentinel)


def test_raw_store_then_load_is_identity_under_other_tables(oracle):
    L, nb, bs, H, D = 3, 64, 16, 2, 16
    src = make_cache(oracle, 22, L, nb, bs, H, D)
    a, b = synth.disjoint_block_tables(8, nb, [10, 10])
    ch = oracle.store(src, a, 0, 160, RAW)
    dst = make_cache(oracle, 23, L, nb, bs, H, D)
    oracle.load(ch, dst, b, 0)
    for base_s, base_d in ((src.k, dst.k), (src.v, dst.v)):
        assert np.array_equal(base_d[:, b], base_s[:, a])


def test_strided_cache_layout_is_honoured(oracle):
    """Same data seen through a layout with padded token and head strides."""
    import ctypes as C
    L, nb, bs, H, D = 2, 6, 4, 2, 8
    dense = make_cache(oracle, 24, L, nb, bs, H, D)
    pad = np.zeros((L, nb, bs, H + 1, D + 8), dtype=np.uint16)
    padv = np.zeros_like(pad)
    pad[:, :, :, :H, :D] = dense.k
    padv[:, :, :, :H, :D] = dense.v
    bt = np.array([4, 1, 5], dtype=np.int32)
    want = oracle.store(dense, bt, 1, 9, INT8)
    d = dense.desc()
    d.k, d.v = pad.ctypes.data, padv.ctypes.data
    hs = D + 8
    d.head_stride, d.token_stride = hs, (H + 1) * hs
    d.block_stride, d.layer_stride = bs * (H + 1) * hs, nb * bs * (H + 1) * hs
    got = np.zeros_like(want.data)
    rc = oracle.lib().kdno_store(C.byref(d), bt.ctypes.data, 3, 1, 9, INT8, got.ctypes.data, 0, L)
    assert rc == 0 and np.array_equal(got, want.data)


# ------------------------------------------------------------------- quantiser
def _rows(seed, n, D, scale_pow=0):
    return synth.normal_bf16(seed, (n, D), stream=20)


def test_golden_quantiser_rows(oracle):
    """Hand-worked rows from tests/golden/quantiser_rows.txt."""
    path = os.path.join(os.path.dirname(__file__), "golden", "quantiser_rows.txt")
    n = 0
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        xs, qs, sc = (p.strip() for p in line.split("|"))
        x = np.array([float(t) for t in xs.split()], dtype=np.float32)
        xb = torch.from_numpy(x).to(torch.bfloat16)
        assert np.array_equal(xb.float().numpy(), x), "golden inputs must be bf16-exact"
        q, s = oracle.quantise_row(xb.view(torch.int16).numpy().view(np.uint16))
        assert q.tolist() == [int(t) for t in qs.split()]
        assert float(s) == float(sc)
        n += 1
    assert n >= 5


def test_scale_is_amax_over_127_and_peak_code_is_127(oracle):
    D = 64
    rows = _rows(31, 400, D)
    for r in rows:
        x = bf16_bits_to_f64(r)
        q, s = oracle.quantise_row(r)
        amax = np.max(np.abs(x))
        # exact quotient in float64, one rounding to fp32 (innocuous double rounding: 53 >= 2*24+2)
        assert np.float32(s) == np.float32(amax / 127.0)
        assert abs(float(s) * 127.0 - amax) <= np.spacing(np.float32(amax))
        assert np.max(np.abs(q.astype(np.int32))) == 127
        assert q[np.argmax(np.abs(x))] == (127 if x[np.argmax(np.abs(x))] > 0 else -127)
        assert q.min() >= -127


def test_codes_equal_mathematical_rounding_except_at_ties(oracle):
    """Every finite bf16 value as x, for several amax: code == nearbyint(127 x / amax)
    evaluated in float64, except where that value sits within 2^-16 of a tie (the
    room fp32 rounding of 127/amax and of the product can use)."""
    allb = np.arange(0, 65536, dtype=np.uint32)
    allb = allb[(allb & 0x7F80) != 0x7F80].astype(np.uint16)
    vals = bf16_bits_to_f64(allb)
    n_slop = 0
    for amax_bits in (0x3F80, 0x4049, 0x4123, 0x3DCC, 0x0880, 0x7E12, 0x40FE):
        amax = float(bf16_bits_to_f64(np.array([amax_bits]))[0])
        sel = np.abs(vals) <= amax
        xb = allb[sel]
        D = 128
        pad = (-len(xb)) % (D - 1)
        xb = np.concatenate([xb, np.zeros(pad, dtype=np.uint16)])
        for row in xb.reshape(-1, D - 1):
            r = np.concatenate([[np.uint16(amax_bits)], row])       # pin the row's amax
            q, s = oracle.quantise_row(r)
            exact = 127.0 * bf16_bits_to_f64(r) / amax
            want = np.rint(exact)
            bad = q.astype(np.float64) != want
            near_tie = np.abs(np.abs(exact - np.floor(exact)) - 0.5) < 2.0 ** -16
            assert not np.any(bad & ~near_tie)
            n_slop += int(np.sum(bad))
    assert n_slop < 2000


def test_quantisation_error_within_half_a_step(oracle):
    D = 128
    rows = _rows(33, 500, D)
    for r in rows:
        x = bf16_bits_to_f64(r)
        q, s = oracle.quantise_row(r)
        y = oracle.dequantise_row(q, s).astype(np.float64)
        assert np.all(np.abs(x - y) <= float(s) * (0.5 + 1e-4))
        # dequantisation is one fp32 product
        assert np.array_equal(y.astype(np.float32), (q.astype(np.float64) * float(s)).astype(np.float32))


def test_zero_and_tiny_rows(oracle):
    D = 32
    z = np.zeros(D, dtype=np.uint16)
    z[3] = 0x8000                                        # -0.0
    q, s = oracle.quantise_row(z)
    assert s == 0 and not q.any()
    assert np.all(oracle.dequantise_row(q, s) == 0)
    tiny = np.zeros(D, dtype=np.uint16)
    tiny[0] = 0x0340                                     # 2^-121 * 1.5 -> kept
    q, s = oracle.quantise_row(tiny)
    assert q[0] == 127 and s > 0 and np.isfinite(127.0 / bf16_bits_to_f64(tiny[:1])[0])
    below = np.zeros(D, dtype=np.uint16)
    below[0] = 0x02FF                                    # just under 2^-121 -> flushed row
    q, s = oracle.quantise_row(below)
    assert s == 0 and not q.any()
    # scale that is an fp32 denormal (amax = 127e-38) still round-trips to within half a step
    den = torch.tensor([1.27e-36, -0.5e-36, 1e-37, 0.0] * 8).to(torch.bfloat16)
    db = den.view(torch.int16).numpy().view(np.uint16)
    q, s = oracle.quantise_row(db)
    assert 0 < float(s) < 1.1754944e-38
    y = oracle.dequantise_row(q, s).astype(np.float64)
    assert np.all(np.abs(bf16_bits_to_f64(db) - y) <= float(s) * 0.5001)


# ------------------------------------------------------------------- int4, groups of 32
def unpack_nibbles(packed):
    """Independent decode: even element in the low nibble, two's complement."""
    lo = (packed & 0xF).astype(np.int8)
    hi = (packed >> 4).astype(np.int8)
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    return np.stack([lo, hi], axis=-1).reshape(packed.shape[:-1] + (packed.shape[-1] * 2,))


def test_golden_int4_groups(oracle):
    """Hand-worked groups from tests/golden/int4_groups.txt (first 8 elements of a group
    are listed, the other 24 are zero)."""
    path = os.path.join(os.path.dirname(__file__), "golden", "int4_groups.txt")
    n = 0
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        xs, bs_, sc = (p.strip() for p in line.split("|"))
        x = np.zeros(32, dtype=np.float32)
        vals = [float(t) for t in xs.split()]
        x[:len(vals)] = vals
        xb = torch.from_numpy(x).to(torch.bfloat16)
        assert np.array_equal(xb.float().numpy(), x)
        packed, s = oracle.quantise_row_int4(xb.view(torch.int16).numpy().view(np.uint16))
        want = [int(t, 16) for t in bs_.split()]
        assert packed[:len(want)].tolist() == want and not packed[len(want):].any()
        assert float(s[0]) == float(sc)
        n += 1
    assert n >= 4


def test_int4_codes_scales_and_error_bound(oracle):
    D = 128
    rows = _rows(35, 300, D)
    for r in rows:
        x = bf16_bits_to_f64(r)
        packed, s = oracle.quantise_row_int4(r)
        q = unpack_nibbles(packed).astype(np.float64)
        xg, qg = x.reshape(-1, 32), q.reshape(-1, 32)
        amax = np.max(np.abs(xg), axis=1)
        assert np.array_equal(s, (amax / 7.0).astype(np.float32))       # exact quotient, one rounding
        assert np.all(np.max(np.abs(qg), axis=1) == 7) and q.min() >= -7
        exact = 7.0 * xg / amax[:, None]
        near_tie = np.abs(np.abs(exact - np.floor(exact)) - 0.5) < 2.0 ** -16
        assert not np.any((qg != np.rint(exact)) & ~near_tie)
        y = oracle.dequantise_row_int4(packed, s).astype(np.float64)
        assert np.all(np.abs(x - y) <= np.repeat(s.astype(np.float64), 32) * (0.5 + 1e-4))
        assert np.array_equal(y.astype(np.float32), (q * np.repeat(s.astype(np.float64), 32)).astype(np.float32))


def test_int4_groups_are_independent_and_tiny_groups_flush(oracle):
    D = 64
    r = _rows(36, 1, D)[0].copy()
    p0, s0 = oracle.quantise_row_int4(r)
    r2 = r.copy()
    r2[32:] = _rows(37, 1, D)[0][32:]
    p1, s1 = oracle.quantise_row_int4(r2)
    assert np.array_equal(p0[:16], p1[:16]) and s0[0] == s1[0] and not np.array_equal(p0[16:], p1[16:])
    z = np.zeros(D, dtype=np.uint16)
    z[5] = 0x8000
    z[40] = 0x02FF                       # below 2^-121: the group is flushed
    p, s = oracle.quantise_row_int4(z)
    assert not p.any() and not s.any()
    z[41] = 0x0300                       # exactly 2^-121: kept
    p, s = oracle.quantise_row_int4(z)
    assert s[0] == 0 and s[1] > 0 and unpack_nibbles(p)[41] == 7


def test_int4_every_bf16_value_against_mathematical_rounding(oracle):
    allb = np.arange(0, 65536, dtype=np.uint32)
    allb = allb[(allb & 0x7F80) != 0x7F80].astype(np.uint16)
    vals = bf16_bits_to_f64(allb)
    n_slop = 0
    for amax_bits in (0x3F80, 0x40E0, 0x4049, 0x0880, 0x7E12):
        amax = float(bf16_bits_to_f64(np.array([amax_bits]))[0])
        xb = allb[np.abs(vals) <= amax]
        xb = np.concatenate([xb, np.zeros((-len(xb)) % 31, dtype=np.uint16)])
        for grp in xb.reshape(-1, 31):
            g = np.concatenate([[np.uint16(amax_bits)], grp])
            packed, s = oracle.quantise_row_int4(g)
            q = unpack_nibbles(packed).astype(np.float64)
            exact = 7.0 * bf16_bits_to_f64(g) / amax
            bad = q != np.rint(exact)
            near_tie = np.abs(np.abs(exact - np.floor(exact)) - 0.5) < 2.0 ** -16
            assert not np.any(bad & ~near_tie)
            n_slop += int(bad.sum())
    assert n_slop < 500


# ------------------------------------------------------------------- fp8 (e4m3), row scale
def test_e4m3_decode_of_every_code_matches_torch(oracle):
    codes = np.arange(256, dtype=np.uint8)
    got = oracle.e4m3_to_f32(codes)
    want = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[~np.isnan(got)].view(np.uint32), want[~np.isnan(want)].view(np.uint32))
    assert got[0x7E] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6


def test_e4m3_encode_matches_torch_below_saturation(oracle):
    """torch's CPU cast to float8_e4m3fn is the independent reference inside the finite
    range; above it torch gives NaN where this format saturates (never reached by the
    quantiser, whose products stay below 448(1 + 2^-24))."""
    rng = np.random.default_rng(31)
    grid = oracle.e4m3_to_f32(np.arange(0, 0x7F, dtype=np.uint8)).astype(np.float64)
    mids = (grid[:-1] + grid[1:]) / 2                       # every tie
    x = np.concatenate([grid, mids, np.nextafter(mids.astype(np.float32), np.float32(0)),
                        np.nextafter(mids.astype(np.float32), np.float32(1000)),
                        rng.uniform(-448, 448, 20000), rng.standard_normal(20000) * 0.01,
                        [448.0, 448.00003, -448.00003, 2.0 ** -10, 2.0 ** -10 * 1.0001, 0.0, -0.0]]).astype(np.float32)
    x = np.concatenate([x, -x])
    got = oracle.f32_to_e4m3(x)
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    inside = np.abs(x) <= 448.0
    assert np.array_equal(got[inside], want[inside])
    assert np.all((got[~inside] & 0x7F) == 0x7E)
    # saturation starts right above 448, not at the next binade: 465..479 would round to the NaN code
    over = np.array([464.0, 465.0, 479.0, 480.0, 1e9, -1e9, np.inf, -470.0], dtype=np.float32)
    assert oracle.f32_to_e4m3(over).tolist() == [0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0x7E, 0xFE]


def test_fp8_rows(oracle):
    D = 128
    rows = _rows(38, 300, D)
    for r in rows:
        x = bf16_bits_to_f64(r)
        q, s = oracle.quantise_row_fp8(r)
        amax = np.max(np.abs(x))
        assert np.float32(s) == np.float32(amax / 448.0)
        assert (q[np.argmax(np.abs(x))] & 0x7F) == 0x7E                 # the peak maps to +-448
        y = oracle.dequantise_row_fp8(q, s).astype(np.float64)
        # relative error of a 3-bit mantissa: half a step of 1/8 at most, plus the subnormal floor
        assert np.all(np.abs(x - y) <= np.abs(x) * (1 / 16 + 1e-3) + float(s) * 2.0 ** -10 * 1.01)
        # codes are the torch cast of the fp32 products
        inv = np.float32(448.0) / np.float32(amax)
        prod = (bf16_bits_to_f32(r) * inv).astype(np.float32)
        want = torch.from_numpy(np.minimum(np.abs(prod), 448.0) * np.sign(prod)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(q, want)
    z = np.zeros(D, dtype=np.uint16)
    z[3] = 0x0400                        # 2^-119 * ... below? 0x0400 = 2^-119: kept
    q, s = oracle.quantise_row_fp8(z)
    assert s > 0 and (q[3] & 0x7F) == 0x7E
    z[3] = 0x03FF                        # just under 2^-119: flushed
    q, s = oracle.quantise_row_fp8(z)
    assert s == 0 and not q.any()


# --------------------------------------------------------------------- rotation
def test_rope_table_values(oracle):
    for base, D, d in ((10000.0, 64, 256), (500000.0, 128, 24576), (10000.0, 128, -777)):
        cs = oracle.rope_table(base, D, d).astype(np.float64)
        j = np.arange(D // 2, dtype=np.float64)
        theta = base ** (-2.0 * j / D)
        assert theta[0] == 1.0
        assert np.isclose(theta[-1], base ** (-(D - 2) / D), rtol=1e-15)
        assert np.allclose(cs[:, 0], np.cos(d * theta), rtol=0, atol=6.1e-8)
        assert np.allclose(cs[:, 1], np.sin(d * theta), rtol=0, atol=6.1e-8)
        assert np.allclose(cs[:, 0] ** 2 + cs[:, 1] ** 2, 1.0, atol=2.0 ** -22)


def test_rope_tables_compose_like_complex_numbers(oracle):
    base, D = 500000.0, 128
    z = lambda d: (lambda t: t[:, 0] + 1j * t[:, 1])(oracle.rope_table(base, D, d).astype(np.float64))
    assert np.allclose(z(300) * z(212), z(512), atol=1e-6)
    assert np.allclose(z(4096) * z(-4096), 1.0, atol=1e-6)
    assert np.allclose(z(-5), np.conj(z(5)), atol=1e-7)


def test_single_pair_is_a_plane_rotation(oracle):
    """D = 2: theta_0 = 1 for any base, so the shift is a 2-D rotation by d radians."""
    rng = np.random.default_rng(5)
    for base in (10000.0, 3.0):
        for d in (1, 2, -3, 10, 100):
            cs = oracle.rope_table(base, 2, d)
            a, b = rng.standard_normal(2)
            y = oracle.rotate_row(np.array([a, b], dtype=np.float32), cs)
            w = complex(np.float32(a), np.float32(b)) * np.exp(1j * d)
            assert abs(y[0] - w.real) < 1e-6 and abs(y[1] - w.imag) < 1e-6


def test_shift_of_key_at_p_equals_key_at_p_plus_d(oracle):
    """R(d) K(p) = K(p+d) with half-split pairing (j, j + D/2)."""
    rng = np.random.default_rng(9)
    for base, D in ((10000.0, 64), (500000.0, 128)):
        half = D // 2
        theta = base ** (-2.0 * np.arange(half) / D)
        for p, d in ((0, 17), (100, 256), (511, 3584), (9000, -8192), (5, 24576)):
            k_raw = rng.standard_normal(D)
            zr = k_raw[:half] + 1j * k_raw[half:]
            kp = zr * np.exp(1j * p * theta)
            kpd = zr * np.exp(1j * (p + d) * theta)
            want = np.concatenate([kpd.real, kpd.imag])
            x32 = np.concatenate([kp.real, kp.imag]).astype(np.float32)
            cs = oracle.rope_table(base, D, d)
            got = oracle.rotate_row(x32, cs).astype(np.float64)
            norm = np.abs(kpd)
            assert np.all(np.abs(got - want) <= 1e-5 * np.concatenate([norm, norm]) + 1e-7)
            # bf16 in, bf16 out: within 2 bf16 ulp of the pair norm
            xb = oracle.f32_to_bf16(x32)
            gotb = bf16_bits_to_f64(oracle.f32_to_bf16(
                oracle.rotate_row(bf16_bits_to_f32(xb), cs)))
            ulp = 2.0 ** (np.floor(np.log2(np.maximum(norm, 1e-30))) - 7)
            assert np.all(np.abs(gotb - want) <= 2.0 * np.concatenate([ulp, ulp]) + 1e-6)


def test_rotation_keeps_pair_norm_and_inverts(oracle):
    rng = np.random.default_rng(10)
    D = 128
    x = rng.standard_normal(D).astype(np.float32)
    cs = oracle.rope_table(500000.0, D, 1234)
    y = oracle.rotate_row(x, cs)
    n0 = np.hypot(x[:64].astype(np.float64), x[64:])
    n1 = np.hypot(y[:64].astype(np.float64), y[64:])
    assert np.allclose(n0, n1, rtol=3e-7)
    back = oracle.rotate_row(y, oracle.rope_table(500000.0, D, -1234))
    assert np.allclose(back, x, atol=5e-7 * np.max(n0))
    # a wrong sign on either sine term breaks this: rotating (1, 0) by +90 degrees gives (0, 1)
    quarter = np.array([[0.0, 1.0]], dtype=np.float32)
    assert oracle.rotate_row(np.array([1.0, 0.0], dtype=np.float32), quarter).tolist() == [0.0, 1.0]
    assert oracle.rotate_row(np.array([0.0, 1.0], dtype=np.float32), quarter).tolist() == [-1.0, 0.0]


# ----------------------------------------------------------------------- compose
def _setup_compose(oracle, fmt, seed=41):
    L, nb, bs, H, D = 2, 48, 8, 2, 64
    src = make_cache(oracle, seed, L, nb, bs, H, D)
    t1, t2, t3, dst_bt = synth.disjoint_block_tables(seed, nb, [4, 3, 5, 12])
    chunks = [oracle.store(src, t1, 0, 29, fmt), oracle.store(src, t2, 2, 20, fmt),
              oracle.store(src, t3, 5, 33, fmt)]
    return src, chunks, dst_bt


@pytest.mark.parametrize("fmt", [RAW, INT8, INT4, FP8])
def test_zero_offset_compose_is_concatenation(oracle, fmt):
    src, chunks, dst_bt = _setup_compose(oracle, fmt)
    a = make_cache(oracle, 77, src.L, src.nb, src.bs, src.H, src.D)
    b = a.copy()
    oracle.compose(chunks, [0, 0, 0], a, dst_bt, 10000.0, dest=3)
    S = 3
    for c in chunks:
        oracle.load(c, b, dst_bt, S)
        S += c.T
    assert np.array_equal(a.k, b.k) and np.array_equal(a.v, b.v)
    # and the concatenation holds what an independent dequantise-and-place gives
    bs = src.bs
    S = 3
    for c in chunks:
        if fmt == RAW:
            rows = c.raw()
        else:
            if fmt == INT8:
                y = c.codes().astype(np.float32) * c.scales()[..., None]
            elif fmt == FP8:
                y = torch.from_numpy(c.codes().copy()).view(torch.float8_e4m3fn).float().numpy() * c.scales()[..., None]
            else:
                y = unpack_nibbles(c.packed4()).astype(np.float32) * np.repeat(c.scales4(), 32, axis=-1)
            rows = torch.from_numpy(y).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        for t in range(c.T):
            blk, slot = int(dst_bt[(S + t) // bs]), (S + t) % bs
            assert np.array_equal(a.k[:, blk, slot], rows[:, 0, t])
            assert np.array_equal(a.v[:, blk, slot], rows[:, 1, t])
        S += c.T


@pytest.mark.parametrize("fmt", [RAW, INT8, INT4, FP8])
def test_compose_equals_independent_single_chunk_composes(oracle, fmt):
    src, chunks, dst_bt = _setup_compose(oracle, fmt, seed=42)
    offs = [0, 29, -7]
    a = make_cache(oracle, 78, src.L, src.nb, src.bs, src.H, src.D)
    b = a.copy()
    before = a.copy()
    oracle.compose(chunks, offs, a, dst_bt, 10000.0)
    S = 0
    for c, d in zip(chunks, offs):
        oracle.compose([c], [d], b, dst_bt, 10000.0, dest=S)
        S += c.T
    assert np.array_equal(a.k, b.k) and np.array_equal(a.v, b.v)
    # V ignores offsets; K of the shifted chunks does change; blocks outside the table do not
    c = before.copy()
    oracle.compose(chunks, [0, 0, 0], c, dst_bt, 10000.0)
    assert np.array_equal(a.v, c.v)
    assert not np.array_equal(a.k, c.k)
    outside = np.setdiff1d(np.arange(src.nb), dst_bt)
    assert np.array_equal(a.k[:, outside], before.k[:, outside])
    total = sum(ch.T for ch in chunks)
    last_blk, used = int(dst_bt[total // src.bs]), total % src.bs
    assert np.array_equal(a.k[:, last_blk, used:], before.k[:, last_blk, used:])


def test_composed_keys_follow_the_rotation_of_the_dequantised_rows(oracle):
    """K rows of a shifted int8 chunk = bf16(rotate(q * scale)), evaluated with float64
    complex arithmetic and compared within one bf16 step; V rows = bf16(q * scale)."""
    src, chunks, dst_bt = _setup_compose(oracle, INT8, seed=43)
    dst = make_cache(oracle, 79, src.L, src.nb, src.bs, src.H, src.D)
    base, d = 10000.0, 300
    oracle.compose([chunks[2]], [d], dst, dst_bt, base)
    c = chunks[2]
    D, half, bs = src.D, src.D // 2, src.bs
    theta = base ** (-2.0 * np.arange(half) / D)
    y = c.codes().astype(np.float64) * c.scales()[..., None].astype(np.float64)
    z = (y[:, 0, :, :, :half] + 1j * y[:, 0, :, :, half:]) * np.exp(1j * d * theta)
    want_k = np.concatenate([z.real, z.imag], axis=-1)
    for t in range(c.T):
        blk, slot = int(dst_bt[t // bs]), t % bs
        got = bf16_bits_to_f64(dst.k[:, blk, slot])
        w = want_k[:, t]
        step = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(w), 1e-30))) - 7)
        assert np.all(np.abs(got - w) <= 0.51 * step + 1e-6)
        gv = bf16_bits_to_f64(dst.v[:, blk, slot])
        wv = y[:, 1, t]
        stepv = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(wv), 1e-30))) - 7)
        assert np.all(np.abs(gv - wv) <= 0.5 * stepv)


def test_slices_of_a_stored_chunk(oracle):
    """A token view (parent length as stride) places the same rows as a chunk stored
    from that token range alone."""
    L, nb, bs, H, D = 2, 32, 4, 2, 16
    src = make_cache(oracle, 44, L, nb, bs, H, D)
    a, b = synth.disjoint_block_tables(44, nb, [10, 10])
    whole = oracle.store(src, a, 0, 40, INT8)
    part = oracle.store(src, a, 12, 17, INT8)
    d1 = make_cache(oracle, 80, L, nb, bs, H, D)
    d2 = d1.copy()
    oracle.compose([whole.slice(12, 17)], [64], d1, b, 10000.0, dest=5)
    oracle.compose([part], [64], d2, b, 10000.0, dest=5)
    assert np.array_equal(d1.k, d2.k) and np.array_equal(d1.v, d2.v)
    assert np.array_equal(whole.codes()[:, :, 12:29], part.codes())
    assert np.array_equal(whole.scales()[:, :, 12:29], part.scales())


def test_layer_ranges_partition_the_work(oracle):
    L, nb, bs, H, D = 4, 16, 4, 2, 16
    src = make_cache(oracle, 45, L, nb, bs, H, D)
    a, b = synth.disjoint_block_tables(45, nb, [5, 5])
    whole = oracle.store(src, a, 0, 20, INT8)
    parts = oracle.store(src, a, 0, 20, INT8, layers=(0, 1))
    oracle.store(src, a, 0, 20, INT8, layers=(1, 4), out=parts)
    assert np.array_equal(whole.data, parts.data)


def test_bad_ranges_are_refused(oracle):
    L, nb, bs, H, D = 1, 8, 4, 1, 16
    src = make_cache(oracle, 46, L, nb, bs, H, D)
    bt = np.arange(4, dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.store(src, bt, 10, 7, RAW)                # runs past the table
    ch = oracle.store(src, bt, 0, 16, RAW)
    with pytest.raises(ValueError):
        oracle.load(ch, src, bt, 1)
    with pytest.raises(ValueError):
        oracle.load(ch, src, np.array([0, 1, 2, 99], dtype=np.int32), 0)   # block id out of range


# ------------------------------------------------------------- RoPE variants, patching
def test_interleaved_pairs_are_complex_multiplications(oracle):
    """Pair (2j, 2j+1) as a complex number times exp(i d theta_j)."""
    rng = np.random.default_rng(21)
    for base, D, d in ((10000.0, 64, 100), (500000.0, 128, -3000)):
        x = rng.standard_normal(D).astype(np.float32)
        cs = oracle.rope_table_spec(base, None, D, d)
        y = oracle.rotate_row_spec(x, D, oracle.PAIR_INTERLEAVED, cs).astype(np.float64)
        theta = base ** (-2.0 * np.arange(D // 2) / D)
        z = (x[0::2].astype(np.float64) + 1j * x[1::2]) * np.exp(1j * d * theta)
        assert np.allclose(y[0::2], z.real, atol=2e-6) and np.allclose(y[1::2], z.imag, atol=2e-6)
        # and shifting K(p) by d gives K(p+d) in this pairing too
        k_raw = rng.standard_normal(D)
        zr = k_raw[0::2] + 1j * k_raw[1::2]
        kp, kpd = zr * np.exp(1j * 17 * theta), zr * np.exp(1j * (17 + d) * theta)
        xin = np.empty(D, dtype=np.float32)
        xin[0::2], xin[1::2] = kp.real, kp.imag
        got = oracle.rotate_row_spec(xin, D, oracle.PAIR_INTERLEAVED, cs).astype(np.float64)
        assert np.allclose(got[0::2], kpd.real, atol=1e-5) and np.allclose(got[1::2], kpd.imag, atol=1e-5)


def test_partial_rotary_rotates_the_leading_dims_only(oracle):
    rng = np.random.default_rng(22)
    D, rot, base, d = 128, 64, 10000.0, 77
    x = rng.standard_normal(D).astype(np.float32)
    cs = oracle.rope_table_spec(base, None, rot, d)
    for pairing in (oracle.PAIR_HALF_SPLIT, oracle.PAIR_INTERLEAVED):
        y = oracle.rotate_row_spec(x, rot, pairing, cs)
        assert np.array_equal(y[rot:], x[rot:])
        # the rotated part is what a full rotation of a rot-wide row gives (theta from rot, not D)
        small = oracle.rotate_row_spec(x[:rot].copy(), rot, pairing, cs)
        assert np.array_equal(y[:rot], small)
        assert not np.array_equal(y[:rot], x[:rot])
    theta = base ** (-2.0 * np.arange(rot // 2) / rot)
    assert np.allclose(cs[:, 0], np.cos(d * theta), atol=6.1e-8)
    # half-split with rot_dim == D is the plain rotation, bit for bit
    full = oracle.rope_table(base, D, d)
    assert np.array_equal(oracle.rope_table_spec(base, None, D, d), full)
    assert np.array_equal(oracle.rotate_row_spec(x, D, oracle.PAIR_HALF_SPLIT, full), oracle.rotate_row(x, full))


def test_explicit_frequencies(oracle):
    D, d = 64, 123
    base = 10000.0
    freq = np.array([base ** (-(2.0 * j) / D) for j in range(D // 2)])
    assert np.array_equal(oracle.rope_table_spec(base, freq, D, d), oracle.rope_table(base, D, d))
    scaled = freq / np.where(np.arange(D // 2) >= 16, 8.0, 1.0)        # low frequencies slowed down
    cs = oracle.rope_table_spec(base, scaled, D, d).astype(np.float64)
    assert np.allclose(cs[:, 0], np.cos(d * scaled), atol=6.1e-8)
    assert np.allclose(cs[:, 1], np.sin(d * scaled), atol=6.1e-8)


@pytest.mark.parametrize("fmt", [RAW, INT8, INT4])
def test_compose_spec_matches_row_wise_rotation(oracle, fmt):
    """compose with a variant = dequantise, rotate each K row with rotate_row_spec, round, place."""
    src, chunks, dst_bt = _setup_compose(oracle, fmt, seed=47)
    D, bs = src.D, src.bs
    freq = 10000.0 ** (-2.0 * np.arange(16) / 32) / 3.0
    for pairing, rot, inv_freq in ((oracle.PAIR_INTERLEAVED, 0, None), (oracle.PAIR_HALF_SPLIT, 32, freq),
                                   (oracle.PAIR_INTERLEAVED, 32, None)):
        dst = make_cache(oracle, 81, src.L, src.nb, src.bs, src.H, src.D)
        before = dst.copy()
        d = 45
        oracle.compose_spec([chunks[0]], [d], dst, dst_bt, 10000.0, inv_freq=inv_freq, rot_dim=rot,
                            pairing=pairing, dest=2)
        c = chunks[0]
        if fmt == RAW:
            y = bf16_bits_to_f32(c.raw())
        elif fmt == INT8:
            y = c.codes().astype(np.float32) * c.scales()[..., None]
        else:
            y = unpack_nibbles(c.packed4()).astype(np.float32) * np.repeat(c.scales4(), 32, axis=-1)
        cs = oracle.rope_table_spec(10000.0, inv_freq, rot or D, d)
        for t in range(c.T):
            blk, slot = int(dst_bt[(2 + t) // bs]), (2 + t) % bs
            for l in range(src.L):
                for h in range(src.H):
                    want_k = oracle.f32_to_bf16(oracle.rotate_row_spec(y[l, 0, t, h], rot or D, pairing, cs))
                    assert np.array_equal(dst.k[l, blk, slot, h], want_k)
                    assert np.array_equal(dst.v[l, blk, slot, h], oracle.f32_to_bf16(y[l, 1, t, h]))
        outside = np.setdiff1d(np.arange(src.nb), dst_bt)
        assert np.array_equal(dst.k[:, outside], before.k[:, outside])


def test_patch_rows_overwrites_exactly_the_named_tokens(oracle):
    L, nb, bs, H, D = 2, 16, 4, 2, 8
    cache = make_cache(oracle, 48, L, nb, bs, H, D)
    before = cache.copy()
    bt = synth.disjoint_block_tables(48, nb, [6])[0]
    tokens = np.array([3, 0, 17, 22, 9], dtype=np.int32)
    rows = synth.normal_bf16(49, (L, 2, len(tokens), H, D))
    oracle.patch_rows(rows, tokens, cache, bt)
    touched = np.zeros((nb, bs), dtype=bool)
    for i, t in enumerate(tokens):
        blk, slot = int(bt[t // bs]), t % bs
        touched[blk, slot] = True
        assert np.array_equal(cache.k[:, blk, slot], rows[:, 0, i])
        assert np.array_equal(cache.v[:, blk, slot], rows[:, 1, i])
    assert np.array_equal(cache.k[:, ~touched], before.k[:, ~touched])
    assert np.array_equal(cache.v[:, ~touched], before.v[:, ~touched])
    with pytest.raises(ValueError):
        oracle.patch_rows(rows, np.array([3, 0, 17, 24, 9]), cache, bt)     # token 24 is past the table


@pytest.mark.parametrize("fmt", [RAW, INT8, INT4])
def test_store_of_a_token_list(oracle, fmt):
    """Row t of the chunk is request token tokens[t]: raw rows by brute force over a
    tagged cache, quantised rows equal to the quantiser applied to those rows."""
    L, nb, bs, H, D = 2, 40, 4, 3, 32
    cache = _tagged_cache(oracle, L, nb, bs, H, D, False) if fmt == RAW else make_cache(oracle, 50, L, nb, bs, H, D)
    bt = synth.disjoint_block_tables(50, nb, [9])[0]
    tokens = np.array([35, 0, 7, 8, 22, 21, 3], dtype=np.int32)
    ch = oracle.store_tokens(cache, bt, tokens, fmt)
    assert ch.Tp == len(tokens)
    for l in range(L):
        for side, base in enumerate((cache.k, cache.v)):
            for i, tok in enumerate(tokens):
                row = base[l, int(bt[tok // bs]), tok % bs]            # [H][D]
                for h in range(H):
                    if fmt == RAW:
                        assert np.array_equal(ch.raw()[l, side, i, h], row[h])
                    elif fmt == INT8:
                        q, s_ = oracle.quantise_row(row[h])
                        assert np.array_equal(ch.codes()[l, side, i, h], q) and ch.scales()[l, side, i, h] == s_
                    else:
                        pk, s_ = oracle.quantise_row_int4(row[h])
                        assert np.array_equal(ch.packed4()[l, side, i, h], pk)
                        assert np.array_equal(ch.scales4()[l, side, i, h], s_)
    with pytest.raises(ValueError):
        oracle.store_tokens(cache, bt, np.array([1, 36]), fmt)          # 36 is past the table


# ------------------------------------------------- the quantised store, row by row
def _quantise(oracle, fmt, row):
    """(codes, scales) of one source row through the row quantiser of the format."""
    if fmt == INT8:
        return oracle.quantise_row(row)
    if fmt == FP8:
        return oracle.quantise_row_fp8(row)
    return oracle.quantise_row_int4(row)


@pytest.mark.parametrize("fmt", [INT8, INT4, FP8])
def test_quantised_store_puts_each_source_row_and_its_scale_in_its_own_slot(oracle, fmt):
    """Which source row feeds which stored row and which scale slot: for a ragged token
    range over a shuffled table, row (l, side, t, h) of the chunk holds the quantised
    row cache[l, bt[(t0+t)//bs], (t0+t)%bs, h], codes and scale(s) alike.  The row
    quantisers are pinned on their own above; this pins the indexing around them."""
    L, nb, bs, H, D = 3, 40, 4, 3, 64
    cache = make_cache(oracle, 51, L, nb, bs, H, D)
    bt = synth.disjoint_block_tables(51, nb, [9])[0]
    t0, T = 6, 27                                        # starts and ends inside a block
    ch = oracle.store(cache, bt, t0, T, fmt)
    assert ch.Tp == T and ch.data.nbytes == L * 2 * T * H * (D // 2 + D // 8 if fmt == INT4 else D + 4)
    seen_rows = set()
    for l in range(L):
        for side, base in enumerate((cache.k, cache.v)):
            for t in range(T):
                tok = t0 + t
                rows = base[l, int(bt[tok // bs]), tok % bs]               # [H][D]
                for h in range(H):
                    q, s = _quantise(oracle, fmt, rows[h])
                    if fmt == INT4:
                        assert np.array_equal(ch.packed4()[l, side, t, h], q)
                        assert np.array_equal(ch.scales4()[l, side, t, h], s)
                    else:
                        assert np.array_equal(ch.codes()[l, side, t, h], q)
                        assert ch.scales()[l, side, t, h] == s
                    seen_rows.add(q.tobytes())
    # the rows are distinguishable: a permuted placement could not pass by coincidence
    assert len(seen_rows) == L * 2 * T * H


@pytest.mark.parametrize("fmt", [INT8, INT4])
def test_store_then_load_is_within_half_a_step_of_the_source(oracle, fmt):
    """The round trip of a store: the dequantised value of every stored element lies
    within half a quantisation step of the SOURCE element it came from (step taken in
    float64 from the source row's own maximum, not from the chunk), and what a load
    into another table writes is that value rounded once more to bf16."""
    L, nb, bs, H, D = 2, 48, 8, 2, 64
    src = make_cache(oracle, 52, L, nb, bs, H, D)
    a, b = synth.disjoint_block_tables(52, nb, [6, 7])
    t0, T, dest = 5, 37, 3
    ch = oracle.store(src, a, t0, T, fmt)
    dst = make_cache(oracle, 53, L, nb, bs, H, D)
    oracle.load(ch, dst, b, dest)
    qmax, group = (127.0, D) if fmt == INT8 else (7.0, 32)
    if fmt == INT8:
        codes = ch.codes().astype(np.float64)
        scales = np.repeat(ch.scales().astype(np.float64)[..., None], D, axis=-1)
    else:
        codes = unpack_nibbles(ch.packed4()).astype(np.float64)
        scales = np.repeat(ch.scales4().astype(np.float64), 32, axis=-1)
    for side, (sb, db) in enumerate(((src.k, dst.k), (src.v, dst.v))):
        for t in range(T):
            s_blk, s_slot = int(a[(t0 + t) // bs]), (t0 + t) % bs
            d_blk, d_slot = int(b[(dest + t) // bs]), (dest + t) % bs
            x = bf16_bits_to_f64(sb[:, s_blk, s_slot])                     # [L][H][D], the source
            step = np.abs(x).reshape(L, H, D // group, group).max(-1) / qmax
            step = np.repeat(step, group, axis=-1).reshape(L, H, D)
            y = codes[:, side, t] * scales[:, side, t]
            assert np.all(np.abs(x - y) <= step * (0.5 + 1e-4))
            got = bf16_bits_to_f64(db[:, d_blk, d_slot])
            half_ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(y), 1e-300))) - 8)
            assert np.all(np.abs(got - y) <= half_ulp)
            assert np.all(np.abs(got - x) <= step * (0.5 + 1e-4) + half_ulp)
