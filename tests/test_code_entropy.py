"""Why there is no lossless stage behind the int8 codes (CPU only).

The paper's delivery module compresses KV by quantising and then encoding it (Sec. 3.2,
"KV-cache delivery").  Whether an encoding stage pays off on this library's stored form is an
empirical question about the codes the quantiser emits; this test answers it with the oracle's
store on the stand-in inputs and pins the figures the design notes quote: the zeroth-order
entropy of the codes (what any order-0 entropy coder could at best reach) and the size of a
byte-aligned packing (per group of 32 codes, the bit width of its largest code, one header
byte per group), per 128-element row against the 128 bytes of plain codes.
"""
import numpy as np
import torch

from paper_2409_13761_amd import synth

INT8 = 1


def _codes_of(oracle, kv_bits):
    """int8 codes [rows][128] of a cache filled with the given bf16 rows, through oracle.store."""
    L, nb, bs, H, D = kv_bits.shape
    cache = oracle.PagedCache(kv_bits, kv_bits.copy())
    ch = oracle.store(cache, np.arange(nb, dtype=np.int32), 0, nb * bs, INT8)
    return ch.codes()[:, 0].reshape(-1, D)


def _entropy_bits(codes):
    counts = np.bincount(codes.astype(np.int16).ravel() + 128, minlength=256).astype(np.float64)
    p = counts[counts > 0] / counts.sum()
    return float(-(p * np.log2(p)).sum())


def _packed_bytes_per_row(codes, group=32):
    """Each group of 32 codes stored at the width of its largest code (sign included), plus one
    header byte that names the width."""
    g = np.abs(codes.astype(np.int16)).reshape(codes.shape[0], -1, group).max(-1)     # [rows][groups]
    width = np.where(g == 0, 0, np.floor(np.log2(np.maximum(g, 1))) + 2)             # magnitude bits + sign
    return float((width * group / 8 + 1).sum(-1).mean())


def test_codes_of_gaussian_rows_leave_nothing_for_a_lossless_stage(oracle):
    kv = synth.normal_bf16(901, (1, 32, 16, 8, 128), stream=30)                      # 4096 rows of N(0,1)
    codes = _codes_of(oracle, kv)
    assert codes.shape == (4096, 128) and np.abs(codes).max() == 127
    h = _entropy_bits(codes)
    packed = _packed_bytes_per_row(codes)
    print("N(0,1): entropy %.3f bits per code, byte-aligned packing %.1f bytes per row" % (h, packed))
    assert 7.45 < h < 7.60                      # an ideal order-0 coder saves at most 6-7% of the code bytes
    assert 131.0 < packed < 132.5               # the byte-aligned packing is LARGER than the 128 plain bytes


def test_codes_of_heavy_tailed_channels_gain_little(oracle):
    """Channels with log-normal scales (sigma 1): a few large channels set the row maximum and the
    others use fewer levels.  The byte-aligned packing then gains about an eighth of the code
    bytes; an ideal order-0 entropy coder (variable-length rows, serial decode) about 40%: real,
    but below what the fixed-stride int4 form gives (80 bytes per row, scales included)."""
    base = synth.normal_bf16(902, (1, 32, 16, 8, 128), stream=31)
    x = (base.astype(np.uint32) << 16).view(np.float32)
    scale = np.exp(synth._rng(903, 32).standard_normal(128)).astype(np.float32)      # one scale per channel
    kv = torch.from_numpy(x * scale).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    codes = _codes_of(oracle, np.ascontiguousarray(kv))
    h = _entropy_bits(codes)
    packed = _packed_bytes_per_row(codes)
    print("log-normal channel scales: entropy %.3f bits per code, byte-aligned packing %.1f bytes per row" % (h, packed))
    assert 108.0 < packed < 117.0               # 112 of 128 bytes
    assert 4.5 < h < 5.2                        # 4.8 bits: 77 bytes per row at best, against 80 for int4 with its scales
