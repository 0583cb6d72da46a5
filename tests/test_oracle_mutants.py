"""Mutation check of the oracle's pins (CPU only, no GPU).

Each entry plants ONE mistake in a scratch copy of oracle/kdn_oracle.c (an exact
substring replacement), builds that copy beside itself and runs the pins of
tests/test_oracle_pins.py against it in a child process.  A pin must fail for every
planted mistake; a mistake that every pin lets through is a hole in the pins.
The oracle in the tree is never touched, and nothing here runs on a GPU.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "kdn_oracle.c")

# (what the mistake is, text in the oracle, text that replaces it)
MUTANTS = [
    # rotation
    ("sign of the sine term of the lower element", "y[j] = fmaf(-b, s, ac);", "y[j] = fmaf(b, s, ac);"),
    ("sign of the sine term of the upper element", "y[j + half] = fmaf(a, s, bc);", "y[j + half] = fmaf(-a, s, bc);"),
    ("pair operands transposed", "float a = y[j], b = y[j + half];", "float a = y[j + half], b = y[j];"),
    ("frequency exponent j for 2j", "double theta = pow(base, -(double)(2 * j) / (double)D);",
     "double theta = pow(base, -(double)(j) / (double)D);"),
    ("cos slot holds sin", "cs[2 * j] = (float)cos(phi);\n        cs[2 * j + 1] = (float)sin(phi);\n    }\n}\n\n/* ---- RoPE variants",
     "cs[2 * j] = (float)sin(phi);\n        cs[2 * j + 1] = (float)sin(phi);\n    }\n}\n\n/* ---- RoPE variants"),
    ("rotation applied to V instead of K", "int rotate = (side == 0 && d != 0);", "int rotate = (side == 1 && d != 0);"),
    ("rotation applied to K and V", "int rotate = (side == 0 && d != 0);", "int rotate = (d != 0);"),
    # int8 quantiser
    ("scale = amax/128", "*scale = amax / 127.0f;", "*scale = amax / 128.0f;"),
    ("inv = 126/amax", "float inv = 127.0f / amax;", "float inv = 126.0f / amax;"),
    ("codes truncated instead of rounded", "float r = rintf(kdno_bf16_to_f32(x[j]) * inv);",
     "float r = truncf(kdno_bf16_to_f32(x[j]) * inv);"),
    ("amax skips element 0", "        if (a > amax)\n            amax = a;\n    }\n    if (amax < 0x1p-121f) {",
     "        if (a > amax && j > 0)\n            amax = a;\n    }\n    if (amax < 0x1p-121f) {"),
    ("dequantised value scaled by 1 + 2^-23", "y[j] = (float)q[j] * scale;", "y[j] = (float)q[j] * scale * 1.0000001f;"),
    # bf16 narrowing
    ("bf16 rounding: ties away from zero", "u += 0x7fffu + keep_lsb;", "u += 0x8000u;"),
    ("bf16 rounding: truncation", "u += 0x7fffu + keep_lsb;", "u += 0;"),
    # addressing
    ("slot off by one", "int32_t slot = tok % c->bs;\n                if (block < 0 || block >= c->nb)\n                    return -1;\n                for (int32_t h = 0; h < H; ++h) {\n                    const uint16_t *src",
     "int32_t slot = (tok + 1) % c->bs;\n                if (block < 0 || block >= c->nb)\n                    return -1;\n                for (int32_t h = 0; h < H; ++h) {\n                    const uint16_t *src"),
    ("destination slot off by one", "int32_t slot = tok % c->bs;\n                if (block < 0 || block >= c->nb)\n                    return -1;\n                for (int32_t h = 0; h < H; ++h) {\n                    uint16_t *dst",
     "int32_t slot = (tok + 1) % c->bs;\n                if (block < 0 || block >= c->nb)\n                    return -1;\n                for (int32_t h = 0; h < H; ++h) {\n                    uint16_t *dst"),
    ("placement prefix sum off by one after the first chunk", "        S += T[i];\n    }\n    return 0;\n}\n\n/* Compose with a RoPE variant",
     "        S += T[i]; if (i == 0) S += 1;\n    }\n    return 0;\n}\n\n/* Compose with a RoPE variant"),
    ("view offset of a slice ignored", "int64_t r = row_index(l, side, Tp, tok_start + t, H, h);", "int64_t r = row_index(l, side, Tp, t, H, h);"),
    ("head stride taken as D", "+ (int64_t)h * c->head_stride;", "+ (int64_t)h * c->D;"),
    ("K and V planes of the chunk swapped", "return (((int64_t)l * 2 + side) * Tp + t) * H + h;",
     "return (((int64_t)l * 2 + (1 - side)) * Tp + t) * H + h;"),
    # the store's indexing around the row quantisers
    ("int8 store quantises the neighbouring head's row", "                        kdno_quantise_row(src, D, codes + r * D, scales + r);",
     "                        kdno_quantise_row(cache_row(c, l, side, block, slot, (h + 1) % H), D, codes + r * D, scales + r);"),
    ("int8 store writes the scale to the neighbouring slot", "                        kdno_quantise_row(src, D, codes + r * D, scales + r);",
     "                        kdno_quantise_row(src, D, codes + r * D, scales + (r ^ 1));"),
    ("fp8 store writes the scale to the neighbouring slot", "kdno_quantise_row_fp8(src, D, (uint8_t *)codes + r * D, scales + r);",
     "kdno_quantise_row_fp8(src, D, (uint8_t *)codes + r * D, scales + (r ^ 1));"),
    ("fp8 store writes the codes one row further", "kdno_quantise_row_fp8(src, D, (uint8_t *)codes + r * D, scales + r);",
     "kdno_quantise_row_fp8(src, D, (uint8_t *)codes + (r ^ 1) * D, scales + r);"),
    ("int4 store writes the group scales of the neighbouring row",
     "kdno_quantise_row_int4(src, D, codes4 + r * (D / 2), scales4 + r * (D / KDNO_GROUP));",
     "kdno_quantise_row_int4(src, D, codes4 + r * (D / 2), scales4 + (r ^ 1) * (D / KDNO_GROUP));"),
    ("int4 store row stride of the scales taken as 1", "kdno_quantise_row_int4(src, D, codes4 + r * (D / 2), scales4 + r * (D / KDNO_GROUP));",
     "kdno_quantise_row_int4(src, D, codes4 + r * (D / 2), scales4 + r);"),
    ("store reads token t0 + t from the wrong block-table entry", "                int32_t tok = t0 + t;\n                int32_t block = bt[tok / c->bs];",
     "                int32_t tok = t0 + t;\n                int32_t block = bt[t / c->bs];"),
    # int4
    ("nibble order swapped in the packer", "(uint8_t)((q[0] & 0xF) | ((q[1] & 0xF) << 4))", "(uint8_t)((q[1] & 0xF) | ((q[0] & 0xF) << 4))"),
    ("int4 scale = amax/8", "scales[g] = keep ? amax / 7.0f : 0.0f;", "scales[g] = keep ? amax / 8.0f : 0.0f;"),
    ("int4 inv = 8/amax", "float inv = keep ? 7.0f / amax : 0.0f;", "float inv = keep ? 8.0f / amax : 0.0f;"),
    ("nibbles not sign-extended", "int q = nib >= 8 ? nib - 16 : nib;", "int q = nib;"),
    ("every group dequantised with scale 0", "y[j] = (float)q * scales[j / KDNO_GROUP];", "y[j] = (float)q * scales[0];"),
    ("nibble order swapped in the decoder", "int nib = (packed[j / 2] >> (4 * (j & 1))) & 0xF;",
     "int nib = (packed[j / 2] >> (4 * (1 - (j & 1)))) & 0xF;"),
    ("int4 codes truncated", "float r = keep ? rintf(kdno_bf16_to_f32(xg[j + e]) * inv) : 0.0f;",
     "float r = keep ? truncf(kdno_bf16_to_f32(xg[j + e]) * inv) : 0.0f;"),
    ("place reads int4 scales with row stride 1", "kdno_dequantise_row_int4(codes4 + r * (D / 2), scales4 + r * (D / KDNO_GROUP), D, y);",
     "kdno_dequantise_row_int4(codes4 + r * (D / 2), scales4 + r, D, y);"),
    # RoPE variants, patch
    ("interleaved pair operands transposed", "int32_t ib = pairing == KDNO_PAIR_INTERLEAVED ? 2 * j + 1 : j + half;",
     "int32_t ib = pairing == KDNO_PAIR_INTERLEAVED ? 2 * j + 1 : j + half; if (pairing == KDNO_PAIR_INTERLEAVED) { int32_t t = ia; ia = ib; ib = t; }"),
    ("variant frequencies use 128 for rot_dim", "double theta = inv_freq ? inv_freq[j] : pow(base, -(double)(2 * j) / (double)rot_dim);",
     "double theta = inv_freq ? inv_freq[j] : pow(base, -(double)(2 * j) / 128.0);"),
    ("explicit frequencies: entry 0 for all", "double theta = inv_freq ? inv_freq[j] :", "double theta = inv_freq ? inv_freq[0] :"),
    ("variant pairing ignored in place", "kdno_rotate_row_spec(y, rot_dim, pairing, cs);\n                    for",
     "kdno_rotate_row_spec(y, rot_dim, KDNO_PAIR_HALF_SPLIT, cs);\n                    for"),
    ("patch swaps K and V", "rows + ((((int64_t)l * 2 + side) * n + i) * c->H + h) * c->D", "rows + ((((int64_t)l * 2 + (1 - side)) * n + i) * c->H + h) * c->D"),
    ("patch slot from the list index", "int32_t block = bt[tokens[i] / c->bs], slot = tokens[i] % c->bs;",
     "int32_t block = bt[tokens[i] / c->bs], slot = i % c->bs;"),
    # fp8
    ("e4m3 saturation starts a binade late", "if (a >= 448.0f)", "if (a >= 480.0f)"),
    ("e4m3 subnormal ties round up", "int q = (int)rintf(a * 0x1p9f); ", "int q = (int)(a * 0x1p9f + 0.5f); "),
    ("e4m3 normal ties round up", "int q = (int)rintf((m - 1.0f) * 8.0f); ", "int q = (int)((m - 1.0f) * 8.0f + 0.5f); "),
    ("e4m3 exponent bias 8", "return (uint8_t)(sign | ((e + 7) << 3) | q);", "return (uint8_t)(sign | ((e + 8) << 3) | q);"),
    ("e4m3 subnormal step 2^-10", "v = ldexpf((float)q, -9);", "v = ldexpf((float)q, -10);"),
    ("fp8 flush threshold 2^-121", "if (amax < 0x1p-119f) {", "if (amax < 0x1p-121f) {"),
    ("fp8 scale = amax/240", "*scale = amax / 448.0f;", "*scale = amax / 240.0f;"),
    ("fp8 inv as reciprocal of the scale", "float inv = 448.0f / amax;", "float inv = 1.0f / (amax / 448.0f);"),
    # token-list store
    ("token-list store: slot from the list index", "int32_t block = bt[tokens[t] / c->bs], slot = tokens[t] % c->bs;",
     "int32_t block = bt[tokens[t] / c->bs], slot = t % c->bs;"),
    ("token-list store: rows written in reverse", "int64_t r = row_index(l, side, n, t, H, h);", "int64_t r = row_index(l, side, n, n - 1 - t, H, h);"),
]


def _run_mutant(args):
    i, (what, old, new), tmp = args
    text = open(SRC).read()
    if text.count(old) != 1:
        return i, what, "not applicable: the oracle holds %d copies of the text to replace" % text.count(old)
    d = os.path.join(tmp, "m%02d" % i)
    os.makedirs(d)
    path = os.path.join(d, "kdn_oracle.c")
    with open(path, "w") as f:
        f.write(text.replace(old, new))
    env = dict(os.environ, KDN_ORACLE_SRC=path, PYTHONDONTWRITEBYTECODE="1")
    proc = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                           "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    if proc.returncode == 0:
        return i, what, "SURVIVED: every pin passed"
    if " failed" not in proc.stdout:
        return i, what, "the run broke without a failing pin:\n" + proc.stdout[-800:]
    return i, what, None


def test_every_planted_mistake_fails_a_pin(tmp_path):
    workers = max(1, min(8, len(os.sched_getaffinity(0))))
    jobs = [(i, m, str(tmp_path)) for i, m in enumerate(MUTANTS)]
    with ThreadPoolExecutor(workers) as pool:
        results = list(pool.map(_run_mutant, jobs))
    bad = ["mutant %d (%s): %s" % (i, what, why) for i, what, why in results if why]
    assert not bad, "\n".join(bad)
    assert len(MUTANTS) >= 45


def test_the_unmutated_oracle_passes_through_the_same_door(tmp_path):
    """The override that points the pins at another source is itself exercised: a verbatim
    copy of the oracle must pass them (otherwise every 'failure' above could be the door's)."""
    path = os.path.join(str(tmp_path), "kdn_oracle.c")
    with open(path, "w") as f:
        f.write(open(SRC).read())
    env = dict(os.environ, KDN_ORACLE_SRC=path, PYTHONDONTWRITEBYTECODE="1")
    proc = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                           "-x", "-q", "-p", "no:cacheprovider", "-k", "store or quantis or rope or bf16"],
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert proc.returncode == 0, proc.stdout[-1500:]
    assert os.path.exists(os.path.join(str(tmp_path), "libkdn_oracle.so"))
