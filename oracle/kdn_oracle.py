"""ctypes front end of the CPU oracle (kdn_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
module.  It marshals numpy arrays (bf16 as uint16 bit patterns) into the plain
C oracle and holds none of the method's arithmetic itself.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# KDN_ORACLE_SRC names another copy of the C source (the mutation test plants one mistake
# per copy and expects the pins to fail); its library is built beside that copy.
_SRC = os.environ.get("KDN_ORACLE_SRC") or os.path.join(_HERE, "kdn_oracle.c")
_LIB = os.path.join(os.path.dirname(os.path.abspath(_SRC)), "libkdn_oracle.so")

FMT_RAW_BF16 = 0
FMT_INT8_ROWSCALE = 1
FMT_INT4_GROUP32 = 2
FMT_FP8_ROWSCALE = 3
GROUP = 32
PAIR_HALF_SPLIT = 0
PAIR_INTERLEAVED = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (scalar code, no contraction)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".%d.tmp" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared",
             "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Cache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p),
                ("L", C.c_int32), ("H", C.c_int32), ("D", C.c_int32),
                ("bs", C.c_int32), ("nb", C.c_int32),
                ("layer_stride", C.c_int64), ("block_stride", C.c_int64),
                ("token_stride", C.c_int64), ("head_stride", C.c_int64)]


_lib = None
_lock = threading.Lock()


def lib():
    global _lib
    with _lock:
        if _lib is None:
            L = C.CDLL(build())
            L.kdno_bf16_to_f32.restype = C.c_float
            L.kdno_bf16_to_f32.argtypes = [C.c_uint16]
            L.kdno_f32_to_bf16.restype = C.c_uint16
            L.kdno_f32_to_bf16.argtypes = [C.c_float]
            L.kdno_f32_to_bf16_array.restype = None
            L.kdno_f32_to_bf16_array.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
            L.kdno_chunk_bytes.restype = C.c_int64
            L.kdno_chunk_bytes.argtypes = [C.c_int32] * 5
            L.kdno_quantise_row.restype = None
            L.kdno_quantise_row.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
            L.kdno_quantise_row_int4.restype = None
            L.kdno_quantise_row_int4.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
            L.kdno_dequantise_row_int4.restype = None
            L.kdno_dequantise_row_int4.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
            L.kdno_f32_to_e4m3.restype = C.c_uint8
            L.kdno_f32_to_e4m3.argtypes = [C.c_float]
            L.kdno_e4m3_to_f32.restype = C.c_float
            L.kdno_e4m3_to_f32.argtypes = [C.c_uint8]
            L.kdno_quantise_row_fp8.restype = None
            L.kdno_quantise_row_fp8.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
            L.kdno_dequantise_row_fp8.restype = None
            L.kdno_dequantise_row_fp8.argtypes = [C.c_void_p, C.c_float, C.c_int32, C.c_void_p]
            L.kdno_dequantise_row.restype = None
            L.kdno_dequantise_row.argtypes = [C.c_void_p, C.c_float, C.c_int32, C.c_void_p]
            L.kdno_rope_table.restype = None
            L.kdno_rope_table.argtypes = [C.c_double, C.c_int32, C.c_int32, C.c_void_p]
            L.kdno_rotate_row.restype = None
            L.kdno_rotate_row.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
            L.kdno_store.restype = C.c_int
            L.kdno_store.argtypes = [C.POINTER(_Cache), C.c_void_p, C.c_int32, C.c_int32,
                                     C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_int32]
            L.kdno_load.restype = C.c_int
            L.kdno_load.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                    C.POINTER(_Cache), C.c_void_p, C.c_int32, C.c_int32,
                                    C.c_int32, C.c_int32]
            L.kdno_compose.restype = C.c_int
            L.kdno_compose.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.POINTER(_Cache), C.c_void_p, C.c_int32, C.c_int32,
                                       C.c_double, C.c_int32, C.c_int32]
            L.kdno_rope_table_spec.restype = None
            L.kdno_rope_table_spec.argtypes = [C.c_double, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
            L.kdno_rotate_row_spec.restype = None
            L.kdno_rotate_row_spec.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
            L.kdno_compose_spec.restype = C.c_int
            L.kdno_compose_spec.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.POINTER(_Cache), C.c_void_p, C.c_int32, C.c_int32,
                                            C.c_double, C.c_void_p, C.c_int32, C.c_int32,
                                            C.c_int32, C.c_int32]
            L.kdno_store_tokens.restype = C.c_int
            L.kdno_store_tokens.argtypes = [C.POINTER(_Cache), C.c_void_p, C.c_int32, C.c_void_p,
                                            C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_int32]
            L.kdno_patch_rows.restype = C.c_int
            L.kdno_patch_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(_Cache),
                                          C.c_void_p, C.c_int32]
            _lib = L
    return _lib


def _ptr(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


class PagedCache:
    """Host copy of an engine's paged KV memory: k, v are uint16 arrays of bf16
    bit patterns shaped [L][num_blocks][bs][H][D] (any element strides with
    contiguous D could be described; this wrapper uses the dense ones)."""

    def __init__(self, k: np.ndarray, v: np.ndarray):
        assert k.dtype == np.uint16 and v.dtype == np.uint16
        assert k.shape == v.shape and k.ndim == 5
        assert k.flags["C_CONTIGUOUS"] and v.flags["C_CONTIGUOUS"]
        self.k, self.v = k, v
        self.L, self.nb, self.bs, self.H, self.D = (int(x) for x in k.shape)

    def desc(self) -> _Cache:
        H, D, bs, nb = self.H, self.D, self.bs, self.nb
        return _Cache(_ptr(self.k), _ptr(self.v), self.L, H, D, bs, nb,
                      nb * bs * H * D, bs * H * D, H * D, D)

    def copy(self) -> "PagedCache":
        return PagedCache(self.k.copy(), self.v.copy())


class Chunk:
    """A stored chunk (or a token view of one) in host memory."""

    def __init__(self, data: np.ndarray, fmt: int, L: int, H: int, D: int,
                 Tp: int, tok_start: int = 0, T: int | None = None):
        assert data.dtype == np.uint8 and data.flags["C_CONTIGUOUS"]
        self.data, self.fmt, self.L, self.H, self.D = data, fmt, L, H, D
        self.Tp, self.tok_start = Tp, tok_start
        self.T = Tp - tok_start if T is None else T
        assert data.nbytes == chunk_bytes(L, H, D, Tp, fmt)

    def slice(self, tok_start: int, T: int) -> "Chunk":
        assert 0 <= tok_start and tok_start + T <= self.T
        return Chunk(self.data, self.fmt, self.L, self.H, self.D, self.Tp,
                     self.tok_start + tok_start, T)

    # typed views of the parent buffer, for tests
    def codes(self) -> np.ndarray:
        assert self.fmt in (FMT_INT8_ROWSCALE, FMT_FP8_ROWSCALE)
        n = self.L * 2 * self.Tp * self.H * self.D
        dt = np.int8 if self.fmt == FMT_INT8_ROWSCALE else np.uint8
        return self.data[:n].view(dt).reshape(self.L, 2, self.Tp, self.H, self.D)

    def scales(self) -> np.ndarray:
        assert self.fmt in (FMT_INT8_ROWSCALE, FMT_FP8_ROWSCALE)
        n = self.L * 2 * self.Tp * self.H * self.D
        return self.data[n:].view(np.float32).reshape(self.L, 2, self.Tp, self.H)

    def raw(self) -> np.ndarray:
        assert self.fmt == FMT_RAW_BF16
        return self.data.view(np.uint16).reshape(self.L, 2, self.Tp, self.H, self.D)

    def packed4(self) -> np.ndarray:
        assert self.fmt == FMT_INT4_GROUP32
        n = self.L * 2 * self.Tp * self.H * (self.D // 2)
        return self.data[:n].reshape(self.L, 2, self.Tp, self.H, self.D // 2)

    def scales4(self) -> np.ndarray:
        assert self.fmt == FMT_INT4_GROUP32
        n = self.L * 2 * self.Tp * self.H * (self.D // 2)
        return self.data[n:].view(np.float32).reshape(self.L, 2, self.Tp, self.H, self.D // GROUP)


def chunk_bytes(L: int, H: int, D: int, Tp: int, fmt: int) -> int:
    return int(lib().kdno_chunk_bytes(L, H, D, Tp, fmt))


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().kdno_f32_to_bf16_array(_ptr(x), _ptr(out), x.size)
    return out


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    f = lib().kdno_bf16_to_f32
    flat = np.ascontiguousarray(b, dtype=np.uint16).ravel()
    return np.array([f(int(v)) for v in flat], dtype=np.float32).reshape(np.shape(b))


def quantise_row(x_bf16: np.ndarray):
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    q = np.empty(x.size, dtype=np.int8)
    s = np.empty(1, dtype=np.float32)
    lib().kdno_quantise_row(_ptr(x), x.size, _ptr(q), _ptr(s))
    return q, np.float32(s[0])


def dequantise_row(q: np.ndarray, scale) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.int8)
    y = np.empty(q.size, dtype=np.float32)
    lib().kdno_dequantise_row(_ptr(q), C.c_float(float(scale)), q.size, _ptr(y))
    return y


def quantise_row_int4(x_bf16: np.ndarray):
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    packed = np.empty(x.size // 2, dtype=np.uint8)
    s = np.empty(x.size // GROUP, dtype=np.float32)
    lib().kdno_quantise_row_int4(_ptr(x), x.size, _ptr(packed), _ptr(s))
    return packed, s


def dequantise_row_int4(packed: np.ndarray, scales: np.ndarray) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    y = np.empty(packed.size * 2, dtype=np.float32)
    lib().kdno_dequantise_row_int4(_ptr(packed), _ptr(scales), y.size, _ptr(y))
    return y


def f32_to_e4m3(x: np.ndarray) -> np.ndarray:
    f = lib().kdno_f32_to_e4m3
    flat = np.ascontiguousarray(x, dtype=np.float32).ravel()
    return np.array([f(float(v)) for v in flat], dtype=np.uint8).reshape(np.shape(x))


def e4m3_to_f32(c: np.ndarray) -> np.ndarray:
    f = lib().kdno_e4m3_to_f32
    flat = np.ascontiguousarray(c, dtype=np.uint8).ravel()
    return np.array([f(int(v)) for v in flat], dtype=np.float32).reshape(np.shape(c))


def quantise_row_fp8(x_bf16: np.ndarray):
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    q = np.empty(x.size, dtype=np.uint8)
    s = np.empty(1, dtype=np.float32)
    lib().kdno_quantise_row_fp8(_ptr(x), x.size, _ptr(q), _ptr(s))
    return q, np.float32(s[0])


def dequantise_row_fp8(q: np.ndarray, scale) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.uint8)
    y = np.empty(q.size, dtype=np.float32)
    lib().kdno_dequantise_row_fp8(_ptr(q), C.c_float(float(scale)), q.size, _ptr(y))
    return y


def rope_table(base: float, D: int, d: int) -> np.ndarray:
    cs = np.empty((D // 2, 2), dtype=np.float32)
    lib().kdno_rope_table(float(base), D, int(d), _ptr(cs))
    return cs


def rotate_row(y: np.ndarray, cs: np.ndarray) -> np.ndarray:
    y = np.array(y, dtype=np.float32, copy=True)
    cs = np.ascontiguousarray(cs, dtype=np.float32)
    lib().kdno_rotate_row(_ptr(y), y.size, _ptr(cs))
    return y


def _bt(block_table) -> np.ndarray:
    return np.ascontiguousarray(block_table, dtype=np.int32)


def store(cache: PagedCache, block_table, t0: int, T: int, fmt: int,
          layers: tuple[int, int] | None = None, out: Chunk | None = None) -> Chunk:
    bt = _bt(block_table)
    if out is None:
        out = Chunk(np.zeros(chunk_bytes(cache.L, cache.H, cache.D, T, fmt), dtype=np.uint8),
                    fmt, cache.L, cache.H, cache.D, T)
    l0, l1 = layers if layers is not None else (0, cache.L)
    d = cache.desc()
    rc = lib().kdno_store(C.byref(d), _ptr(bt), bt.size, t0, T, fmt, _ptr(out.data), l0, l1)
    if rc:
        raise ValueError("kdno_store: bad range or block id")
    return out


def load(chunk: Chunk, cache: PagedCache, block_table, dest: int,
         layers: tuple[int, int] | None = None) -> None:
    bt = _bt(block_table)
    l0, l1 = layers if layers is not None else (0, cache.L)
    d = cache.desc()
    rc = lib().kdno_load(_ptr(chunk.data), chunk.fmt, chunk.Tp, chunk.tok_start, chunk.T,
                         C.byref(d), _ptr(bt), bt.size, dest, l0, l1)
    if rc:
        raise ValueError("kdno_load: bad range or block id")


def compose(chunks, offsets, cache: PagedCache, block_table, rope_base: float,
            dest: int = 0, layers: tuple[int, int] | None = None) -> None:
    bt = _bt(block_table)
    n = len(chunks)
    assert len(offsets) == n
    data = (C.c_void_p * max(n, 1))(*[_ptr(c.data) for c in chunks])
    fmt = np.array([c.fmt for c in chunks], dtype=np.int32)
    Tp = np.array([c.Tp for c in chunks], dtype=np.int32)
    ts = np.array([c.tok_start for c in chunks], dtype=np.int32)
    T = np.array([c.T for c in chunks], dtype=np.int32)
    off = np.ascontiguousarray(offsets, dtype=np.int32)
    l0, l1 = layers if layers is not None else (0, cache.L)
    d = cache.desc()
    rc = lib().kdno_compose(n, C.cast(data, C.c_void_p), _ptr(fmt), _ptr(Tp), _ptr(ts),
                            _ptr(T), _ptr(off), C.byref(d), _ptr(bt), bt.size, dest,
                            float(rope_base), l0, l1)
    if rc:
        raise ValueError("kdno_compose: bad range or block id")


def rope_table_spec(base: float, inv_freq, rot_dim: int, d: int) -> np.ndarray:
    cs = np.empty((rot_dim // 2, 2), dtype=np.float32)
    f = None if inv_freq is None else np.ascontiguousarray(inv_freq, dtype=np.float64)
    lib().kdno_rope_table_spec(float(base), None if f is None else _ptr(f), rot_dim, int(d), _ptr(cs))
    return cs


def rotate_row_spec(y: np.ndarray, rot_dim: int, pairing: int, cs: np.ndarray) -> np.ndarray:
    y = np.array(y, dtype=np.float32, copy=True)
    cs = np.ascontiguousarray(cs, dtype=np.float32)
    lib().kdno_rotate_row_spec(_ptr(y), rot_dim, pairing, _ptr(cs))
    return y


def compose_spec(chunks, offsets, cache: PagedCache, block_table, rope_base: float = 10000.0,
                 inv_freq=None, rot_dim: int = 0, pairing: int = PAIR_HALF_SPLIT, dest: int = 0,
                 layers: tuple[int, int] | None = None) -> None:
    bt = _bt(block_table)
    n = len(chunks)
    assert len(offsets) == n
    data = (C.c_void_p * max(n, 1))(*[_ptr(c.data) for c in chunks])
    fmt = np.array([c.fmt for c in chunks], dtype=np.int32)
    Tp = np.array([c.Tp for c in chunks], dtype=np.int32)
    ts = np.array([c.tok_start for c in chunks], dtype=np.int32)
    T = np.array([c.T for c in chunks], dtype=np.int32)
    off = np.ascontiguousarray(offsets, dtype=np.int32)
    f = None if inv_freq is None else np.ascontiguousarray(inv_freq, dtype=np.float64)
    l0, l1 = layers if layers is not None else (0, cache.L)
    d = cache.desc()
    rc = lib().kdno_compose_spec(n, C.cast(data, C.c_void_p), _ptr(fmt), _ptr(Tp), _ptr(ts),
                                 _ptr(T), _ptr(off), C.byref(d), _ptr(bt), bt.size, dest,
                                 float(rope_base), None if f is None else _ptr(f), rot_dim, pairing,
                                 l0, l1)
    if rc:
        raise ValueError("kdno_compose_spec: bad range, block id or rope variant")


def patch_rows(rows: np.ndarray, tokens, cache: PagedCache, block_table) -> None:
    """rows: uint16 [L][2][n][H][D]; tokens: n distinct request token indices."""
    bt = _bt(block_table)
    tok = np.ascontiguousarray(tokens, dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.uint16)
    assert rows.shape == (cache.L, 2, tok.size, cache.H, cache.D)
    d = cache.desc()
    rc = lib().kdno_patch_rows(_ptr(rows), _ptr(tok), tok.size, C.byref(d), _ptr(bt), bt.size)
    if rc:
        raise ValueError("kdno_patch_rows: token or block id out of range")


def store_tokens(cache: PagedCache, block_table, tokens, fmt: int) -> Chunk:
    """Chunk whose row t holds request token tokens[t]."""
    bt = _bt(block_table)
    tok = np.ascontiguousarray(tokens, dtype=np.int32)
    out = Chunk(np.zeros(chunk_bytes(cache.L, cache.H, cache.D, tok.size, fmt), dtype=np.uint8),
                fmt, cache.L, cache.H, cache.D, int(tok.size))
    d = cache.desc()
    rc = lib().kdno_store_tokens(C.byref(d), _ptr(bt), bt.size, _ptr(tok), tok.size, fmt,
                                 _ptr(out.data), 0, cache.L)
    if rc:
        raise ValueError("kdno_store_tokens: token or block id out of range")
    return out
