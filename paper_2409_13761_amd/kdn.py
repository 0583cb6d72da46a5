"""Thin Python binding of the C ABI in include/kdn.h.

Argument marshalling only: every step of store / load / compose runs in the HIP
kernels of libkdn.so.  PyTorch supplies device memory (tensors) and streams.
There is no CPU fallback: if the library is missing or was not built, importing
this module's entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkdn.so")

FMT_RAW_BF16 = 0
FMT_INT8_ROWSCALE = 1
FMT_INT4_GROUP32 = 2
FMT_FP8_ROWSCALE = 3

OK, EINVAL, EALIGN, ERANGE, ESIZE, EDEVICE, EUNSUPPORTED, ENOTFOUND, EFULL = 0, -1, -2, -3, -4, -5, -6, -7, -8


class KdnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, status_str(status), status))


class CacheDesc(C.Structure):
    _fields_ = [("k_base", C.c_void_p), ("v_base", C.c_void_p),
                ("num_layers", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_size", C.c_int32), ("num_blocks", C.c_int32),
                ("layer_stride", C.c_int64), ("block_stride", C.c_int64),
                ("token_stride", C.c_int64), ("head_stride", C.c_int64)]


class ChunkDesc(C.Structure):
    _fields_ = [("data", C.c_void_p), ("bytes", C.c_uint64), ("fmt", C.c_int32),
                ("num_layers", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("parent_tokens", C.c_int32), ("token_start", C.c_int32), ("num_tokens", C.c_int32)]


class RopeSpecDesc(C.Structure):
    _fields_ = [("base", C.c_double), ("inv_freq", C.POINTER(C.c_double)),
                ("rot_dim", C.c_int32), ("pairing", C.c_int32)]


ROPE_HALF_SPLIT = 0
ROPE_INTERLEAVED = 1


class LaunchOpts(C.Structure):
    _fields_ = [("max_workgroups", C.c_int32)]


class ArenaInfo(C.Structure):
    _fields_ = [("bytes", C.c_uint64), ("granule", C.c_uint64), ("in_use", C.c_uint64), ("largest_free", C.c_uint64),
                ("free_granules", C.c_uint64), ("stride", C.c_uint64), ("striped_gbs", C.c_float),
                ("packed_gbs", C.c_float), ("seconds", C.c_float), ("reserved", C.c_int32)]

    def as_dict(self) -> dict:
        return {"bytes": self.bytes, "granule": self.granule, "in_use": self.in_use, "largest_free": self.largest_free,
                "free_granules": self.free_granules, "stride": self.stride,
                "striped_gbs": round(self.striped_gbs, 1), "packed_gbs": round(self.packed_gbs, 1),
                "seconds": round(self.seconds, 3)}


class PoolStats(C.Structure):
    _fields_ = [("hits", C.c_uint64), ("misses", C.c_uint64), ("inserts", C.c_uint64),
                ("evictions", C.c_uint64), ("bytes", C.c_uint64), ("entries", C.c_uint64)]


class RequestDesc(C.Structure):
    _fields_ = [("chunks", C.POINTER(ChunkDesc)), ("offsets", C.POINTER(C.c_int32)),
                ("n_chunks", C.c_int32), ("block_table_dev", C.c_void_p),
                ("table_len", C.c_int32), ("dest_token_start", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """Load libkdn.so (built beforehand by build.build_library / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libkdn.so is not built: run `python -m paper_2409_13761_amd.build` "
                              "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, u64 = C.c_void_p, C.c_int32, C.c_uint64
        L.kdn_chunk_bytes.restype = u64
        L.kdn_chunk_bytes.argtypes = [i32, i32, i32, i32, i32]
        L.kdn_chunk_init.restype = C.c_int
        L.kdn_chunk_init.argtypes = [C.POINTER(ChunkDesc), vp, u64, i32, i32, i32, i32, i32]
        L.kdn_chunk_slice.restype = C.c_int
        L.kdn_chunk_slice.argtypes = [C.POINTER(ChunkDesc), i32, i32, C.POINTER(ChunkDesc)]
        L.kdn_store_chunk.restype = C.c_int
        L.kdn_store_chunk.argtypes = [C.POINTER(CacheDesc), vp, i32, i32, i32, C.POINTER(ChunkDesc), vp]
        L.kdn_store_chunk_opts.restype = C.c_int
        L.kdn_store_chunk_opts.argtypes = [C.POINTER(CacheDesc), vp, i32, i32, i32, C.POINTER(ChunkDesc),
                                           C.POINTER(LaunchOpts), vp]
        L.kdn_compose_opts.restype = C.c_int
        L.kdn_compose_opts.argtypes = [C.POINTER(ChunkDesc), C.POINTER(i32), i32, C.POINTER(CacheDesc),
                                       vp, i32, i32, C.c_double, C.POINTER(RopeSpecDesc),
                                       C.POINTER(LaunchOpts), vp]
        L.kdn_store_tokens.restype = C.c_int
        L.kdn_store_tokens.argtypes = [C.POINTER(CacheDesc), vp, i32, vp, i32, C.POINTER(ChunkDesc), vp]
        L.kdn_store_to_host.restype = C.c_int
        L.kdn_store_to_host.argtypes = [C.POINTER(CacheDesc), vp, i32, i32, i32, C.POINTER(ChunkDesc),
                                        vp, u64, i32, vp]
        L.kdn_store_staging_bytes.restype = u64
        L.kdn_store_staging_bytes.argtypes = [C.POINTER(CacheDesc), i32, i32, i32]
        L.kdn_load_chunk.restype = C.c_int
        L.kdn_load_chunk.argtypes = [C.POINTER(ChunkDesc), C.POINTER(CacheDesc), vp, i32, i32, vp]
        L.kdn_compose.restype = C.c_int
        L.kdn_compose.argtypes = [C.POINTER(ChunkDesc), C.POINTER(i32), i32, C.POINTER(CacheDesc),
                                  vp, i32, i32, C.c_double, vp]
        L.kdn_compose_batch.restype = C.c_int
        L.kdn_compose_batch.argtypes = [C.POINTER(RequestDesc), i32, C.POINTER(CacheDesc),
                                        C.c_double, vp]
        L.kdn_compose_batch_static.restype = C.c_int
        L.kdn_compose_batch_static.argtypes = [C.POINTER(RequestDesc), i32, C.POINTER(CacheDesc),
                                               C.c_double, vp]
        L.kdn_compose_rope.restype = C.c_int
        L.kdn_compose_rope.argtypes = [C.POINTER(ChunkDesc), C.POINTER(i32), i32, C.POINTER(CacheDesc),
                                       vp, i32, i32, C.POINTER(RopeSpecDesc), vp]
        L.kdn_compose_batch_rope.restype = C.c_int
        L.kdn_compose_batch_rope.argtypes = [C.POINTER(RequestDesc), i32, C.POINTER(CacheDesc),
                                             C.POINTER(RopeSpecDesc), vp]
        L.kdn_patch_rows.restype = C.c_int
        L.kdn_patch_rows.argtypes = [vp, vp, i32, C.POINTER(CacheDesc), vp, i32, vp]
        L.kdn_pool_create.restype = C.c_int
        L.kdn_pool_create.argtypes = [u64, i32, C.POINTER(vp)]
        L.kdn_pool_destroy.restype = None
        L.kdn_pool_destroy.argtypes = [vp]
        L.kdn_pool_hash.restype = u64
        L.kdn_pool_hash.argtypes = [vp, i32]
        L.kdn_pool_lookup.restype = C.c_int
        L.kdn_pool_lookup.argtypes = [vp, vp, i32, C.POINTER(ChunkDesc)]
        L.kdn_pool_insert.restype = C.c_int
        L.kdn_pool_insert.argtypes = [vp, vp, i32, C.POINTER(ChunkDesc), C.POINTER(ChunkDesc), i32,
                                      C.POINTER(i32)]
        L.kdn_pool_remove.restype = C.c_int
        L.kdn_pool_remove.argtypes = [vp, vp, i32, C.POINTER(ChunkDesc)]
        L.kdn_pool_get_stats.restype = C.c_int
        L.kdn_pool_get_stats.argtypes = [vp, C.POINTER(PoolStats)]
        L.kdn_compose_from_host.restype = C.c_int
        L.kdn_compose_from_host.argtypes = [C.POINTER(ChunkDesc), C.POINTER(i32), i32,
                                            C.POINTER(CacheDesc), vp, i32, i32, C.c_double,
                                            vp, u64, i32, vp]
        L.kdn_compose_from_host_staged.restype = C.c_int
        L.kdn_compose_from_host_staged.argtypes = [C.POINTER(ChunkDesc), C.POINTER(i32), i32,
                                                   C.POINTER(CacheDesc), vp, i32, i32, C.c_double,
                                                   vp, u64, i32, C.POINTER(vp), i32, vp]
        L.kdn_staging_bytes.restype = u64
        L.kdn_staging_bytes.argtypes = [C.POINTER(ChunkDesc), i32, i32]
        L.kdn_compose_plan.restype = C.c_int
        L.kdn_compose_plan.argtypes = [vp, i32, vp, vp, i32, C.POINTER(i32)]
        L.kdn_host_stage_plan.restype = C.c_int
        L.kdn_host_stage_plan.argtypes = [C.POINTER(ChunkDesc), i32, i32, i32, vp, i32, C.POINTER(i32), vp]
        L.kdn_tile_tokens.restype = i32
        L.kdn_tile_tokens.argtypes = [C.POINTER(CacheDesc)]
        L.kdn_rope_prepare.restype = C.c_int
        L.kdn_rope_prepare.argtypes = [C.c_double, i32, C.POINTER(i32), i32]
        L.kdn_rope_prepare_spec.restype = C.c_int
        L.kdn_rope_prepare_spec.argtypes = [C.POINTER(RopeSpecDesc), i32, C.POINTER(i32), i32]
        L.kdn_rope_release.restype = C.c_int
        L.kdn_rope_release.argtypes = []
        L.kdn_validate_block_table.restype = C.c_int
        L.kdn_validate_block_table.argtypes = [vp, i32, i32, vp]
        L.kdn_probe_stream.restype = C.c_int
        L.kdn_probe_stream.argtypes = [vp, vp, vp, C.c_uint32, i32, i32, i32, vp]
        L.kdn_f32_to_bf16.restype = C.c_int
        L.kdn_f32_to_bf16.argtypes = [vp, vp, u64, vp]
        L.kdn_arena_create.restype = C.c_int
        L.kdn_arena_create.argtypes = [u64, i32, C.POINTER(ArenaInfo)]
        L.kdn_arena_alloc.restype = C.c_int
        L.kdn_arena_alloc.argtypes = [u64, C.POINTER(vp)]
        L.kdn_arena_free.restype = C.c_int
        L.kdn_arena_free.argtypes = [vp]
        L.kdn_arena_query.restype = C.c_int
        L.kdn_arena_query.argtypes = [C.POINTER(ArenaInfo)]
        L.kdn_arena_destroy.restype = C.c_int
        L.kdn_arena_destroy.argtypes = []
        L.kdn_shutdown.restype = C.c_int
        L.kdn_shutdown.argtypes = []
        L.kdn_status_str.restype = C.c_char_p
        L.kdn_status_str.argtypes = [C.c_int]
        L.kdn_version.restype = C.c_char_p
        L.kdn_version.argtypes = []
        from . import build as _build
        built_from = L.kdn_version().decode().rsplit("src:", 1)[-1]
        if built_from != _build.source_fingerprint():
            raise ImportError("libkdn.so was built from other sources (it carries %s, the tree is %s): "
                              "run `python -m paper_2409_13761_amd.build`" % (built_from, _build.source_fingerprint()))
        _lib = L
    return _lib


EXPORTS = ["kdn_chunk_bytes", "kdn_chunk_init", "kdn_chunk_slice", "kdn_store_chunk", "kdn_store_tokens",
           "kdn_store_to_host", "kdn_store_staging_bytes", "kdn_store_chunk_opts", "kdn_compose_opts",
           "kdn_load_chunk", "kdn_compose", "kdn_compose_batch", "kdn_compose_batch_static", "kdn_compose_rope",
           "kdn_compose_batch_rope", "kdn_patch_rows", "kdn_compose_from_host", "kdn_compose_from_host_staged",
           "kdn_staging_bytes", "kdn_host_stage_plan", "kdn_compose_plan", "kdn_tile_tokens", "kdn_rope_prepare", "kdn_rope_prepare_spec", "kdn_rope_release",
           "kdn_validate_block_table", "kdn_probe_stream", "kdn_f32_to_bf16", "kdn_shutdown", "kdn_status_str",
           "kdn_version", "kdn_pool_create", "kdn_pool_destroy", "kdn_pool_hash", "kdn_pool_lookup",
           "kdn_pool_insert", "kdn_pool_remove", "kdn_pool_get_stats", "kdn_arena_create", "kdn_arena_alloc",
           "kdn_arena_free", "kdn_arena_query", "kdn_arena_destroy"]


def status_str(status: int) -> str:
    return lib().kdn_status_str(status).decode()


def _check(status: int, where: str) -> None:
    if status != OK:
        raise KdnError(status, where)


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


# ------------------------------------------------------------------ descriptors
@dataclass
class PagedCache:
    """An engine's paged KV memory held in two bf16 tensors shaped
    [L][num_blocks][block_size][H][D] (last dimension contiguous)."""
    k: torch.Tensor
    v: torch.Tensor

    def __post_init__(self):
        for t in (self.k, self.v):
            assert t.dtype == torch.bfloat16 and t.dim() == 5 and t.stride(4) == 1
        assert self.k.shape == self.v.shape and self.k.stride() == self.v.stride()

    @property
    def shape(self):
        L, nb, bs, H, D = self.k.shape
        return L, nb, bs, H, D

    def desc(self) -> CacheDesc:
        L, nb, bs, H, D = self.k.shape
        s = self.k.stride()
        return CacheDesc(self.k.data_ptr(), self.v.data_ptr(), L, H, D, bs, nb,
                         s[0], s[1], s[2], s[3])


class Chunk:
    """A stored chunk (or token view) over a uint8 device tensor."""

    def __init__(self, data: torch.Tensor, desc: ChunkDesc):
        self.data, self.desc = data, desc

    @property
    def fmt(self) -> int:
        return self.desc.fmt

    @property
    def num_tokens(self) -> int:
        return self.desc.num_tokens

    def slice(self, token_start: int, num_tokens: int) -> "Chunk":
        return chunk_slice(self, token_start, num_tokens)

    def _split(self):
        d = self.desc
        n = d.num_layers * 2 * d.parent_tokens * d.num_kv_heads * d.head_dim
        return d, n

    def codes(self) -> torch.Tensor:
        d, n = self._split()
        assert d.fmt in (FMT_INT8_ROWSCALE, FMT_FP8_ROWSCALE)
        return self.data[:n].view(torch.int8 if d.fmt == FMT_INT8_ROWSCALE else torch.uint8).view(d.num_layers, 2, d.parent_tokens,
                                                   d.num_kv_heads, d.head_dim)

    def scales(self) -> torch.Tensor:
        d, n = self._split()
        assert d.fmt in (FMT_INT8_ROWSCALE, FMT_FP8_ROWSCALE)
        return self.data[n:n + n // d.head_dim * 4].view(torch.float32).view(
            d.num_layers, 2, d.parent_tokens, d.num_kv_heads)

    def packed4(self) -> torch.Tensor:
        d, n = self._split()
        assert d.fmt == FMT_INT4_GROUP32
        return self.data[:n // 2].view(d.num_layers, 2, d.parent_tokens, d.num_kv_heads, d.head_dim // 2)

    def scales4(self) -> torch.Tensor:
        d, n = self._split()
        assert d.fmt == FMT_INT4_GROUP32
        return self.data[n // 2:n // 2 + n // 32 * 4].view(torch.float32).view(
            d.num_layers, 2, d.parent_tokens, d.num_kv_heads, d.head_dim // 32)

    def raw(self) -> torch.Tensor:
        d, n = self._split()
        assert d.fmt == FMT_RAW_BF16
        return self.data[:2 * n].view(torch.bfloat16).view(d.num_layers, 2, d.parent_tokens,
                                                           d.num_kv_heads, d.head_dim)


# ------------------------------------------------------------------ calls
def kdn_chunk_bytes(L: int, H: int, D: int, num_tokens: int, fmt: int) -> int:
    return int(lib().kdn_chunk_bytes(L, H, D, num_tokens, fmt))


def alloc_chunk(cache: PagedCache, num_tokens: int, fmt: int, arena: bool = False) -> Chunk:
    """Allocate the device buffer of a chunk (with torch, or from the striped arena) and describe it."""
    L, _, _, H, D = cache.shape
    n = kdn_chunk_bytes(L, H, D, num_tokens, fmt)
    if n == 0:
        raise KdnError(EINVAL, "kdn_chunk_bytes")
    data = arena_tensor(n) if arena else torch.empty(n, dtype=torch.uint8, device=cache.k.device)
    d = ChunkDesc()
    _check(lib().kdn_chunk_init(C.byref(d), data.data_ptr(), n, fmt, L, H, D, num_tokens),
           "kdn_chunk_init")
    return Chunk(data, d)


def chunk_from_buffer(data: torch.Tensor, fmt: int, L: int, H: int, D: int, num_tokens: int) -> Chunk:
    d = ChunkDesc()
    _check(lib().kdn_chunk_init(C.byref(d), data.data_ptr(), data.numel() * data.element_size(),
                                fmt, L, H, D, num_tokens), "kdn_chunk_init")
    return Chunk(data, d)


def chunk_slice(chunk: Chunk, token_start: int, num_tokens: int) -> Chunk:
    d = ChunkDesc()
    _check(lib().kdn_chunk_slice(C.byref(chunk.desc), token_start, num_tokens, C.byref(d)),
           "kdn_chunk_slice")
    return Chunk(chunk.data, d)


def kdn_store_chunk(cache: PagedCache, block_table: torch.Tensor, token_start: int,
                    num_tokens: int, out: Chunk, stream=None, max_workgroups: int = 0) -> Chunk:
    """max_workgroups > 0 goes through kdn_store_chunk_opts (a capped launch)."""
    assert block_table.dtype == torch.int32 and block_table.is_contiguous()
    cd = cache.desc()
    if max_workgroups:
        opts = LaunchOpts(int(max_workgroups))
        _check(lib().kdn_store_chunk_opts(C.byref(cd), block_table.data_ptr(), block_table.numel(),
                                          token_start, num_tokens, C.byref(out.desc), C.byref(opts),
                                          _stream(stream)), "kdn_store_chunk_opts")
        return out
    _check(lib().kdn_store_chunk(C.byref(cd), block_table.data_ptr(), block_table.numel(),
                                 token_start, num_tokens, C.byref(out.desc), _stream(stream)),
           "kdn_store_chunk")
    return out


def kdn_store_tokens(cache: PagedCache, block_table: torch.Tensor, tokens: torch.Tensor,
                     out: Chunk, stream=None) -> Chunk:
    assert block_table.dtype == torch.int32 and block_table.is_contiguous()
    assert tokens.dtype == torch.int32 and tokens.is_contiguous() and tokens.is_cuda
    cd = cache.desc()
    _check(lib().kdn_store_tokens(C.byref(cd), block_table.data_ptr(), block_table.numel(),
                                  tokens.data_ptr(), tokens.numel(), C.byref(out.desc), _stream(stream)),
           "kdn_store_tokens")
    return out


def alloc_host_chunk(cache: PagedCache, num_tokens: int, fmt: int) -> Chunk:
    """A chunk buffer in pinned host memory (a pinned torch tensor)."""
    L, _, _, H, D = cache.shape
    n = kdn_chunk_bytes(L, H, D, num_tokens, fmt)
    if n == 0:
        raise KdnError(EINVAL, "kdn_chunk_bytes")
    data = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    d = ChunkDesc()
    _check(lib().kdn_chunk_init(C.byref(d), data.data_ptr(), n, fmt, L, H, D, num_tokens), "kdn_chunk_init")
    return Chunk(data, d)


def kdn_store_staging_bytes(cache: PagedCache, num_tokens: int, fmt: int, layers_per_stage: int) -> int:
    cd = cache.desc()
    return int(lib().kdn_store_staging_bytes(C.byref(cd), num_tokens, fmt, layers_per_stage))


def kdn_store_to_host(cache: PagedCache, block_table: torch.Tensor, token_start: int, num_tokens: int,
                      out_host: Chunk, staging: torch.Tensor, layers_per_stage: int, stream=None) -> Chunk:
    assert block_table.dtype == torch.int32 and block_table.is_contiguous()
    assert staging.is_cuda and staging.is_contiguous() and not out_host.data.is_cuda
    cd = cache.desc()
    _check(lib().kdn_store_to_host(C.byref(cd), block_table.data_ptr(), block_table.numel(), token_start,
                                   num_tokens, C.byref(out_host.desc), staging.data_ptr(),
                                   staging.numel() * staging.element_size(), layers_per_stage,
                                   _stream(stream)), "kdn_store_to_host")
    return out_host


def kdn_load_chunk(chunk: Chunk, cache: PagedCache, block_table: torch.Tensor,
                   dest_token_start: int = 0, stream=None) -> None:
    assert block_table.dtype == torch.int32 and block_table.is_contiguous()
    cd = cache.desc()
    _check(lib().kdn_load_chunk(C.byref(chunk.desc), C.byref(cd), block_table.data_ptr(),
                                block_table.numel(), dest_token_start, _stream(stream)),
           "kdn_load_chunk")


def _chunk_array(chunks):
    arr = (ChunkDesc * len(chunks))()
    for i, c in enumerate(chunks):
        arr[i] = c.desc
    return arr


def kdn_compose(chunks, offsets, cache: PagedCache, block_table: torch.Tensor, rope_base: float,
                dest_token_start: int = 0, stream=None, max_workgroups: int = 0, spec=None) -> None:
    """max_workgroups > 0 (a capped launch) or spec (a pair from rope_spec()) go through
    kdn_compose_opts."""
    assert block_table.dtype == torch.int32 and block_table.is_contiguous()
    assert len(chunks) == len(offsets)
    cd = cache.desc()
    arr = _chunk_array(chunks)
    off = (C.c_int32 * len(offsets))(*[int(o) for o in offsets])
    if max_workgroups or spec is not None:
        opts = LaunchOpts(int(max_workgroups))
        _check(lib().kdn_compose_opts(arr, off, len(chunks), C.byref(cd), block_table.data_ptr(),
                                      block_table.numel(), dest_token_start, float(rope_base),
                                      C.byref(spec[0]) if spec is not None else None, C.byref(opts),
                                      _stream(stream)), "kdn_compose_opts")
        return
    _check(lib().kdn_compose(arr, off, len(chunks), C.byref(cd), block_table.data_ptr(),
                             block_table.numel(), dest_token_start, float(rope_base),
                             _stream(stream)), "kdn_compose")


class BatchPlan:
    """Marshalled arguments of a batched compose, reusable across calls."""

    def __init__(self, requests):
        """requests: list of (chunks, offsets, block_table, dest_token_start)."""
        self._keep = []
        self.arr = (RequestDesc * len(requests))()
        for i, (chunks, offsets, bt, dest) in enumerate(requests):
            assert bt.dtype == torch.int32 and bt.is_contiguous() and len(chunks) == len(offsets)
            ca = _chunk_array(chunks)
            oa = (C.c_int32 * len(offsets))(*[int(o) for o in offsets])
            self._keep += [ca, oa, bt, chunks]
            self.arr[i] = RequestDesc(ca, oa, len(chunks), bt.data_ptr(), bt.numel(), int(dest))
        self.n = len(requests)


def kdn_compose_batch(plan_or_requests, cache: PagedCache, rope_base: float, stream=None) -> None:
    plan = plan_or_requests if isinstance(plan_or_requests, BatchPlan) else BatchPlan(plan_or_requests)
    cd = cache.desc()
    _check(lib().kdn_compose_batch(plan.arr, plan.n, C.byref(cd), float(rope_base), _stream(stream)),
           "kdn_compose_batch")


def kdn_compose_batch_static(plan_or_requests, cache: PagedCache, rope_base: float, stream=None) -> None:
    """kdn_compose_batch through the entry point that allocates nothing (its tables live in
    the library's static scratch array)."""
    plan = plan_or_requests if isinstance(plan_or_requests, BatchPlan) else BatchPlan(plan_or_requests)
    cd = cache.desc()
    _check(lib().kdn_compose_batch_static(plan.arr, plan.n, C.byref(cd), float(rope_base), _stream(stream)),
           "kdn_compose_batch_static")


class PlacementDesc(C.Structure):
    _fields_ = [("request", C.c_int32), ("chunk", C.c_int32), ("fmt", C.c_int32), ("launch", C.c_int32),
                ("dest_token", C.c_int32), ("num_tokens", C.c_int32), ("offset", C.c_int32),
                ("shares_rows", C.c_int32), ("follows", C.c_int32)]


def kdn_compose_plan(plan_or_requests, cache: PagedCache):
    """The placements of a batched compose, in kernel order, as dicts of the C record's fields."""
    plan = plan_or_requests if isinstance(plan_or_requests, BatchPlan) else BatchPlan(plan_or_requests)
    cd = cache.desc()
    n = C.c_int32(0)
    _check(lib().kdn_compose_plan(plan.arr, plan.n, C.byref(cd), None, 0, C.byref(n)), "kdn_compose_plan")
    out = (PlacementDesc * n.value)()
    _check(lib().kdn_compose_plan(plan.arr, plan.n, C.byref(cd), out, n.value, C.byref(n)), "kdn_compose_plan")
    return [{f: getattr(r, f) for f, _ in PlacementDesc._fields_} for r in out]


def kdn_tile_tokens(cache: PagedCache) -> int:
    """Tokens per tile for this cache (the modulus of the chaining rule of kdn_compose_plan)."""
    cd = cache.desc()
    return int(lib().kdn_tile_tokens(C.byref(cd)))


def rope_spec(base: float = 10000.0, inv_freq=None, rot_dim: int = 0,
              pairing: int = ROPE_HALF_SPLIT):
    """Marshal a RoPE variant; returns (RopeSpecDesc, keep-alive)."""
    arr = None
    if inv_freq is not None:
        arr = (C.c_double * len(inv_freq))(*[float(f) for f in inv_freq])
    d = RopeSpecDesc(float(base), C.cast(arr, C.POINTER(C.c_double)) if arr is not None else None,
                     int(rot_dim), int(pairing))
    return d, arr


def kdn_compose_rope(chunks, offsets, cache: PagedCache, block_table: torch.Tensor, spec,
                     dest_token_start: int = 0, stream=None) -> None:
    """spec: the pair returned by rope_spec()."""
    assert block_table.dtype == torch.int32 and block_table.is_contiguous()
    assert len(chunks) == len(offsets)
    cd = cache.desc()
    arr = _chunk_array(chunks)
    off = (C.c_int32 * len(offsets))(*[int(o) for o in offsets])
    _check(lib().kdn_compose_rope(arr, off, len(chunks), C.byref(cd), block_table.data_ptr(),
                                  block_table.numel(), dest_token_start, C.byref(spec[0]),
                                  _stream(stream)), "kdn_compose_rope")


def kdn_compose_batch_rope(plan_or_requests, cache: PagedCache, spec, stream=None) -> None:
    plan = plan_or_requests if isinstance(plan_or_requests, BatchPlan) else BatchPlan(plan_or_requests)
    cd = cache.desc()
    _check(lib().kdn_compose_batch_rope(plan.arr, plan.n, C.byref(cd), C.byref(spec[0]), _stream(stream)),
           "kdn_compose_batch_rope")


def kdn_patch_rows(rows: torch.Tensor, tokens: torch.Tensor, cache: PagedCache,
                   block_table: torch.Tensor, stream=None) -> None:
    """rows: bf16 [L][2][n][H][D] on the device; tokens: int32 [n] on the device."""
    L, _, _, H, D = cache.shape
    assert rows.dtype == torch.bfloat16 and rows.is_contiguous() and rows.is_cuda
    assert tokens.dtype == torch.int32 and tokens.is_contiguous() and tokens.is_cuda
    assert tuple(rows.shape) == (L, 2, tokens.numel(), H, D)
    assert block_table.dtype == torch.int32 and block_table.is_contiguous()
    cd = cache.desc()
    _check(lib().kdn_patch_rows(rows.data_ptr(), tokens.data_ptr(), tokens.numel(), C.byref(cd),
                                block_table.data_ptr(), block_table.numel(), _stream(stream)),
           "kdn_patch_rows")


def pinned_host_copy(chunk: Chunk) -> Chunk:
    """The same stored bytes in pinned host memory (a torch pinned tensor), described as
    a chunk whose data pointer is a host address, for kdn_compose_from_host."""
    host = torch.empty(chunk.data.shape, dtype=torch.uint8, pin_memory=True)
    host.copy_(chunk.data)
    d = ChunkDesc.from_buffer_copy(chunk.desc)
    d.data = host.data_ptr()
    return Chunk(host, d)


def kdn_staging_bytes(chunks, layers_per_stage: int) -> int:
    return int(lib().kdn_staging_bytes(_chunk_array(chunks), len(chunks), layers_per_stage))


class StageCopyDesc(C.Structure):
    _fields_ = [("chunk", C.c_int32), ("rows", C.c_int32), ("src_offset", C.c_uint64),
                ("src_pitch", C.c_uint64), ("width", C.c_uint64), ("dst_offset", C.c_uint64)]


def kdn_host_stage_plan(chunks, layers_per_stage: int, stage: int):
    """(copies, view_offsets): the link transfers of one stage and where each view's staged
    image starts; each copy is a dict of the C record's fields."""
    arr, n = _chunk_array(chunks), C.c_int32(0)
    _check(lib().kdn_host_stage_plan(arr, len(chunks), layers_per_stage, stage, None, 0, C.byref(n), None),
           "kdn_host_stage_plan")
    out = (StageCopyDesc * n.value)()
    views = (C.c_uint64 * len(chunks))()
    _check(lib().kdn_host_stage_plan(arr, len(chunks), layers_per_stage, stage, out, n.value, C.byref(n), views),
           "kdn_host_stage_plan")
    return ([{f: getattr(c, f) for f, _ in StageCopyDesc._fields_} for c in out], list(views))


def kdn_compose_from_host(chunks, offsets, cache: PagedCache, block_table: torch.Tensor,
                          rope_base: float, staging: torch.Tensor, layers_per_stage: int,
                          dest_token_start: int = 0, stream=None, stage_events=None) -> None:
    """stage_events: optional list of torch.cuda.Event, one per stage, each recorded at least
    once before (torch creates the HIP event on first record); the library records event s
    behind the kernels of stage s."""
    assert block_table.dtype == torch.int32 and block_table.is_contiguous()
    assert len(chunks) == len(offsets) and staging.is_cuda and staging.is_contiguous()
    cd = cache.desc()
    arr = _chunk_array(chunks)
    off = (C.c_int32 * len(offsets))(*[int(o) for o in offsets])
    if stage_events is None:
        _check(lib().kdn_compose_from_host(arr, off, len(chunks), C.byref(cd), block_table.data_ptr(),
                                           block_table.numel(), dest_token_start, float(rope_base),
                                           staging.data_ptr(), staging.numel() * staging.element_size(),
                                           layers_per_stage, _stream(stream)), "kdn_compose_from_host")
        return
    evs = (C.c_void_p * len(stage_events))(*[int(e.cuda_event) for e in stage_events])
    _check(lib().kdn_compose_from_host_staged(arr, off, len(chunks), C.byref(cd), block_table.data_ptr(),
                                              block_table.numel(), dest_token_start, float(rope_base),
                                              staging.data_ptr(), staging.numel() * staging.element_size(),
                                              layers_per_stage, evs, len(stage_events), _stream(stream)),
           "kdn_compose_from_host_staged")


def kdn_rope_prepare(rope_base: float, head_dim: int, offsets) -> None:
    off = (C.c_int32 * len(offsets))(*[int(o) for o in offsets])
    _check(lib().kdn_rope_prepare(float(rope_base), head_dim, off, len(offsets)), "kdn_rope_prepare")


def kdn_rope_prepare_spec(spec, head_dim: int, offsets) -> None:
    """spec: the pair returned by rope_spec()."""
    off = (C.c_int32 * len(offsets))(*[int(o) for o in offsets])
    _check(lib().kdn_rope_prepare_spec(C.byref(spec[0]), head_dim, off, len(offsets)), "kdn_rope_prepare_spec")


def kdn_rope_release() -> None:
    _check(lib().kdn_rope_release(), "kdn_rope_release")


def kdn_validate_block_table(block_table: torch.Tensor, num_blocks: int, stream=None) -> int:
    """Returns the status (OK or ERANGE) instead of raising."""
    return int(lib().kdn_validate_block_table(block_table.data_ptr(), block_table.numel(),
                                              num_blocks, _stream(stream)))


def kdn_probe_stream(small: torch.Tensor, big: torch.Tensor, tiles: int, tile_ids: torch.Tensor | None = None,
                     tile_kib: int = 32, direction: int = 0, max_workgroups: int = 0, stream=None) -> None:
    """The streaming yardstick: per tile, tile_kib/2 KiB of `small` and tile_kib KiB of `big`
    (tile i of `small` with tile tile_ids[i] of `big` when ids are given; the ids are the caller's
    to keep inside `big`: nothing here reads them back, a call only enqueues).  direction 0 reads
    `small` and writes `big` (load, compose), direction 1 the reverse (store), direction 2 only
    writes `big`, direction 3 only reads it."""
    assert small.is_cuda and big.is_cuda and small.is_contiguous() and big.is_contiguous()
    assert small.numel() * small.element_size() >= tiles * tile_kib * 512
    if tile_ids is None:
        assert big.numel() * big.element_size() >= tiles * tile_kib * 1024
    else:
        assert tile_ids.dtype == torch.int32 and tile_ids.is_cuda and tile_ids.numel() >= tiles
    _check(lib().kdn_probe_stream(small.data_ptr(), big.data_ptr(), tile_ids.data_ptr() if tile_ids is not None else None,
                                  tiles, tile_kib, direction, max_workgroups, _stream(stream)), "kdn_probe_stream")


def kdn_f32_to_bf16(x: torch.Tensor, out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    assert x.dtype == torch.float32 and x.is_contiguous()
    if out is None:
        out = torch.empty(x.shape, dtype=torch.bfloat16, device=x.device)
    _check(lib().kdn_f32_to_bf16(x.data_ptr(), out.data_ptr(), x.numel(), _stream(stream)),
           "kdn_f32_to_bf16")
    return out


# ------------------------------------------------------------------ striped device arena
def kdn_arena_create(nbytes: int, granule_mib: int = 0) -> dict:
    """Create the current device's arena (include/kdn_arena.h); returns what was measured."""
    info = ArenaInfo()
    _check(lib().kdn_arena_create(nbytes, granule_mib, C.byref(info)), "kdn_arena_create")
    return info.as_dict()


def kdn_arena_query() -> dict:
    info = ArenaInfo()
    _check(lib().kdn_arena_query(C.byref(info)), "kdn_arena_query")
    return info.as_dict()


def kdn_arena_alloc(nbytes: int) -> int:
    p = C.c_void_p()
    _check(lib().kdn_arena_alloc(nbytes, C.byref(p)), "kdn_arena_alloc")
    return int(p.value)


def kdn_arena_free(ptr: int) -> None:
    _check(lib().kdn_arena_free(ptr), "kdn_arena_free")


def kdn_arena_destroy() -> None:
    """Every tensor from arena_tensor must be gone (or never used again) before this."""
    _check(lib().kdn_arena_destroy(), "kdn_arena_destroy")


class _ArenaBlock:
    """Owns one kdn_arena_alloc block; torch holds it for as long as a tensor views the memory."""

    def __init__(self, nbytes: int):
        self.ptr = kdn_arena_alloc(nbytes)
        self.__cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (self.ptr, False),
                                         "version": 2}

    def __del__(self):
        ptr, self.ptr = getattr(self, "ptr", 0), 0
        if ptr and _lib is not None:
            _lib.kdn_arena_free(ptr)     # ENOTFOUND after kdn_arena_destroy: nothing left to give back


def arena_tensor(nbytes: int) -> torch.Tensor:
    """A uint8 tensor of nbytes on the current device whose memory is cut from the arena; the
    block goes back to the arena when the last tensor that views it is collected."""
    return torch.as_tensor(_ArenaBlock(nbytes), device="cuda")


def kdn_shutdown() -> None:
    _check(lib().kdn_shutdown(), "kdn_shutdown")


def kdn_version() -> str:
    return lib().kdn_version().decode()


# ------------------------------------------------------------------ text-keyed index
def _ids_arg(token_ids):
    import numpy as np
    a = np.ascontiguousarray(token_ids, dtype=np.int32)
    return a, a.ctypes.data, int(a.size)


def kdn_pool_hash(token_ids) -> int:
    a, ptr, n = _ids_arg(token_ids)
    return int(lib().kdn_pool_hash(ptr, n))


class Pool:
    """Binding of the kdn_pool_* calls: token ids -> chunk descriptor, byte-bounded."""

    def __init__(self, capacity_bytes: int, policy: int = 0):
        self._h = C.c_void_p()
        _check(lib().kdn_pool_create(capacity_bytes, policy, C.byref(self._h)), "kdn_pool_create")

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.kdn_pool_destroy(self._h)
            self._h = None

    def lookup(self, token_ids):
        a, ptr, n = _ids_arg(token_ids)
        out = ChunkDesc()
        st = lib().kdn_pool_lookup(self._h, ptr, n, C.byref(out))
        if st == ENOTFOUND:
            return None
        _check(st, "kdn_pool_lookup")
        return out

    def insert(self, token_ids, chunk_desc: ChunkDesc, max_evicted: int = 64):
        a, ptr, n = _ids_arg(token_ids)
        ev = (ChunkDesc * max(max_evicted, 1))()
        cnt = C.c_int32(0)
        _check(lib().kdn_pool_insert(self._h, ptr, n, C.byref(chunk_desc), ev if max_evicted else None,
                                     max_evicted, C.byref(cnt)), "kdn_pool_insert")
        return [ChunkDesc.from_buffer_copy(ev[i]) for i in range(cnt.value)]

    def remove(self, token_ids):
        a, ptr, n = _ids_arg(token_ids)
        out = ChunkDesc()
        st = lib().kdn_pool_remove(self._h, ptr, n, C.byref(out))
        if st == ENOTFOUND:
            return None
        _check(st, "kdn_pool_remove")
        return out

    def stats(self) -> PoolStats:
        out = PoolStats()
        _check(lib().kdn_pool_get_stats(self._h, C.byref(out)), "kdn_pool_get_stats")
        return out
