"""Shared plumbing of the GPU parity tests: host <-> device copies and comparisons.
No arithmetic of the method lives here."""
import numpy as np
import torch

from oracle import kdn_oracle as O
from paper_2409_13761_amd import kdn, synth

RAW, INT8, INT4, FP8 = 0, 1, 2, 3
K_TOL = 1e-2        # absolute tolerance on RoPE-shifted bf16 keys for N(0,1) inputs


def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bits_of(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def f32_of_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def host_cache(seed, L, nb, bs, H, D) -> O.PagedCache:
    return O.PagedCache(synth.normal_bf16(seed, (L, nb, bs, H, D), stream=10),
                        synth.normal_bf16(seed, (L, nb, bs, H, D), stream=11))


def dev_cache(h: O.PagedCache) -> kdn.PagedCache:
    return kdn.PagedCache(to_dev_bf16(h.k), to_dev_bf16(h.v))


def dev_table(bt: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bt, dtype=np.int32)).cuda()


def chunk_to_dev(h: O.Chunk) -> kdn.Chunk:
    data = torch.from_numpy(h.data).cuda()
    c = kdn.chunk_from_buffer(data, h.fmt, h.L, h.H, h.D, h.Tp)
    if h.tok_start != 0 or h.T != h.Tp:
        c = c.slice(h.tok_start, h.T)
    return c


def assert_chunk_equal(dev: kdn.Chunk, host: O.Chunk):
    torch.cuda.synchronize()
    got = dev.data.cpu().numpy()
    assert got.nbytes == host.data.nbytes
    if not np.array_equal(got, host.data):
        bad = np.flatnonzero(got != host.data)
        raise AssertionError("stored chunk differs in %d bytes, first at %d" % (bad.size, bad[0]))


def assert_cache_equal(dev: kdn.PagedCache, host: O.PagedCache, k_exact=True):
    """V, and K where no rotation applies, must match bit for bit.  Rotated K must be
    within K_TOL; with k_exact the stricter design target (no differing bit) is
    asserted as well."""
    torch.cuda.synchronize()
    gv, gk = bits_of(dev.v), bits_of(dev.k)
    assert np.array_equal(gv, host.v), "V differs"
    if np.array_equal(gk, host.k):
        return 0.0, 0
    diff = np.abs(f32_of_bits(gk).astype(np.float64) - f32_of_bits(host.k).astype(np.float64))
    n_diff = int(np.count_nonzero(gk != host.k))
    mx = float(np.nanmax(diff))
    assert mx <= K_TOL, "K differs by %g in %d elements" % (mx, n_diff)
    assert not k_exact, "K within tolerance but %d elements differ (max %g)" % (n_diff, mx)
    return mx, n_diff
