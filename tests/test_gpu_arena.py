"""The striped device arena on the GPU: what kdn_arena_create reports, the block list, and
store / load / compose on chunks and a paged pool cut from it, against the oracle."""
import gc
import math

import numpy as np
import pytest
import torch

import notes
from helpers import INT8, RAW, assert_cache_equal, assert_chunk_equal, dev_table, host_cache
from oracle import kdn_oracle as O
from paper_2409_13761_amd import kdn, synth

pytestmark = pytest.mark.gpu

GIB = 1 << 30
ARENA_BYTES = 3 * GIB + 5                      # rounded up to whole granules


@pytest.fixture(scope="module")
def arena():
    gc.collect()
    torch.cuda.empty_cache()
    torch.zeros(1, device="cuda")
    print("[arena] creating %d bytes" % ARENA_BYTES, flush=True)
    info = kdn.kdn_arena_create(ARENA_BYTES)
    notes.note("[arena] %d granules of %d MiB drawn with stride %d from %d free ones; scattered tile writes over the "
               "first GiB %.0f GB/s, over as much memory in the driver's order %.0f GB/s; created in %.2f s"
               % (info["bytes"] // info["granule"], info["granule"] >> 20, info["stride"], info["free_granules"],
                  info["striped_gbs"], info["packed_gbs"], info["seconds"]))
    yield info
    gc.collect()
    torch.cuda.synchronize()
    kdn.kdn_arena_destroy()
    with pytest.raises(kdn.KdnError) as e:
        kdn.kdn_arena_query()
    assert e.value.status == kdn.ENOTFOUND


def test_what_create_reports_is_consistent(arena):
    g = 16 << 20
    assert arena["granule"] == g and arena["bytes"] == (ARENA_BYTES + g - 1) // g * g
    assert arena["in_use"] == 0 and arena["largest_free"] == arena["bytes"]
    n, N, stride = arena["bytes"] // g, arena["free_granules"], arena["stride"]
    assert N >= n and 0 < stride < N and math.gcd(stride, N) == 1      # no free granule is taken twice
    assert abs(stride / N - 0.382) < 0.01 or N < 1000                  # neighbours lie 38% of the free memory apart
    assert arena["seconds"] < 60
    # both rates were measured and are rates of this device; which is higher is the bench's business
    assert 1000 < arena["striped_gbs"] < 8000 and 1000 < arena["packed_gbs"] < 8000
    with pytest.raises(kdn.KdnError) as e:                         # one arena per device
        kdn.kdn_arena_create(GIB)
    assert e.value.status == kdn.EINVAL


def test_blocks_are_disjoint_aligned_and_join_up_again_when_freed(arena):
    total = arena["bytes"]
    sizes = [1, 4096, 4097, 10 << 20, 100 << 20, (16 << 20) - 1, 333333]
    ptrs = [kdn.kdn_arena_alloc(s) for s in sizes]
    spans = sorted((p, p + (s + 4095) // 4096 * 4096) for p, s in zip(ptrs, sizes))
    assert all(p % 4096 == 0 for p in ptrs)
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
    assert spans[-1][1] - spans[0][0] <= total
    q = kdn.kdn_arena_query()
    assert q["in_use"] == sum(b - a for a, b in spans) and q["largest_free"] == total - q["in_use"]
    for bad, status in ((total + 1, kdn.ESIZE), (q["largest_free"] + 1, kdn.ESIZE), (0, kdn.EINVAL)):
        with pytest.raises(kdn.KdnError) as e:
            kdn.kdn_arena_alloc(bad)
        assert e.value.status == status
    with pytest.raises(kdn.KdnError) as e:                         # an address inside a block is not a block
        kdn.kdn_arena_free(ptrs[3] + 4096)
    assert e.value.status == kdn.EINVAL
    # free every other block: the holes are reused first fit, and do not join across a live block
    for i in (1, 3, 5):
        kdn.kdn_arena_free(ptrs[i])
    again = kdn.kdn_arena_alloc(10 << 20)
    assert again == ptrs[3]
    small = kdn.kdn_arena_alloc(4096)
    assert small == ptrs[1]
    for p in (again, small, ptrs[0], ptrs[2], ptrs[4], ptrs[6]):
        kdn.kdn_arena_free(p)
    with pytest.raises(kdn.KdnError) as e:                         # freed twice
        kdn.kdn_arena_free(ptrs[0])
    assert e.value.status == kdn.EINVAL
    q = kdn.kdn_arena_query()
    assert q["in_use"] == 0 and q["largest_free"] == total         # every stretch joined up again
    assert kdn.kdn_arena_alloc(total) == spans[0][0]
    kdn.kdn_arena_free(spans[0][0])


def test_a_tensor_holds_its_block_until_it_is_collected(arena):
    t = kdn.arena_tensor(5 << 20)
    assert t.is_cuda and t.dtype == torch.uint8 and t.numel() == 5 << 20
    view = t[4096:8192].view(torch.bfloat16)
    del t
    gc.collect()
    assert kdn.kdn_arena_query()["in_use"] == 5 << 20              # the view keeps the block
    view.fill_(1.5)
    assert float(view.float().sum()) == 1.5 * 2048
    del view
    gc.collect()
    assert kdn.kdn_arena_query()["in_use"] == 0


def _arena_cache(h: O.PagedCache) -> kdn.PagedCache:
    out = []
    for bits in (h.k, h.v):
        t = kdn.arena_tensor(bits.nbytes).view(torch.bfloat16).view(bits.shape)
        t.copy_(torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16))
        out.append(t)
    return kdn.PagedCache(*out)


@pytest.mark.parametrize("fmt", [INT8, RAW])
def test_store_load_compose_on_arena_memory_equal_the_oracle(arena, fmt):
    """Chunk and pool both larger than a stripe, so every kernel crosses granule boundaries."""
    L, bs, H, D, T = 4, 16, 8, 128, 2048
    nb = 3 * (T // bs) + 7
    print("[arena] parity fmt %d: chunk %d bytes, pool planes of %d bytes" %
          (fmt, kdn.kdn_chunk_bytes(L, H, D, T, fmt), L * nb * bs * H * D * 2), flush=True)
    hc = host_cache(77, L, nb, bs, H, D)
    src, dst_load, dst_comp = synth.disjoint_block_tables(78, nb, [T // bs] * 3)
    dc = _arena_cache(hc)
    chunk = kdn.alloc_chunk(dc, T, fmt, arena=True)
    assert kdn.kdn_arena_query()["in_use"] >= chunk.data.numel() + 2 * dc.k.numel() * 2
    kdn.kdn_store_chunk(dc, dev_table(src), 0, T, chunk)
    h = O.store(hc, src, 0, T, fmt)
    assert_chunk_equal(chunk, h)
    kdn.kdn_load_chunk(chunk, dc, dev_table(dst_load), 0)
    O.load(h, hc, dst_load, 0)
    assert_cache_equal(dc, hc)
    parts = [(0, 640), (640, 1408)]                                # two slices, the second shifted by RoPE
    kdn.kdn_compose([chunk.slice(a, n) for a, n in parts], [0, 640], dc, dev_table(dst_comp), 500000.0)
    O.compose([h.slice(a, n) for a, n in parts], [0, 640], hc, dst_comp, 500000.0)
    assert_cache_equal(dc, hc)
