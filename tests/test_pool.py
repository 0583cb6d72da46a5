"""The text-keyed chunk index: the Python reference model against hand-worked traces, and
the library's C++ index against the reference on seeded popularity-skewed traces.
No GPU is needed: the index holds descriptors only."""
import ctypes as C
import os

import numpy as np
import pytest

from oracle.pool_oracle import LFU, LRU, PoolOracle
from paper_2409_13761_amd import build, kdn, synth

HERE = os.path.dirname(os.path.abspath(__file__))


# ------------------------------------------------------------------ the reference model
def test_reference_model_on_hand_worked_traces():
    n = 0
    for line in open(os.path.join(HERE, "golden", "pool_traces.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        policy, cap, seq, want, resident = (p.strip() for p in line.split("|"))
        pool = PoolOracle(int(cap), LRU if policy == "LRU" else LFU)
        got = []
        for key in seq.split():
            hit = pool.lookup(key) is not None
            got.append(int(hit))
            if not hit:
                assert pool.insert(key, key, 1) is not None
        assert got == [int(x) for x in want.split()], line
        assert sorted(k[0] if isinstance(k, tuple) and len(k) == 1 else "".join(k) for k in pool.entries) \
            == sorted(resident.split()), line
        n += 1
    assert n >= 4


def test_reference_model_invariants_on_a_skewed_trace():
    draws = synth.zipf_distinct_draws(7, 400, 1, 64)[:, 0]
    for policy in (LRU, LFU):
        pool = PoolOracle(10 * 100, policy)
        for c in draws:
            key = (int(c),)
            if pool.lookup(key) is None:
                ev = pool.insert(key, int(c), 100)
                assert ev is not None and len(ev) <= 1
            assert pool.bytes <= pool.capacity and len(pool.entries) <= 10
        assert pool.hits + pool.misses == len(draws)
        assert pool.inserts == pool.misses and pool.evictions == pool.inserts - len(pool.entries)
        # a popularity-skewed trace must hit far more often than 10/64 uniform residency would
        assert pool.hits / len(draws) > 0.35


# ------------------------------------------------------------------ the library
@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(build.LIB_PATH):
        build.build_library()
    return kdn.lib()


def _ids(c, n=24):
    rng = np.random.default_rng(1000 + int(c))
    return np.ascontiguousarray(rng.integers(0, 128000, size=n), dtype=np.int32)


def _chunk(tag, nbytes):
    return kdn.ChunkDesc(0x100000 + 0x1000 * int(tag), nbytes, 1, 2, 4, 64, 16, 0, 16)


@pytest.mark.parametrize("policy", [LRU, LFU])
def test_library_index_follows_the_reference_on_zipf_traces(lib, policy):
    sizes = {c: 100 + 37 * (c % 5) for c in range(96)}            # unequal chunk sizes
    cap = 1500
    pool = kdn.Pool(cap, policy)
    ref = PoolOracle(cap, policy)
    draws = synth.zipf_distinct_draws(11 + policy, 1500, 1, 96)[:, 0]
    for step, c in enumerate(draws):
        c = int(c)
        got = pool.lookup(_ids(c))
        want = ref.lookup(tuple(_ids(c)))
        assert (got is None) == (want is None), "step %d" % step
        if got is None:
            ev = pool.insert(_ids(c), _chunk(c, sizes[c]))
            ev_ref = ref.insert(tuple(_ids(c)), c, sizes[c])
            assert [(e.data - 0x100000) // 0x1000 for e in ev] == ev_ref, "step %d" % step
        else:
            assert (got.data - 0x100000) // 0x1000 == c and got.bytes == sizes[c]
        if step % 100 == 0:                                       # occasionally re-insert a resident key
            ev = pool.insert(_ids(c), _chunk(c, sizes[c]))
            ev_ref = ref.insert(tuple(_ids(c)), c, sizes[c])
            assert [(e.data - 0x100000) // 0x1000 for e in ev] == ev_ref
    st = pool.stats()
    assert (st.hits, st.misses, st.inserts, st.evictions) == (ref.hits, ref.misses, ref.inserts, ref.evictions)
    assert st.bytes == ref.bytes <= cap and st.entries == len(ref.entries)


def test_library_index_edge_cases(lib):
    pool = kdn.Pool(300, LRU)
    a, b = _ids(1), _ids(2)
    assert pool.lookup(a) is None
    assert pool.insert(a, _chunk(1, 200)) == []
    with pytest.raises(kdn.KdnError) as e:                        # larger than the whole pool
        pool.insert(b, _chunk(2, 301))
    assert e.value.status == kdn.ESIZE
    with pytest.raises(kdn.KdnError) as e:                        # would need an eviction, none allowed
        pool.insert(b, _chunk(2, 200), max_evicted=0)
    assert e.value.status == kdn.ESIZE
    assert pool.lookup(a) is not None and pool.stats().entries == 1
    ev = pool.insert(b, _chunk(2, 200))
    assert len(ev) == 1 and ev[0].bytes == 200 and pool.lookup(a) is None
    # same hash bucket is not assumed: a prefix of the ids is a different key
    assert pool.lookup(b[:-1]) is None
    assert pool.remove(b).bytes == 200 and pool.remove(b) is None
    assert pool.stats().bytes == 0
    assert kdn.kdn_pool_hash(a) != kdn.kdn_pool_hash(b)
    assert kdn.kdn_pool_hash(a) == kdn.kdn_pool_hash(a.copy())
    p = C.c_void_p()
    assert lib.kdn_pool_create(0, 0, C.byref(p)) == kdn.EINVAL
    assert lib.kdn_pool_create(10, 9, C.byref(p)) == kdn.EINVAL
