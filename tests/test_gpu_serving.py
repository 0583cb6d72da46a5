"""The serving loop over the text-keyed index on the GPU: store on miss, compose on hit.

Each request names a few texts by Zipf popularity.  A text whose KV is resident in the
index is a hit; on a miss its KV is stored from the engine's paged memory (kdn_store_chunk)
into a buffer from the free list and indexed, and what the index evicts goes back to the
free list.  The request's chunks are then composed into its block table (kdn_compose).
Every hit / miss / eviction decision is compared with the reference model of the index,
and the paged cache with the oracle's store and compose replayed from the same trace.
"""
import numpy as np
import pytest
import torch

import notes
from helpers import INT8, assert_cache_equal, dev_cache, dev_table, host_cache
from oracle import kdn_oracle as O
from oracle.pool_oracle import LFU, LRU, PoolOracle
from paper_2409_13761_amd import kdn, synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("policy", [LRU, LFU])
def test_store_on_miss_compose_on_hit_over_a_zipf_trace(policy):
    L, bs, H, D = 2, 16, 2, 64
    n_texts, per_req, Tc, resident, n_req = 24, 3, 48, 6, 60
    cb = Tc // bs
    nb = n_texts * cb + 2 * per_req * cb + 5                    # 5 blocks nobody may touch
    print("[serving] policy %d: %d requests x %d of %d texts, %d resident" % (policy, n_req, per_req, n_texts, resident),
          flush=True)
    hc = host_cache(401, L, nb, bs, H, D)
    dc = dev_cache(hc)
    tabs = synth.disjoint_block_tables(401, nb, [cb] * n_texts + [per_req * cb] * 2)
    src_tabs, dst_tabs = tabs[:n_texts], tabs[n_texts:]
    d_src = [dev_table(t) for t in src_tabs]
    d_dst = [dev_table(t) for t in dst_tabs]
    text_ids = [np.ascontiguousarray(synth._rng(402, 100 + t).integers(0, 128000, size=Tc), dtype=np.int32)
                for t in range(n_texts)]
    draws = synth.zipf_distinct_draws(403, n_req, per_req, n_texts, 1.0)
    offsets = [0, Tc, 2 * Tc]
    base = 10000.0

    chunk_bytes = kdn.kdn_chunk_bytes(L, H, D, Tc, INT8)
    free = [kdn.alloc_chunk(dc, Tc, INT8) for _ in range(resident + per_req)]     # taken from the front
    by_ptr = {c.data.data_ptr(): c for c in free}
    text_in = {}                                                # buffer address -> text it holds
    index = kdn.Pool(resident * chunk_bytes, policy)
    model = PoolOracle(resident * chunk_bytes, policy)
    stored_h = {}                                               # text -> the oracle's stored chunk
    hits = 0

    for i in range(n_req):
        chunks, hchunks = [], []
        for t in (int(x) for x in draws[i]):
            got = index.lookup(text_ids[t])
            want = model.lookup(text_ids[t])
            assert (got is None) == (want is None), "request %d text %d: hit/miss differs" % (i, t)
            if got is None:
                buf = free.pop(0)
                kdn.kdn_store_chunk(dc, d_src[t], 0, Tc, buf)
                text_in[buf.data.data_ptr()] = t
                evicted = []
                for e in index.insert(text_ids[t], buf.desc):
                    evicted.append(text_in.pop(e.data))         # the text that buffer held
                    free.append(by_ptr[e.data])
                assert evicted == model.insert(text_ids[t], t, chunk_bytes), "request %d text %d: evictions" % (i, t)
                stored_h[t] = O.store(hc, src_tabs[t], 0, Tc, INT8)
                chunks.append(buf)
            else:
                hits += 1
                assert want == t and text_in[got.data] == t, "request %d text %d: wrong chunk" % (i, t)
                chunks.append(by_ptr[got.data])
            hchunks.append(stored_h[t])
        kdn.kdn_compose(chunks, offsets, dc, d_dst[i % 2], base)
        O.compose(hchunks, offsets, hc, dst_tabs[i % 2], base)
        if i % 10 == 9 or i == n_req - 1:
            assert_cache_equal(dc, hc)
            for c, h in zip(chunks, hchunks):                   # the chunks the request read are the oracle's
                assert np.array_equal(c.data.cpu().numpy(), h.data)
    st = index.stats()
    assert (st.hits, st.misses, st.inserts, st.evictions) == (model.hits, model.misses, model.inserts, model.evictions)
    assert st.hits == hits and st.hits + st.misses == n_req * per_req
    assert st.entries == len(model.entries) <= resident and st.bytes == model.bytes
    assert len(free) + len(text_in) == resident + per_req
    rate = st.hits / (st.hits + st.misses)
    notes.note("[serving] policy %d: %d requests, hit rate %.3f, %d evictions: every decision equal to the reference "
               "model's, paged cache equal to the oracle's replay" % (policy, n_req, rate, st.evictions))
    assert 0.2 < rate < 0.95                                    # the trace exercises both branches
