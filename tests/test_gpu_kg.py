"""GPU parity of the knowledge-graph augmentation: logical edges against the oracle's (exact), and the search with
entity branches (Section 4.2.3, Algorithm 2) replayed by the oracle on the GPU's own scores (ids, scores and the
number of scored documents bit for bit)."""
import time

import numpy as np
import pytest
import torch

import oracle as O
from paper_2511_00855_amd import binding as B
from paper_2511_00855_amd.synth import make_entity_graph, make_workload

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def shard():
    w = make_workload("tiny", seed=27, n=3000, nq=40)
    docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
    ix = B.Index.build(docs, B.build_params(w.degree))
    kgs = make_entity_graph(3000, 40, seed=5, n_ent=400)
    kgs.q_ent[::7] = -1                                   # some queries name no entity
    kgs.q_ent[3, 0], kgs.q_ent[3, 1] = -1, kgs.q_ent[3, 0]   # an unused slot before a used one
    D = O.encode_docs(w.docs); Q = O.VS(w.queries)
    sem, _, _, ent = [t.cpu().numpy() for t in ix.export_graph()]
    wq = np.random.default_rng(2).uniform(0.1, 1.0, (qs.n, 3)).astype(np.float32)
    table = ix.hybrid_scores(qs, np.tile(np.arange(docs.n, dtype=np.int32), (qs.n, 1)), wq).cpu().numpy()[:, :, 3]
    yield w, docs, qs, ix, kgs, D, Q, sem, ent, wq, table
    ix.close()


def test_logical_edges_match_the_oracle(shard):
    w, docs, qs, ix, kgs, D, Q, sem, ent, wq, table = shard
    with pytest.raises(RuntimeError, match="no knowledge graph"):
        ix.search_batch_entities(qs, 5, 16, kgs.q_ent, 0.5)
    for cap in (4, 16):
        _say(f"logical edges, at most {cap} per document")
        ix.set_knowledge_graph(kgs, le_cap=cap)
        le, cnt, en_ip, en = [t.cpu().numpy() for t in ix.export_logical_edges()]
        ole, ocnt, oen_ip, oen = O.logical_edges(kgs, docs.n, cap)
        assert np.array_equal(en_ip, oen_ip) and np.array_equal(en, oen)
        assert np.array_equal(cnt, ocnt) and np.array_equal(le, ole)
        assert (cnt == cap).any() and (cnt < cap).any()
    bad = make_entity_graph(3000, 4, seed=5, n_ent=400)
    bad.doc_ent = bad.doc_ent.copy(); bad.doc_ent[5] = 400
    with pytest.raises(RuntimeError, match="entity ids"):
        ix.set_knowledge_graph(bad)
    # row offsets that run backwards or past the end are refused before any row is read
    for arr, at in (("doc_ent_indptr", 7), ("kg_indptr", 3)):
        bad = make_entity_graph(3000, 4, seed=5, n_ent=400)
        ip = getattr(bad, arr).copy(); ip[at] = ip[-1] + 5
        setattr(bad, arr, ip)
        with pytest.raises(RuntimeError, match="row offsets"):
            ix.set_knowledge_graph(bad)
    ix.set_knowledge_graph(kgs, le_cap=16)


def test_entity_search_skips_mark_deleted_documents(shard):
    w, docs, qs, ix, kgs, D, Q, sem, ent, wq, table = shard
    ix.set_knowledge_graph(kgs, le_cap=16)
    le, cnt, en_ip, en = [t.cpu().numpy() for t in ix.export_logical_edges()]
    k, L, w_k, hops = 10, 48, 0.5, 2
    base_ids, base_sc = [t.cpu().numpy() for t in ix.search_batch_entities(qs, k, L, kgs.q_ent, w_k, hops, wq)]
    base_counts = ix.search_stats(qs.n)[0].cpu().numpy()
    rng = np.random.default_rng(8)
    dele = np.unique(np.concatenate([rng.choice(docs.n, docs.n // 4, replace=False), base_ids[:, 0], base_ids[:, 5]])).astype(np.int32)
    dele = dele[dele >= 0]
    _say(f"entity search with {len(dele)} mark-deleted documents")
    try:
        ix.mark_deleted(dele)
        ids, sc = [t.cpu().numpy() for t in ix.search_batch_entities(qs, k, L, kgs.q_ent, w_k, hops, wq)]
        counts = ix.search_stats(qs.n)[0].cpu().numpy()
        assert np.array_equal(counts[:, :2], base_counts[:, :2])          # the traversal did not change
        assert not np.isin(ids[ids >= 0], dele).any()
        for qi in range(qs.n):
            oi, os_, _ = O.search_kg(D, sem, ent, Q, qi, wq[qi], k, L, kgs, le, cnt, en_ip, en, kgs.q_ent[qi], w_k,
                                     max_hops=hops, score_table=table[qi], deleted=dele)
            assert np.array_equal(ids[qi], oi) and np.array_equal(sc[qi], os_), qi
    finally:
        ix.mark_deleted(dele, restore=True)
    ids, sc = [t.cpu().numpy() for t in ix.search_batch_entities(qs, k, L, kgs.q_ent, w_k, hops, wq)]
    assert np.array_equal(ids, base_ids) and np.array_equal(sc, base_sc)
    # an entity id past the last entity is an unused slot, like a negative one
    qe = kgs.q_ent.copy(); qe[qe < 0] = 400 + 17
    ids2, sc2 = [t.cpu().numpy() for t in ix.search_batch_entities(qs, k, L, qe, w_k, hops, wq)]
    assert np.array_equal(ids2, base_ids) and np.array_equal(sc2, base_sc)


def test_entity_search_replay(shard):
    w, docs, qs, ix, kgs, D, Q, sem, ent, wq, table = shard
    ix.set_knowledge_graph(kgs, le_cap=16)
    le, cnt, en_ip, en = [t.cpu().numpy() for t in ix.export_logical_edges()]
    tied = 0
    for (k, L, w_k, hops, iters) in ((10, 64, 0.5, 2, 0), (5, 16, 2.0, 3, 0), (8, 8, 0.5, 1, 5), (10, 128, 0.0, 0, 0), (1, 1, 1.0, 2, 0)):
        _say(f"entity search replay: k={k} beam={L} w_k={w_k} max_hops={hops} iters={iters}")
        ids, sc = [t.cpu().numpy() for t in ix.search_batch_entities(qs, k, L, kgs.q_ent, w_k, hops, wq, iters)]
        counts = ix.search_stats(qs.n)[0].cpu().numpy()
        for qi in range(qs.n):
            oi, os_, log, ann = O.search_kg(D, sem, ent, Q, qi, wq[qi], k, L, kgs, le, cnt, en_ip, en, kgs.q_ent[qi], w_k,
                                            max_hops=hops, max_iters=iters, score_table=table[qi], log=True)
            assert np.array_equal(ids[qi], oi), (qi, k, L, ids[qi], oi)
            assert np.array_equal(sc[qi], os_), (qi, k, L)
            assert counts[qi, 0] == len(log), (qi, counts[qi], len(log))
            tied += int((ann[:, 1] > 0).sum())
    assert tied > 100
    # queries that name no entity are plain searches
    none = (kgs.q_ent < 0).all(axis=1)
    assert none.any()
    ids, sc = [t.cpu().numpy() for t in ix.search_batch_entities(qs, 10, 64, kgs.q_ent, 0.5, 2, wq)]
    pids, psc = [t.cpu().numpy() for t in ix.search_batch(qs, 10, 64, wq)]
    assert np.array_equal(ids[none], pids[none]) and np.array_equal(sc[none], psc[none])
    assert not np.array_equal(ids[~none], pids[~none])


def test_entity_search_cost(shard):
    """Measured, as in the paper's comparison with and without the knowledge graph: what the augmentation costs."""
    w, docs, qs, ix, kgs, D, Q, sem, ent, wq, table = shard
    ix.set_knowledge_graph(kgs, le_cap=16)
    big = B.DeviceVecs(make_workload("tiny", seed=28, n=10, nq=2000).queries)
    wb = np.tile(np.float32(w.weights), (big.n, 1))
    qe = make_entity_graph(3000, big.n, seed=5, n_ent=400).q_ent
    for name, fn in (("plain", lambda: ix.search_batch(big, 10, 64, wb)),
                     ("entities", lambda: ix.search_batch_entities(big, 10, 64, qe, 0.5, 2, wb))):
        fn(); torch.cuda.synchronize()
        t0 = time.time(); fn(); torch.cuda.synchronize()
        _say(f"  {name}: {big.n / (time.time() - t0):,.0f} queries/s, kernel {ix.search_kernel_ms():.2f} ms")


def test_searches_in_slabs_of_queries_give_the_same_bits(shard, debug_knobs):
    """A batch whose visited sets exceed the workspace cap runs in slabs of queries, one launch each: with the cap
    turned down to seven queries' worth, the plain, the keyword-constrained and the entity search return the bits
    and the per-query counters of the single launch."""
    from paper_2511_00855_amd.synth import make_keywords
    w, docs, qs, ix, kgs, D, Q, sem, ent, wq, table = shard
    ix.set_knowledge_graph(kgs, le_cap=16)
    kw = make_keywords(w.queries, seed=3, max_terms=2, stride=2, p_none=0.2)
    runs = (("plain", lambda: ix.search_batch(qs, 10, 96, wq, search_width=2)),
            ("keywords", lambda: ix.search_batch_keywords(qs, 10, 64, kw, wq)),
            ("entities", lambda: ix.search_batch_entities(qs, 10, 64, kgs.q_ent, 0.5, 2, wq)))
    whole = {}
    for name, fn in runs:
        ids, sc = [t.cpu().numpy() for t in fn()]
        whole[name] = (ids, sc, ix.search_stats(qs.n)[0].cpu().numpy())
    words = (docs.n + 31) // 32
    debug_knobs("search_workspace_bytes", 7 * words * 4)         # 40 queries -> 6 slabs of 7, 7, 7, 7, 7, 5
    for name, fn in runs:
        _say(f"search in slabs: {name}")
        ids, sc = [t.cpu().numpy() for t in fn()]
        counts = ix.search_stats(qs.n)[0].cpu().numpy()
        assert np.array_equal(ids, whole[name][0]) and np.array_equal(sc, whole[name][1]), name
        assert np.array_equal(counts, whole[name][2]), name
    # a corpus this small keeps its visited sets in LDS; kept in the global workspace instead, the same bits come out
    debug_knobs("search_workspace_bytes", 0)
    debug_knobs("search_visited_global", 1)
    for name, fn in runs:
        ids, sc = [t.cpu().numpy() for t in fn()]
        counts = ix.search_stats(qs.n)[0].cpu().numpy()
        assert np.array_equal(ids, whole[name][0]) and np.array_equal(sc, whole[name][1]) and np.array_equal(counts, whole[name][2]), name
    debug_knobs("search_workspace_bytes", 7 * words * 4)
    ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, 10, 96, wq, search_width=2)]
    assert np.array_equal(ids, whole["plain"][0]) and np.array_equal(sc, whole["plain"][1])
    debug_knobs("search_workspace_bytes", 1)                     # less than one query's set: one query per launch
    ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, 10, 96, wq, search_width=2)]
    assert np.array_equal(ids, whole["plain"][0]) and np.array_equal(sc, whole["plain"][1])
