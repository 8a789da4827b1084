"""GPU parity: S0 (BM25 encode), S1 (hybrid scores), exhaustive top-k and
S7-S9 (best-first search) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2511_00855_amd import binding as B
from paper_2511_00855_amd.synth import make_workload
from parity import RTOL_F32, RTOL_BF16, assert_ranked_equiv, assert_scores_close, row_norms, score_tol

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def tiny():
    w = make_workload("tiny")
    p = O.default_params(w.degree)
    ob = O.build_index(w.docs, p)                     # oracle-built graph
    docs = B.DeviceVecs(w.docs)
    qs = B.DeviceVecs(w.queries)
    bp = B.build_params(w.degree)
    ix = B.Index.import_graph(docs, bp, ob.graph, ob.entry, ob.ke, ob.ke_count)
    return w, ob, docs, qs, ix


def test_s0_bm25_and_self_sim(tiny):
    w, ob, docs, qs, ix = tiny
    _say("S0 tiny")
    tx_w, df, avgdl, self_sim = [t.cpu().numpy() for t in ix.export_ingest()]
    ow, odf, oavg = O.bm25_encode(w.docs.n, w.docs.tx_vocab, w.docs.tx_indptr, w.docs.tx_idx, w.docs.tx_val)
    assert np.array_equal(df, odf)
    assert abs(float(avgdl[0]) - oavg) <= 1e-6 * oavg
    np.testing.assert_allclose(tx_w, ow, rtol=2e-7, atol=0)
    np.testing.assert_allclose(self_sim, ob.self_sim, rtol=RTOL_F32)


@pytest.mark.parametrize("seed,n,nq,dim", [(1, 333, 7, 128), (2, 1000, 13, 768), (3, 517, 5, 260)])
def test_s1_hybrid_scores_query_doc(seed, n, nq, dim):
    _say(f"S1 query-doc seed={seed} n={n} nq={nq} dim={dim}")
    w = make_workload("tiny", seed=seed, n=n, nq=nq, dim=dim, sp=("poisson", 60), qsp=("poisson", 20), tx=("lognormal", 60))
    docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
    ix = B.Index.ingest(docs, B.build_params(8))
    rng = np.random.default_rng(seed)
    c = 97
    cand = rng.integers(0, n, (nq, c)).astype(np.int32)
    cand[rng.random((nq, c)) < 0.05] = -1
    wq = rng.uniform(-0.5, 1.5, (nq, 3)).astype(np.float32)
    got = ix.hybrid_scores(qs, cand, wq).cpu().numpy()
    D = O.encode_docs(w.docs); Q = O.VS(w.queries)
    ref = O.hybrid_block(Q, np.arange(nq), D, cand, wq)
    qn = row_norms(w.queries)[:, None]; dn = row_norms(w.docs)[np.maximum(cand, 0)]
    assert_scores_close(got, ref, score_tol(ref, wq[:, None, :], qn, dn, RTOL_F32), "query-doc")
    # default weights path
    ix.set_weights((0.25, 2.0, 0.5))
    got = ix.hybrid_scores(qs, cand).cpu().numpy()
    wd = np.tile(np.array([0.25, 2.0, 0.5], np.float32), (nq, 1))
    ref = O.hybrid_block(Q, np.arange(nq), D, cand, wd)
    assert_scores_close(got, ref, score_tol(ref, wd[:, None, :], qn, dn, RTOL_F32), "default weights")
    ix.close()


def test_s1_hybrid_scores_doc_doc_and_bf16():
    _say("S1 doc-doc f32 + bf16")
    for bf16 in (False, True):
        w = make_workload("tiny", seed=9, n=600, nq=4, dim=256, bf16=bf16, sp=("poisson", 100), tx=("lognormal", 60))
        docs = B.DeviceVecs(w.docs, bf16=bf16)
        ix = B.Index.ingest(docs, B.build_params(8))
        rng = np.random.default_rng(0)
        a = rng.integers(0, 600, 50).astype(np.int32)
        cand = rng.integers(0, 600, (50, 40)).astype(np.int32)
        cand[:, 0] = a                                   # self pair
        wv = (1.0, 0.7, 1.3)
        got = ix.hybrid_scores_docs(a, cand, wv).cpu().numpy()
        D = O.encode_docs(w.docs)
        ref = O.hybrid_block(D, a, D, cand, wv)
        dn = row_norms(w.docs)
        tol = score_tol(ref, np.array(wv)[None, None, :], dn[a][:, None], dn[cand], RTOL_BF16 if bf16 else RTOL_F32)
        assert_scores_close(got, ref, tol, f"doc-doc bf16={bf16}")
        if bf16:   # same stored values on both sides: the f32 bound holds too
            assert_scores_close(got, ref, score_tol(ref, np.array(wv)[None, None, :], dn[a][:, None], dn[cand], RTOL_F32), "bf16 tight")
        ix.close()


def test_bruteforce_topk(tiny):
    w, ob, docs, qs, ix = tiny
    _say("exhaustive top-k tiny")
    D = ob.D; Q = O.VS(w.queries)
    nq = qs.n
    rng = np.random.default_rng(5)
    wq = rng.uniform(0, 1, (nq, 3)).astype(np.float32)
    wq[:5] = [[1, 0, 0], [0, 1, 0], [0, 0, 1], [0.5, 0.5, 0], [0.34, 0.33, 0.33]]
    ids, sc = [t.cpu().numpy() for t in ix.bruteforce_topk(qs, 10, wq)]
    oid, osc = O.bruteforce_topk(Q, np.arange(nq), D, wq, 10)
    qn = row_norms(w.queries); dn = row_norms(w.docs)

    def tol_of(r, s):
        return RTOL_F32 * (abs(wq[r, 0]) * qn[r] * dn.max() + abs(s))

    def oscore(r, j):
        return float(O.hybrid_block(Q, [r], D, [[j]], wq[r])[0, 0, 3])
    nmis = assert_ranked_equiv(ids, sc, oid, osc, tol_of, oscore, "bruteforce")
    assert nmis <= nq // 10
    assert (np.abs(sc - osc) <= 2 * RTOL_F32 * (np.abs(osc) + 1)).all()


def test_search_matches_oracle_replay(tiny):
    """Same graph, same queries: the oracle's search, replayed on the GPU's own
    scores, must return exactly the GPU's ids; independently the scores agree
    with the oracle's within tolerance."""
    w, ob, docs, qs, ix = tiny
    D = ob.D; Q = O.VS(w.queries)
    nq, N = qs.n, docs.n
    allc = np.tile(np.arange(N, dtype=np.int32), (nq, 1))
    rng = np.random.default_rng(8)
    wq = np.tile(np.array(w.weights, np.float32), (nq, 1))
    wq[::7] = rng.uniform(0, 1, (len(wq[::7]), 3))
    table = ix.hybrid_scores(qs, allc, wq).cpu().numpy()[:, :, 3]
    ref4 = O.hybrid_block(Q, np.arange(nq), D, allc, wq)
    qn = row_norms(w.queries)[:, None]; dn = row_norms(w.docs)[None, :]
    assert_scores_close(table, ref4[:, :, 3], score_tol(ref4, wq[:, None, :], qn, dn, RTOL_F32)[:, :, 3], "table")
    for (k, L, iters, width) in ((10, 64, 0, 1), (10, 32, 0, 2), (5, 16, 4, 1), (10, 128, 0, 4), (10, 128, 0, 16), (1, 1, 0, 1)):
        _say(f"search tiny k={k} L={L} iters={iters} width={width}")
        ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, k, L, wq, iters, width)]
        for qi in range(nq):
            oi, os_, _ = O.search(D, ob.graph, ob.entry, Q, qi, wq[qi], k, L, iters, width, score_table=table[qi])
            assert np.array_equal(ids[qi], oi), (qi, k, L)
            assert np.array_equal(sc[qi], os_), (qi, k, L)
    # default weights + set_weights, no rebuild
    ix.set_weights((0.0, 1.0, 0.0))
    ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, 10, 64)]
    w010 = np.tile(np.array([0, 1, 0], np.float32), (nq, 1))
    t010 = ix.hybrid_scores(qs, allc, w010).cpu().numpy()[:, :, 3]
    for qi in range(0, nq, 5):
        oi, os_, _ = O.search(D, ob.graph, ob.entry, Q, qi, w010[qi], 10, 64, score_table=t010[qi])
        assert np.array_equal(ids[qi], oi)


def test_search_edge_cases(tiny):
    w, ob, docs, qs, ix = tiny
    _say("search edge cases")
    # zero queries
    empty = make_workload("tiny", seed=1, n=10, nq=1).queries
    e = B.DeviceVecs(empty); e.n = 0
    ids, sc = ix.search_batch(e, 10, 64)
    assert ids.shape == (0, 10)
    # bad arguments come back as errors, not crashes
    with pytest.raises(B.ApError):
        ix.search_batch(qs, 10, 5)          # k > beam
    with pytest.raises(B.ApError):
        ix.search_batch(qs, 10, 16385)
    with pytest.raises(B.ApError):
        ix.search_batch(qs, 10, 64, search_width=17)
    ing = B.Index.ingest(docs, B.build_params(w.degree))
    with pytest.raises(B.ApError):
        ing.search_batch(qs, 10, 64)        # no graph
    ing.close()


def test_search_sparse_graph_missing_results():
    """A graph with holes and few reachable nodes: unreachable results are -1 / -inf."""
    _say("search tiny graph with holes")
    w = make_workload("tiny", seed=4, n=64, nq=9)
    N, R = 64, 4
    graph = np.full((N, R), -1, np.int32)
    graph[0, :2] = [1, 2]; graph[1, 0] = 3; graph[2, 1] = 0
    entry = np.array([0] + [-1] * 3, np.int32)
    docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
    ix = B.Index.import_graph(docs, B.build_params(R, knn_k=8, n_entry=4), graph, entry)
    ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, 6, 8)]
    D = O.encode_docs(w.docs); Q = O.VS(w.queries)
    table = ix.hybrid_scores(qs, np.tile(np.arange(N, dtype=np.int32), (9, 1))).cpu().numpy()[:, :, 3]
    for qi in range(9):
        oi, os_, _ = O.search(D, graph, entry, Q, qi, (1, 1, 1), 6, 8, score_table=table[qi])
        assert np.array_equal(ids[qi], oi) and np.array_equal(sc[qi], os_)
        assert set(ids[qi][:4]) == {0, 1, 2, 3} and (ids[qi][4:] == -1).all() and np.isneginf(sc[qi][4:]).all()
    ix.close()
    # an imported graph is checked once: ids beyond the corpus, ids below -1, keyword counts beyond the row
    bp = B.build_params(R, knn_k=8, n_entry=4)
    for bad in ("edge", "negative", "entry", "kw_count", "kw_edge"):
        g2, e2 = graph.copy(), entry.copy()
        kw = np.full((N, R // 2), -1, np.int32); kc = np.zeros(N, np.int32)
        if bad == "edge": g2[5, 1] = N
        if bad == "negative": g2[7, 0] = -2
        if bad == "entry": e2[1] = N + 3
        if bad == "kw_count": kc[9] = R // 2 + 1
        if bad == "kw_edge": kw[3, 0] = N; kc[3] = 1
        with pytest.raises(RuntimeError, match="out of range"):
            B.Index.import_graph(docs, bp, g2, e2, kw, kc)
    with pytest.raises(RuntimeError, match="come together"):
        B.Index.import_graph(docs, bp, graph, entry, np.full((N, R // 2), -1, np.int32), None)
