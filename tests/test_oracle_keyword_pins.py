"""Pins of the oracle's keyword-constrained search (Section 4.2.2, keyword
branches of Algorithm 2) against things other than itself: the unconstrained
search, exhaustive filtering, a hand-traced six-document example, and a
restatement with Python sets in which the secondary pool is unbounded."""
import numpy as np
import pytest

import oracle as O
from paper_2511_00855_amd.synth import make_workload
from test_oracle_pins import vs_from_lists


@pytest.fixture(scope="module")
def small():
    w = make_workload("tiny", seed=5, n=300, nq=16)
    D = O.encode_docs(w.docs)
    Q = O.VS(w.queries)
    b = O.build_index(w.docs, O.default_params(8, nd_rounds=1, n_entry=4))
    cand = np.tile(np.arange(D.n, dtype=np.int32), (Q.n, 1))
    wq = np.array([0.5, 0.3, 0.2], np.float32)
    table = O.hybrid_block(Q, np.arange(Q.n), D, cand, wq)[:, :, 3]
    return w, D, Q, b, wq, table


def _terms(v, i):
    return set(int(t) for t in v.tx_idx[v.tx_indptr[i]:v.tx_indptr[i + 1]])


def _query_keywords(w, qi, n):
    """n of the query's own tokens (the most frequent in the corpus first, so that some documents match)."""
    t = sorted(_terms(w.queries, qi))
    df = np.bincount(w.docs.tx_idx, minlength=w.docs.tx_vocab)
    t.sort(key=lambda x: -df[x])
    return t[:n]


def _satisfies(w, v, kw, kw_all):
    hit = _terms(w.docs, v) & set(kw)
    return len(hit) == len(set(kw)) if kw_all else len(hit) > 0


def test_no_keywords_is_the_base_search(small):
    w, D, Q, b, wq, table = small
    for qi in range(Q.n):
        a = O.search(D, b.graph, b.entry, Q, qi, wq, 5, 12, 0, 2, log=True)
        c = O.search_kw(D, b.graph, b.ke, b.ke_count, b.entry, Q, qi, wq, 5, 12, [], width=2, log=True)
        for x, y in zip(a, c):
            assert np.array_equal(x, y)


@pytest.mark.parametrize("kw_all", [False, True])
def test_full_beam_is_filtered_bruteforce(small, kw_all):
    """Pool as large as the corpus on a graph that reaches everything: the
    result is the exact top-k of the documents that satisfy the constraint."""
    w, D, Q, b, wq, table = small
    N = D.n
    graph = np.stack([(np.arange(N) + s) % N for s in (1, 7, 31)], axis=1).astype(np.int32)
    ke = np.full((N, 2), -1, np.int32); kc = np.zeros(N, np.int32)
    entry = np.array([3], np.int32)
    nonempty = 0
    for qi in range(Q.n):
        kw = _query_keywords(w, qi, 2)
        ok = [v for v in range(N) if _satisfies(w, v, kw, kw_all)]
        ok.sort(key=lambda v: (-float(table[qi][v]), v))
        ids, sc, nv = O.search_kw(D, graph, ke, kc, entry, Q, qi, wq, 6, N, kw, kw_all=kw_all)
        assert nv == N
        want = ok[:6] + [-1] * (6 - len(ok[:6]))
        assert list(ids) == want, (qi, kw)
        for x, v in zip(sc, want):
            assert (x == -np.inf) if v < 0 else (abs(x - table[qi][v]) <= 1e-6 * max(1, abs(x)))
        nonempty += len(ok) > 0
    assert nonempty >= Q.n // 2


def _six_documents():
    """Dense-only scores 0.90 0.80 0.85 0.70 0.60 0.95 for documents 0..5; term 7 occurs in documents 2 and 5."""
    score = [0.90, 0.80, 0.85, 0.70, 0.60, 0.95]
    docs = vs_from_lists([[s, 0.0] for s in score], [{}] * 6, [{1: 1}, {2: 1}, {7: 1, 3: 1}, {4: 1}, {5: 1}, {7: 2}])
    q = vs_from_lists([[1.0, 0.0]], [{}], [{}])
    graph = np.array([[1, 2], [3, -1], [-1, -1], [4, -1], [-1, -1], [-1, -1]], np.int32)
    ke = np.array([[-1], [-1], [5], [-1], [-1], [-1]], np.int32)
    kc = np.array([0, 0, 1, 0, 0, 0], np.int32)
    return O.VS(docs), O.VS(q), graph, ke, kc


def test_hand_traced_twin_pool_and_keyword_edge():
    """Pool of two, entry 0, keyword {7}.  By hand: 0 enters; expanding 0 scores 1 (0.80) and 2 (0.85): the pool is
    {0, 2} and 1, which lacks the keyword, is dropped.  2 holds the keyword, so expanding it follows its keyword edge
    to 5 (0.95): the pool becomes {5, 0} and the evicted 2 moves to the secondary pool.  5 has no edges.  Result:
    5 then 2.  Without keyword edges 5 is never reached and 2 (still in the pool) is the only match; a keyword that
    no visited document holds gives nothing; with k = 1 only 5 remains."""
    D, Q, graph, ke, kc = _six_documents()
    w = (1.0, 0.0, 0.0)
    entry = np.array([0], np.int32)
    ids, sc, log = O.search_kw(D, graph, ke, kc, entry, Q, 0, w, 2, 2, [7], log=True)
    assert list(ids) == [5, 2] and list(log) == [0, 1, 2, 5]
    assert np.allclose(sc, [0.95, 0.85])
    ids, _, log = O.search_kw(D, graph, ke, kc, entry, Q, 0, w, 2, 2, [7], use_kw_edges=False, log=True)
    assert list(ids) == [2, -1] and list(log) == [0, 1, 2]
    ids, _, _ = O.search_kw(D, graph, ke, kc, entry, Q, 0, w, 2, 2, [9])
    assert list(ids) == [-1, -1]
    ids, _, _ = O.search_kw(D, graph, ke, kc, entry, Q, 0, w, 1, 2, [7])
    assert list(ids) == [5]
    # "all" needs both 7 and 3: only document 2
    ids, _, _ = O.search_kw(D, graph, ke, kc, entry, Q, 0, w, 2, 2, [7, 3], kw_all=True)
    assert list(ids) == [2, -1]
    ids, _, _ = O.search_kw(D, graph, ke, kc, entry, Q, 0, w, 2, 2, [7, 3], kw_all=False)
    assert list(ids) == [5, 2]


def test_rejected_on_arrival_reaches_the_secondary_pool():
    """Same six documents with document 2 scored 0.10: it never enters the pool of two, yet it is the answer."""
    D, Q, graph, ke, kc = _six_documents()
    docs = vs_from_lists([[s, 0.0] for s in [0.90, 0.80, 0.10, 0.70, 0.60, 0.95]], [{}] * 6,
                         [{1: 1}, {2: 1}, {7: 1, 3: 1}, {4: 1}, {5: 1}, {7: 2}])
    D = O.VS(docs)
    ids, sc, log = O.search_kw(D, graph, ke, kc, np.array([0], np.int32), Q, 0, (1.0, 0.0, 0.0), 2, 2, [7], log=True)
    # 0; then 1 and 2 (2 rejected -> secondary); 1 expands to 3 (0.70 < 0.80: dropped); 2 was never in the pool, so its keyword edge is not followed
    assert list(log) == [0, 1, 2, 3] and list(ids) == [2, -1] and np.isclose(sc[0], 0.10)


def _py_search_kw(scores, sat, graph, ke, kc, entry, k, L, width, iters, use_kw_edges=True):
    """Algorithm 2 with its keyword branches restated with Python lists; the secondary pool is the unbounded set of
    everything the pool did not keep."""
    visited = set(); pool = []; order = []; excluded = []
    def offer(v):
        if v < 0 or v in visited:
            return
        visited.add(v); order.append(v)
        pool.append([-float(scores[v]), int(v), False])
        pool.sort(key=lambda t: (t[0], t[1]))
        excluded.extend(t[1] for t in pool[L:])
        del pool[L:]
    for v in entry:
        offer(int(v))
    it = 0
    while iters == 0 or it < iters:
        par = [t for t in pool if not t[2]][:width]
        if not par:
            break
        for t in par:
            t[2] = True
        for t in par:
            for v in graph[t[1]]:
                offer(int(v))
            if use_kw_edges and sat[t[1]]:
                for v in ke[t[1]][:kc[t[1]]]:
                    offer(int(v))
        it += 1
    both = [t[1] for t in pool] + excluded
    res = sorted((v for v in both if sat[v]), key=lambda v: (-float(scores[v]), v))
    return res[:k], order


@pytest.mark.parametrize("kw_all", [False, True])
def test_python_set_restatement(small, kw_all):
    w, D, Q, b, wq, table = small
    N = D.n
    found = 0
    for qi in range(Q.n):
        for nk in (1, 2):
            kw = _query_keywords(w, qi, nk)
            sat = [_satisfies(w, v, kw, kw_all) for v in range(N)]
            for (k, L, width, iters, use) in ((5, 12, 1, 0, True), (5, 12, 2, 0, True), (3, 16, 1, 4, True), (5, 12, 1, 0, False), (8, 8, 1, 0, True)):
                ids, sc, log = O.search_kw(D, b.graph, b.ke, b.ke_count, b.entry, Q, qi, wq, k, L, kw, kw_all=kw_all,
                                           use_kw_edges=use, max_iters=iters, width=width, log=True)
                ids2, sc2, _ = O.search_kw(D, b.graph, b.ke, b.ke_count, b.entry, Q, qi, wq, k, L, kw, kw_all=kw_all,
                                           use_kw_edges=use, max_iters=iters, width=width, score_table=table[qi])
                assert np.array_equal(ids, ids2) and np.array_equal(sc, sc2)
                res, order = _py_search_kw(table[qi], sat, b.graph, b.ke, b.ke_count, b.entry, k, L, width, iters, use)
                assert [int(x) for x in ids if x >= 0] == res, (qi, kw, k, L, width, iters, use)
                assert list(log) == order
                assert all(sat[int(x)] for x in ids if x >= 0)
                found += len(res)
    assert found > 0


# ------------------------------------------------------------- mark-deletion (Section 4.1, updates of the index)
def test_mark_deletion_filters_only_the_answer(small):
    """Deleted documents are searched through and left out of the answer: the visit log does not change, and the
    answer is the undeleted part of the pool.  With a pool as large as the corpus on a graph that reaches
    everything, the answer is the exact top-k of the undeleted documents."""
    w, D, Q, b, wq, table = small
    N = D.n
    rng = np.random.default_rng(12)
    for qi in range(Q.n):
        base_ids, _, base_log = O.search(D, b.graph, b.entry, Q, qi, wq, 12, 12, log=True)
        dele = [int(base_ids[0]), int(base_ids[3]), int(rng.integers(0, N))]
        ids, sc, log = O.search(D, b.graph, b.entry, Q, qi, wq, 5, 12, log=True, deleted=dele)
        assert np.array_equal(log, base_log)
        want = [int(v) for v in base_ids if v >= 0 and v not in dele][:5]
        assert [int(v) for v in ids if v >= 0] == want
        assert np.allclose(sc[:len(want)], table[qi][want], rtol=1e-6)
        # nothing deleted = the plain search
        a = O.search(D, b.graph, b.entry, Q, qi, wq, 5, 12, deleted=[])
        c = O.search(D, b.graph, b.entry, Q, qi, wq, 5, 12)
        assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1])
    ring = np.stack([(np.arange(N) + s) % N for s in (1, 5)], axis=1).astype(np.int32)
    dele = rng.choice(N, N // 3, replace=False)
    for qi in range(4):
        ids, _, nv = O.search(D, ring, np.array([0], np.int32), Q, qi, wq, 7, N, deleted=dele)
        alive = [v for v in np.argsort(-table[qi].astype(np.float64), kind="stable") if v not in set(dele.tolist())]
        alive.sort(key=lambda v: (-float(table[qi][v]), v))
        assert nv == N and list(ids) == alive[:7]


def test_mark_deletion_with_keywords():
    """The six documents of the hand-traced case with document 2 deleted: 2 still satisfies the keyword, so its
    keyword edge to 5 is still followed, but 2 itself is neither kept in the secondary pool nor returned."""
    D, Q, graph, ke, kc = _six_documents()
    w = (1.0, 0.0, 0.0)
    entry = np.array([0], np.int32)
    ids, sc, log = O.search_kw(D, graph, ke, kc, entry, Q, 0, w, 2, 2, [7], log=True, deleted=[2])
    assert list(log) == [0, 1, 2, 5] and list(ids) == [5, -1]
    ids, _, _ = O.search_kw(D, graph, ke, kc, entry, Q, 0, w, 2, 2, [7], deleted=[5])
    assert list(ids) == [2, -1]
    ids, _, _ = O.search_kw(D, graph, ke, kc, entry, Q, 0, w, 2, 2, [7], deleted=[0, 1])
    assert list(ids) == [5, 2]


def test_mark_deletion_keyword_restatement(small):
    w, D, Q, b, wq, table = small
    N = D.n
    rng = np.random.default_rng(3)
    dele = set(rng.choice(N, N // 4, replace=False).tolist())
    for qi in range(Q.n):
        kw = _query_keywords(w, qi, 2)
        sat = [_satisfies(w, v, kw, False) for v in range(N)]
        for (k, L, width) in ((5, 12, 1), (4, 8, 2)):
            ids, sc, log = O.search_kw(D, b.graph, b.ke, b.ke_count, b.entry, Q, qi, wq, k, L, kw, width=width, log=True,
                                       deleted=sorted(dele))
            # the restatement with an unbounded secondary pool returns all satisfying documents it met, in order
            res, order = _py_search_kw(table[qi], sat, b.graph, b.ke, b.ke_count, b.entry, N, L, width, 0)
            assert list(log) == order
            assert [int(x) for x in ids if x >= 0] == [v for v in res if v not in dele][:k]
