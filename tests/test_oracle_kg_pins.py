"""Pins of the oracle's knowledge-graph augmentation (Section 3.4, logical edges; Section 4.2.3 and the entity
branches of Algorithm 2) against things other than itself: set-comprehension brute force for the logical edges,
the base search where the augmentation is inert, a hand-traced six-document case, and a restatement with Python
dictionaries."""
from types import SimpleNamespace

import numpy as np
import pytest

import oracle as O
from paper_2511_00855_amd.synth import make_entity_graph, make_workload
from test_oracle_pins import vs_from_lists


@pytest.fixture(scope="module")
def small():
    w = make_workload("tiny", seed=9, n=300, nq=16)
    D = O.encode_docs(w.docs)
    Q = O.VS(w.queries)
    b = O.build_index(w.docs, O.default_params(8, nd_rounds=1, n_entry=4))
    kgs = make_entity_graph(300, 16, seed=2, n_ent=60)
    le, lc, en_ip, en = O.logical_edges(kgs, 300, 12)
    cand = np.tile(np.arange(D.n, dtype=np.int32), (Q.n, 1))
    wq = np.array([0.5, 0.3, 0.2], np.float32)
    table = O.hybrid_block(Q, np.arange(Q.n), D, cand, wq)[:, :, 3]
    return w, D, Q, b, kgs, le, lc, en_ip, en, wq, table


def _V(kgs, x):
    return [int(e) for e in kgs.doc_ent[kgs.doc_ent_indptr[x]:kgs.doc_ent_indptr[x + 1]]]


def _KG(kgs, e):
    return [int(t) for t in kgs.kg_idx[kgs.kg_indptr[e]:kgs.kg_indptr[e + 1]]]


def test_logical_edges_by_set_comprehension(small):
    """Section 3.4: two documents are joined wherever an entity of one is related to an entity of the other that
    the first does not mention itself."""
    w, D, Q, b, kgs, le, lc, en_ip, en, wq, table = small
    n = D.n
    rel = {(s, t) for s in range(kgs.n_ent) for t in _KG(kgs, s)}
    assert all((t, s) in rel for (s, t) in rel) and all(s != t for (s, t) in rel)
    V = [set(_V(kgs, x)) for x in range(n)]
    many = 0
    for x in range(n):
        want = sorted((s, t, y) for y in range(n) if y != x for t in V[y] - V[x] for s in V[x] if (s, t) in rel)
        got = [(int(a), int(c), int(bb)) for a, bb, c in le[x][:lc[x]]]
        assert got == want[:12], x
        assert lc[x] == min(len(want), 12) and (le[x][lc[x]:] == -1).all()
        many += len(want) > 12
    assert 0 < many < n
    for e in range(kgs.n_ent):
        assert [int(y) for y in en[en_ip[e]:en_ip[e + 1]]] == [x for x in range(n) if e in V[x]]


def test_inert_augmentation_is_the_base_search(small):
    w, D, Q, b, kgs, le, lc, en_ip, en, wq, table = small
    for qi in range(Q.n):
        base = O.search(D, b.graph, b.entry, Q, qi, wq, 5, 12, log=True)
        # no query entities: usual entry points, nobody carries an entity
        got = O.search_kg(D, b.graph, b.entry, Q, qi, wq, 5, 12, kgs, le, lc, en_ip, en, [-1, -1], 0.7, log=True)
        assert np.array_equal(base[0], got[0]) and np.array_equal(base[1], got[1]) and np.array_equal(base[2], got[2])
        assert (got[3][:, 0] == -1).all()
        # query entities, but no reward and no logical hop: the base search started from the documents that mention them
        qe = kgs.q_ent[qi]
        start = []
        for e in qe[qe >= 0]:
            start += [int(y) for y in en[en_ip[e]:en_ip[e + 1]] if int(y) not in start]
        start = start[:len(b.entry)]
        base = O.search(D, b.graph, np.array(start, np.int32), Q, qi, wq, 5, 12, log=True)
        got = O.search_kg(D, b.graph, b.entry, Q, qi, wq, 5, 12, kgs, le, lc, en_ip, en, qe, 0.0, max_hops=0, log=True)
        assert np.array_equal(base[0], got[0]) and np.array_equal(base[1], got[1]) and np.array_equal(base[2], got[2])


def _six():
    """Documents 0..5 with dense-only scores .9 .8 .7 .6 .5 .4; entities V = {0},{},{1},{2},{1},{}; relations 0-1, 1-2;
    semantic edges 0 -> 1, 1 -> 5."""
    docs = vs_from_lists([[s, 0.0] for s in (0.9, 0.8, 0.7, 0.6, 0.5, 0.4)], [{}] * 6, [{}] * 6)
    q = vs_from_lists([[1.0, 0.0]], [{}], [{}])
    graph = np.array([[1, -1], [5, -1], [-1, -1], [-1, -1], [-1, -1], [-1, -1]], np.int32)
    kgs = SimpleNamespace(n_ent=3, doc_ent_indptr=np.array([0, 1, 1, 2, 3, 4, 4], np.int64), doc_ent=np.array([0, 1, 2, 1], np.int32),
                          kg_indptr=np.array([0, 1, 3, 4], np.int64), kg_idx=np.array([1, 0, 2, 1], np.int32))
    return O.VS(docs), O.VS(q), graph, kgs


def test_hand_traced_entity_search():
    """Query entity 0, pool of four, reward 0.3.  By hand: the search starts at document 0 (the only one that
    mentions entity 0; hop 0).  Expanding 0: its semantic neighbour 1 has no entity (0.8); its logical edges lead to
    2 and 4, which mention entity 1, related to 0: hop 1, scores 0.7 + 0.3 and 0.5 + 0.3.  Pool: 2, 0, 1, 4 (1 before 4
    by id).  Expanding 2 (entity 1, hop 1): its logical edge to 0 is visited, the one to 3 gives entity 2, hop 2,
    0.6 + 0.15 = 0.75 < 0.8: rejected.  Expanding 1: document 5 scores 0.4: rejected.  Expanding 4: nothing new."""
    D, Q, graph, kgs = _six()
    le, lc, en_ip, en = O.logical_edges(kgs, 6, 4)
    assert [tuple(t) for t in le[0][:lc[0]]] == [(0, 2, 1), (0, 4, 1)]
    assert [tuple(t) for t in le[2][:lc[2]]] == [(1, 0, 0), (1, 3, 2)] and [tuple(t) for t in le[3][:lc[3]]] == [(2, 2, 1), (2, 4, 1)]
    assert lc[1] == 0 and lc[5] == 0
    entry = np.array([5, 3], np.int32)
    w = (1.0, 0.0, 0.0)
    ids, sc, log, ann = O.search_kg(D, graph, entry, Q, 0, w, 4, 4, kgs, le, lc, en_ip, en, [0], 0.3, max_hops=2, log=True)
    assert list(ids) == [2, 0, 1, 4] and np.allclose(sc, [1.0, 0.9, 0.8, 0.8])
    assert list(log) == [0, 1, 2, 4, 3, 5]
    assert [tuple(a) for a in ann] == [(0, 0), (-1, 0), (1, 1), (1, 1), (2, 2), (-1, 0)]
    # one hop only: document 2's logical edges are not followed
    ids, sc, log, _ = O.search_kg(D, graph, entry, Q, 0, w, 4, 4, kgs, le, lc, en_ip, en, [0], 0.3, max_hops=1, log=True)
    assert list(log) == [0, 1, 2, 4, 5] and list(ids) == [2, 0, 1, 4]
    # no reward: plain scores, and document 3 (0.6) replaces document 4 (0.5)
    ids, sc, log, _ = O.search_kg(D, graph, entry, Q, 0, w, 4, 4, kgs, le, lc, en_ip, en, [0], 0.0, max_hops=2, log=True)
    assert list(ids) == [0, 1, 2, 3] and list(log) == [0, 1, 2, 4, 5, 3]
    # an entity nobody mentions: the usual entry points
    kgs.n_ent = 4
    kgs.kg_indptr = np.append(kgs.kg_indptr, kgs.kg_indptr[-1])
    le, lc, en_ip, en = O.logical_edges(kgs, 6, 4)
    ids, _, log, ann = O.search_kg(D, graph, entry, Q, 0, w, 4, 4, kgs, le, lc, en_ip, en, [3], 0.3, log=True)
    assert list(log) == [5, 3] and (ann[:, 0] == -1).all()


def _py_search_kg(scores, graph, entry, kgs, le, lc, en_ip, en, q_ent, k, L, w_k, max_hops, iters):
    V = lambda x: _V(kgs, x)
    visited = set(); pool = []; order = []; ann = []
    def offer(o, eu, hu, ent0=None):
        visited.add(o); order.append(o)
        ent, hop, s = -1, 0, np.float32(scores[o])
        if ent0 is not None:
            ent = ent0
        elif eu >= 0:
            hits = [t for t in V(o) if t in _KG(kgs, eu)]
            if hits:
                ent, hop = min(hits), hu + 1
                s = np.float32(s + np.float32(w_k) / np.float32(hop))
        ann.append((ent, hop))
        pool.append([-float(s), int(o), False, ent, hop])
        pool.sort(key=lambda t: (t[0], t[1]))
        del pool[L:]
    start = []
    for e in q_ent:
        if e >= 0:
            for y in en[en_ip[e]:en_ip[e + 1]]:
                if int(y) not in [s[0] for s in start] and len(start) < len(entry):
                    start.append((int(y), int(e)))
    if start:
        for y, e in start:
            offer(y, -1, 0, ent0=e)
    else:
        for v in entry:
            if v >= 0 and int(v) not in visited:
                offer(int(v), -1, 0)
    it = 0
    while iters == 0 or it < iters:
        par = [t for t in pool if not t[2]][:1]
        if not par:
            break
        u = par[0]; u[2] = True
        for v in graph[u[1]]:
            if v >= 0 and int(v) not in visited:
                offer(int(v), u[3], u[4])
        if u[3] >= 0 and u[4] < max_hops:
            for s, y, t in le[u[1]][:lc[u[1]]]:
                if s == u[3] and int(y) not in visited:
                    offer(int(y), u[3], u[4])
        it += 1
    return [t[1] for t in pool][:k], [-t[0] for t in pool][:k], order, ann


def test_python_restatement(small):
    w, D, Q, b, kgs, le, lc, en_ip, en, wq, table = small
    rewarded = via_logical = 0
    for qi in range(Q.n):
        for (k, L, w_k, hops, iters) in ((5, 12, 0.5, 2, 0), (8, 8, 2.0, 3, 0), (5, 16, 0.5, 1, 6)):
            ids, sc, log, ann = O.search_kg(D, b.graph, b.entry, Q, qi, wq, k, L, kgs, le, lc, en_ip, en, kgs.q_ent[qi], w_k,
                                            max_hops=hops, max_iters=iters, score_table=table[qi], log=True)
            pi, ps, order, pann = _py_search_kg(table[qi], b.graph, b.entry, kgs, le, lc, en_ip, en, kgs.q_ent[qi], k, L, w_k, hops, iters)
            assert [int(x) for x in ids if x >= 0] == pi, (qi, k, L)
            assert np.allclose(sc[:len(ps)], ps, rtol=1e-6)
            assert list(log) == order and [tuple(a) for a in ann] == pann
            rewarded += sum(1 for a in pann if a[1] > 0)
            via_logical += len(order)
    assert rewarded > 50


def test_mark_deleted_documents_are_searched_through_and_left_out(small):
    """Section 4.1 (updates): with deletions the traversal is the one without them (same documents scored, in the same
    order), and the answer is the undeleted pool's order with the deleted documents struck out."""
    w, D, Q, b, kgs, le, lc, en_ip, en, wq, table = small
    struck = 0
    for qi in range(Q.n):
        k, L = 5, 16
        full, fsc, flog, _ = O.search_kg(D, b.graph, b.entry, Q, qi, wq, L, L, kgs, le, lc, en_ip, en, kgs.q_ent[qi], 0.5,
                                         score_table=table[qi], log=True)
        dele = [int(full[0]), int(full[3])] + list(range(0, D.n, 9))
        ids, sc, log, _ = O.search_kg(D, b.graph, b.entry, Q, qi, wq, k, L, kgs, le, lc, en_ip, en, kgs.q_ent[qi], 0.5,
                                      score_table=table[qi], log=True, deleted=dele)
        assert list(log) == list(flog)
        keep = [(int(i), s) for i, s in zip(full, fsc) if i >= 0 and int(i) not in set(dele)][:k]
        want = [i for i, _ in keep] + [-1] * (k - len(keep))
        assert [int(x) for x in ids] == want, qi
        assert np.array_equal(sc[:len(keep)], np.float32([s for _, s in keep]))
        assert np.isneginf(sc[len(keep):]).all()
        struck += sum(1 for i in full[:k] if int(i) in set(dele))
    assert struck >= 2 * Q.n
