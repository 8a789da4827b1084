"""GPU parity of the keyword-constrained search (Section 4.2.2, Algorithm 2's
keyword branches): ap_search_batch_keywords against the oracle's search_kw,
replayed on the GPU's own scores (ids, scores and the number of scored
documents must agree bit for bit) and run on the oracle's own scores."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2511_00855_amd import binding as B
from paper_2511_00855_amd.synth import make_keywords, make_workload
from parity import RTOL_F32, row_norms

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _kw_list(row):
    return [int(t) for t in row if t >= 0]


def _has(w, v, kw, kw_all):
    t = set(int(x) for x in w.docs.tx_idx[w.docs.tx_indptr[v]:w.docs.tx_indptr[v + 1]])
    return set(kw) <= t if kw_all else bool(set(kw) & t)


@pytest.fixture(scope="module")
def tiny():
    w = make_workload("tiny", seed=21, n=2000, nq=48)
    docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
    ix = B.Index.build(docs, B.build_params(w.degree))
    D = O.encode_docs(w.docs); Q = O.VS(w.queries)
    sem, ke, kc, ent = [t.cpu().numpy() for t in ix.export_graph()]
    wq = np.random.default_rng(2).uniform(0.1, 1.0, (qs.n, 3)).astype(np.float32)
    allc = np.tile(np.arange(docs.n, dtype=np.int32), (qs.n, 1))
    table = ix.hybrid_scores(qs, allc, wq).cpu().numpy()[:, :, 3]
    yield w, docs, qs, ix, D, Q, sem, ke, kc, ent, wq, table
    ix.close()


@pytest.mark.parametrize("kw_all,use_edges", [(False, True), (True, True), (False, False)])
def test_keyword_search_replay(tiny, kw_all, use_edges):
    w, docs, qs, ix, D, Q, sem, ke, kc, ent, wq, table = tiny
    assert kc.max() > 0, "the build produced no keyword edges"
    kw = make_keywords(w.queries, seed=4, max_terms=3, stride=5, p_none=0.15)
    assert (kw[:, 0] < 0).any() and (kw[:, 1] >= 0).any()
    nsat = 0
    for (k, L, iters, width) in ((10, 64, 0, 1), (5, 16, 0, 2), (8, 8, 0, 1), (10, 128, 6, 8), (1, 4, 0, 1), (32, 32, 0, 3)):
        _say(f"keyword search replay: all={kw_all} edges={use_edges} k={k} beam={L} iters={iters} width={width}")
        ids, sc = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, k, L, kw, wq, kw_all, use_edges, iters, width)]
        counts = ix.search_stats(qs.n)[0].cpu().numpy()
        for qi in range(qs.n):
            oi, os_, nv = O.search_kw(D, sem, ke, kc, ent, Q, qi, wq[qi], k, L, _kw_list(kw[qi]), kw_all, use_edges, iters, width,
                                      score_table=table[qi])
            assert np.array_equal(ids[qi], oi), (qi, k, L, iters, width, ids[qi], oi)
            assert np.array_equal(sc[qi], os_), (qi, k, L)
            assert counts[qi, 0] == nv, (qi, counts[qi], nv)
            if (kw[qi] >= 0).any():
                assert all(_has(w, int(v), _kw_list(kw[qi]), kw_all) for v in ids[qi] if v >= 0)
                nsat += int((ids[qi] >= 0).sum())
    assert nsat > 0


def test_keyword_edges_matter_and_unconstrained_rows(tiny):
    """Rows without keywords equal the plain search; keyword edges change what is visited."""
    w, docs, qs, ix, D, Q, sem, ke, kc, ent, wq, table = tiny
    kw = make_keywords(w.queries, seed=9, max_terms=2, stride=2, p_none=0.3)
    plain_ids, plain_sc = [t.cpu().numpy() for t in ix.search_batch(qs, 10, 32, wq)]
    plain_counts = ix.search_stats(qs.n)[0].cpu().numpy()
    ids, sc = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, 10, 32, kw, wq)]
    counts = ix.search_stats(qs.n)[0].cpu().numpy()
    none = (kw < 0).all(axis=1)
    assert none.any() and (~none).any()
    assert np.array_equal(ids[none], plain_ids[none]) and np.array_equal(sc[none], plain_sc[none])
    assert np.array_equal(counts[none][:, :2], plain_counts[none][:, :2])
    ids0, _ = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, 10, 32, kw, wq, use_kw_edges=False)]
    counts0 = ix.search_stats(qs.n)[0].cpu().numpy()
    assert (counts[~none, 0] >= counts0[~none, 0]).all() and (counts[~none, 0] > counts0[~none, 0]).any()
    # all slots unused in every row: the whole batch is the plain search
    ids1, sc1 = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, 10, 32, np.full((qs.n, 1), -1, np.int32), wq)]
    assert np.array_equal(ids1, plain_ids) and np.array_equal(sc1, plain_sc)


def test_keyword_search_on_oracle_scores(tiny):
    """Not a replay: the oracle scores in fp64 on its own.  Results agree up to swaps of scores within tolerance."""
    w, docs, qs, ix, D, Q, sem, ke, kc, ent, wq, table = tiny
    kw = make_keywords(w.queries, seed=4, max_terms=2, stride=2)
    k, L = 10, 64
    ids, sc = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, k, L, kw, wq)]
    qn = row_norms(w.queries); dmax = row_norms(w.docs).max()
    same = 0
    for qi in range(qs.n):
        oi, os_, _ = O.search_kw(D, sem, ke, kc, ent, Q, qi, wq[qi], k, L, _kw_list(kw[qi]))
        same += np.array_equal(ids[qi], oi)
        m = (ids[qi] >= 0) & (oi >= 0)
        tol = RTOL_F32 * (np.abs(os_[m]) + wq[qi].max() * qn[qi] * dmax + 1.0)
        assert (np.abs(sc[qi][m] - os_[m]) <= tol).all(), qi
    assert same >= qs.n - 2, same


def test_keywords_deep_in_long_texts():
    """Texts longer than the 64 entries a wave holds in registers: the required term sits in the tail."""
    w = make_workload("tiny", seed=33, n=500, nq=10, dim=32, tx=("lognormal", 150), sp=("poisson", 20))
    docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
    ix = B.Index.build(docs, B.build_params(8, knn_k=24, nd_rounds=2, nd_sample=6, n_entry=8, sp_len=3))
    D = O.encode_docs(w.docs); Q = O.VS(w.queries)
    sem, ke, kc, ent = [t.cpu().numpy() for t in ix.export_graph()]
    wq = np.tile(np.float32([0.4, 0.3, 0.3]), (qs.n, 1))
    table = ix.hybrid_scores(qs, np.tile(np.arange(docs.n, dtype=np.int32), (qs.n, 1)), wq).cpu().numpy()[:, :, 3]
    lens = w.docs.tx_indptr[1:] - w.docs.tx_indptr[:-1]
    long_docs = np.nonzero(lens > 70)[0]
    assert len(long_docs) >= qs.n
    kw = np.full((qs.n, 2), -1, np.int32)
    for qi in range(qs.n):
        v = long_docs[qi]
        kw[qi, 0] = w.docs.tx_idx[w.docs.tx_indptr[v] + 66 + qi % 4]      # a term beyond position 64 of document v
        kw[qi, 1] = w.docs.tx_idx[w.docs.tx_indptr[long_docs[-1 - qi]] + 1]
    for kw_all in (False, True):
        ids, sc = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, 6, 500, kw, wq, kw_all)]
        hits = 0
        for qi in range(qs.n):
            oi, os_, _ = O.search_kw(D, sem, ke, kc, ent, Q, qi, wq[qi], 6, 500, _kw_list(kw[qi]), kw_all, score_table=table[qi])
            assert np.array_equal(ids[qi], oi) and np.array_equal(sc[qi], os_), (qi, kw_all)
            hits += int(long_docs[qi] in ids[qi])
        _say(f"deep keywords all={kw_all}: planted documents returned for {hits} of {qs.n} queries")
    ix.close()


def test_keyword_argument_checks(tiny):
    w, docs, qs, ix, *_ = tiny
    with pytest.raises(RuntimeError):
        ix.search_batch_keywords(qs, 10, 32, np.full((qs.n, 17), -1, np.int32))
    with pytest.raises(RuntimeError):
        ix.search_batch_keywords(qs, 64, 32, np.full((qs.n, 2), -1, np.int32))


def test_mark_deletion(tiny):
    """Mark-deleted documents are searched through and left out of the answers of both searches; restoring them
    brings the old answers back."""
    w, docs, qs, ix, D, Q, sem, ke, kc, ent, wq, table = tiny
    _say("mark-deletion")
    N = docs.n
    k, L = 10, 32
    base_ids, base_sc = [t.cpu().numpy() for t in ix.search_batch(qs, k, L, wq)]
    base_counts = ix.search_stats(qs.n)[0].cpu().numpy()
    rng = np.random.default_rng(6)
    dele = np.unique(np.concatenate([rng.choice(N, N // 5, replace=False), base_ids[:, 0], base_ids[:, 4]])).astype(np.int32)
    kw = make_keywords(w.queries, seed=4, max_terms=2, stride=2, p_none=0.1)
    try:
        ix.mark_deleted(dele)
        ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, k, L, wq)]
        counts = ix.search_stats(qs.n)[0].cpu().numpy()
        assert np.array_equal(counts[:, :2], base_counts[:, :2])          # the search itself did not change
        assert not np.isin(ids[ids >= 0], dele).any()
        kids, ksc = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, k, L, kw, wq)]
        kids2, ksc2 = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, 8, 8, kw, wq, True, True, 0, 2)]
        for qi in range(qs.n):
            oi, os_, _ = O.search(D, sem, ent, Q, qi, wq[qi], k, L, score_table=table[qi], deleted=dele)
            assert np.array_equal(ids[qi], oi) and np.array_equal(sc[qi], os_), qi
            oi, os_, _ = O.search_kw(D, sem, ke, kc, ent, Q, qi, wq[qi], k, L, _kw_list(kw[qi]), score_table=table[qi], deleted=dele)
            assert np.array_equal(kids[qi], oi) and np.array_equal(ksc[qi], os_), qi
            oi, os_, _ = O.search_kw(D, sem, ke, kc, ent, Q, qi, wq[qi], 8, 8, _kw_list(kw[qi]), True, True, 0, 2,
                                     score_table=table[qi], deleted=dele)
            assert np.array_equal(kids2[qi][:8], oi) and np.array_equal(ksc2[qi][:8], os_), qi
        with pytest.raises(RuntimeError):
            ix.mark_deleted(np.array([3, N, 5], np.int32))
    finally:
        ix.mark_deleted(np.concatenate([dele, [3, 5]]).astype(np.int32), restore=True)
    ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, k, L, wq)]
    assert np.array_equal(ids, base_ids) and np.array_equal(sc, base_sc)


def test_bench_keyword_ground_truth_is_the_constrained_top_k(tiny):
    """bench.py's keyword leg measures recall against a ground truth it computes with torch (mask of the documents
    that hold a required term over the GPU's exhaustive scores, then top-k).  Here the same function against a
    brute force over the oracle's fp64 scores: the satisfying documents enumerated from the CSR rows one by one,
    sorted by (score, id).  Differences are admitted only between near-ties."""
    import bench
    from parity import assert_ranked_equiv, score_tol
    w, docs, qs, ix, D, Q, sem, ke, kc, ent, wq, table = tiny
    k = 10
    kw = make_keywords(w.queries, seed=9, max_terms=2, stride=2)
    sample = np.arange(0, qs.n, 2)
    gt, gs = bench.keyword_ground_truth(w, ix, torch.from_numpy(wq).cuda(), kw, sample, k)
    allc = np.tile(np.arange(docs.n, dtype=np.int32), (len(sample), 1))
    ref = O.hybrid_block(Q, sample, D, allc, wq[sample])
    tol = score_tol(ref, wq[sample][:, None, :], row_norms(w.queries)[sample][:, None], row_norms(w.docs)[None, :], RTOL_F32)[:, :, 3]
    fused = ref[:, :, 3]
    oid = np.full((len(sample), k), -1, np.int64); osc = np.full((len(sample), k), -np.inf)
    nfew = 0
    for x, qi in enumerate(sample):
        sat = [v for v in range(docs.n) if _has(w, v, _kw_list(kw[qi]), False)]
        order = sorted(sat, key=lambda v: (-fused[x, v], v))[:k]
        oid[x, :len(order)] = order; osc[x, :len(order)] = fused[x, order]
        nfew += len(order) < k
    assert (gt >= 0).sum() == (oid >= 0).sum()
    assert_ranked_equiv(gt, gs, oid, osc, lambda r, s_: float(tol[r].max()), lambda r, j: float(fused[r, j]), "keyword ground truth")
    _say(f"keyword ground truth: {len(sample)} queries, {nfew} with fewer than {k} satisfying documents")
