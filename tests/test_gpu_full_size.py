"""Parity at the full size of the benchmark workload (config 2: 100,000
documents, d = 768, 10,000 queries) in the launch configuration bench.py
times, on sampled outputs the oracle can compute one by one; plus the
dynamic-fusion sweep of config 4 (five weight settings on the same index, no
rebuild), and 150,000 documents of config 3's shape (bf16 rows) through the
seed sweep a million-document build uses."""
import time
import types

import numpy as np
import pytest
import torch

import oracle as O
from paper_2511_00855_amd import binding as B
from paper_2511_00855_amd.synth import make_keywords, make_workload
from parity import RTOL_F32, assert_ranked_equiv, assert_scores_close, row_norms, score_tol

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def full():
    t0 = time.time()
    w = make_workload("cfg2", seed=0)
    _say(f"cfg2 generated in {time.time() - t0:.1f}s")
    docs = B.DeviceVecs(w.docs)
    qs = B.DeviceVecs(w.queries)
    bp = B.build_params(w.degree)                      # what bench.py uses
    t0 = time.time()
    ix = B.Index.build(docs, bp)
    torch.cuda.synchronize()
    _say(f"built in {time.time() - t0:.2f}s {ix.build_timings()}")
    D = O.encode_docs(w.docs)
    Q = O.VS(w.queries)
    yield w, docs, qs, bp, ix, D, Q
    ix.close()


def _score_table(w, ix, sample, wq):
    """Fused scores of every document for the sampled queries, from ap_hybrid_scores (what an oracle replay runs on)."""
    N = w.docs.n
    sq = types.SimpleNamespace(n=len(sample), dim=w.queries.dim, dense=w.queries.dense[sample],
                               sp_indptr=None, sp_idx=None, sp_val=None, tx_indptr=None, tx_idx=None, tx_val=None,
                               sp_vocab=w.queries.sp_vocab, tx_vocab=w.queries.tx_vocab)
    for pre in ("sp", "tx"):
        ip = getattr(w.queries, pre + "_indptr")
        lens = (ip[1:] - ip[:-1])[sample]
        setattr(sq, pre + "_indptr", np.concatenate([[0], np.cumsum(lens)]).astype(np.int64))
        setattr(sq, pre + "_idx", np.concatenate([getattr(w.queries, pre + "_idx")[ip[i]:ip[i + 1]] for i in sample]))
        setattr(sq, pre + "_val", np.concatenate([getattr(w.queries, pre + "_val")[ip[i]:ip[i + 1]] for i in sample]))
    dsq = B.DeviceVecs(sq)
    allc = np.tile(np.arange(N, dtype=np.int32), (len(sample), 1))
    return ix.hybrid_scores(dsq, allc, wq[sample]).cpu().numpy()[:, :, 3]


def test_full_size_scores_sampled(full):
    w, docs, qs, bp, ix, D, Q = full
    _say("full size: sampled hybrid scores")
    rng = np.random.default_rng(0)
    nq, N = qs.n, docs.n
    c = 64
    cand = rng.integers(0, N, (nq, c)).astype(np.int32)
    wq = rng.uniform(0, 1, (nq, 3)).astype(np.float32)
    got = ix.hybrid_scores(qs, cand, wq).cpu().numpy()
    rows = rng.choice(nq, 400, replace=False)
    ref = O.hybrid_block(Q, rows, D, cand[rows], wq[rows])
    qn = row_norms(w.queries)[rows][:, None]
    dn = np.linalg.norm(w.docs.dense[cand[rows].ravel()].astype(np.float64), axis=1).reshape(len(rows), c)
    assert_scores_close(got[rows], ref, score_tol(ref, wq[rows][:, None, :], qn, dn, RTOL_F32), "full-size scores")


@pytest.mark.parametrize("beam,width", [(128, 1), (2144, 1), (2112, 16)])
def test_full_size_search_replay(full, beam, width):
    """All 10,000 queries are searched exactly as bench.py does (2112 with sixteen parents per iteration is the setting
    it times on this workload); for a sample the oracle's search, replayed on the GPU's own scores, must return the same
    ids and scores bit for bit."""
    w, docs, qs, bp, ix, D, Q = full
    _say(f"full size: search beam {beam}, {width} parent(s) per iteration")
    nq, N, k = qs.n, docs.n, w.k
    wq = np.tile(np.float32(w.weights), (nq, 1))
    ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, k, beam, wq, 0, width)]
    counts, ms = ix.search_stats(nq)
    counts = counts.cpu().numpy()
    sem, _, _, ent = [t.cpu().numpy() for t in ix.export_graph()]
    sample = np.arange(0, nq, nq // 100)[:100]
    table = _score_table(w, ix, sample, wq)
    for x, qi in enumerate(sample):
        oi, os_, nv = O.search(D, sem, ent, Q, int(qi), wq[qi], k, beam, 0, width, score_table=table[x])
        assert np.array_equal(ids[qi], oi), (qi, beam)
        assert np.array_equal(sc[qi], os_), (qi, beam)
        assert counts[qi, 0] == nv, (qi, counts[qi], nv)     # the same documents were scored
    # scores of the answers agree with the oracle's own arithmetic
    ref = O.hybrid_block(Q, sample, D, ids[sample], wq[sample])
    qn = row_norms(w.queries)[sample][:, None]
    dn = np.linalg.norm(w.docs.dense[ids[sample].ravel()].astype(np.float64), axis=1).reshape(len(sample), k)
    tol = score_tol(ref, wq[sample][:, None, :], qn, dn, RTOL_F32)[:, :, 3]
    assert (np.abs(sc[sample] - ref[:, :, 3]) <= tol).all()
    _say(f"  kernel {ms:.1f} ms, {counts[:, 0].mean():.0f} candidates/query, {counts[:, 2].sum() / counts[:, 0].sum():.2f} without dense row")


@pytest.mark.parametrize("beam,kw_all", [(128, False), (1024, True)])
def test_full_size_keyword_search_replay(full, beam, kw_all):
    """Keyword-constrained search over all 10,000 queries (1-2 required terms drawn from each query's own text);
    sampled queries are replayed by the oracle on the GPU's scores."""
    w, docs, qs, bp, ix, D, Q = full
    _say(f"full size: keyword search beam {beam} all={kw_all}")
    nq, k = qs.n, w.k
    wq = np.tile(np.float32(w.weights), (nq, 1))
    kw = make_keywords(w.queries, seed=1, max_terms=2, stride=2, p_none=0.05)
    ids, sc = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, k, beam, kw, wq, kw_all)]
    counts, ms = ix.search_stats(nq)
    counts = counts.cpu().numpy()
    sem, ke, kc, ent = [t.cpu().numpy() for t in ix.export_graph()]
    sample = np.arange(7, nq, nq // 32)[:32]
    table = _score_table(w, ix, sample, wq)
    for x, qi in enumerate(sample):
        kwl = [int(t) for t in kw[qi] if t >= 0]
        oi, os_, nv = O.search_kw(D, sem, ke, kc, ent, Q, int(qi), wq[qi], k, beam, kwl, kw_all, score_table=table[x])
        assert np.array_equal(ids[qi], oi), (qi, beam)
        assert np.array_equal(sc[qi], os_), (qi, beam)
        assert counts[qi, 0] == nv, (qi, counts[qi], nv)
    # every answer of every query holds its required terms
    ip, tx = w.docs.tx_indptr, w.docs.tx_idx
    for qi in range(0, nq, 37):
        kwl = set(int(t) for t in kw[qi] if t >= 0)
        if not kwl:
            continue
        for v in ids[qi][ids[qi] >= 0]:
            terms = set(tx[ip[v]:ip[v + 1]].tolist())
            assert (kwl <= terms) if kw_all else bool(kwl & terms), (qi, v)
    _say(f"  kernel {ms:.1f} ms, {counts[:, 0].mean():.0f} candidates/query, answers/query {np.mean((ids >= 0).sum(1)):.2f}")


def test_full_size_build_stages_sampled(full):
    """Each construction stage re-run on the GPU for sampled nodes at full size
    and compared with the oracle fed the same inputs."""
    w, docs, qs, bp, ix, D, Q = full
    N, R, K, S, P = docs.n, bp.degree, bp.knn_k, bp.nd_sample, (bp.degree + 5) // 6
    wv = np.array([1, 1, 1], np.float32)
    dn = row_norms(w.docs)
    all_nodes = np.sort(np.random.default_rng(5).choice(N, 1000, replace=False)).astype(np.int32)
    nodes = all_nodes[::10]            # the oracle's exhaustive seed costs 0.1 s a node: 100 of the 1000
    _say("full size: seed")
    ids, sc = [t.cpu().numpy() for t in ix.stage_seed_knn(K, nodes)]
    oid, osc = O.seed_knn(D, nodes, K)
    assert_ranked_equiv(ids, sc, oid, osc, lambda r, s: RTOL_F32 * dn[nodes[r]] * dn.max(),
                        lambda r, j: float(np.dot(D.dense[nodes[r]].astype(np.float64), D.dense[j].astype(np.float64))), "seed")
    _say("full size: refine")
    nodes = all_nodes
    seed_all, seed_sc = ix.stage_seed_knn(K)
    spi = torch.full((3, N, P), -1, dtype=torch.int32, device=docs.device)
    sps = torch.full((3, N, P), -np.inf, dtype=torch.float32, device=docs.device)
    g = [t.cpu().numpy() for t in ix.stage_refine(K, S, P, seed_all, spi, sps, nodes)]
    seed_np = seed_all.cpu().numpy()
    o = O.refine_round(D, wv, K, S, P, seed_np, spi.cpu().numpy(), sps.cpu().numpy(), node_ids=nodes)

    def oscore(r, j, col=3):
        return float(O.hybrid_block(D, [nodes[r]], D, [[j]], wv)[0, 0, col])
    assert_ranked_equiv(g[0], g[1], o[0], o[1], lambda r, s: RTOL_F32 * (dn[nodes[r]] * dn.max() + abs(s)), oscore, "refine")
    for p in range(3):
        tol = (lambda r, s: RTOL_F32 * dn[nodes[r]] * dn.max()) if p == 0 else (lambda r, s: RTOL_F32 * abs(s) + 1e-30)
        assert_ranked_equiv(g[2][p], g[3][p], o[2][p], o[3][p], tol, lambda r, j, p=p: oscore(r, j, p), f"path list {p}")
    _say("full size: prune")
    # one full GPU round gives realistic lists for every node
    ids1, sc1, spi1, sps1 = ix.stage_refine(K, S, P, seed_all, spi, sps)
    pr = ix.stage_prune(K, R, ids1, sc1, nodes)
    pm, count, sorted_ids, se, ke, ke_count, flag = [pr[n].cpu().numpy() for n in ("pm", "count", "sorted_ids", "se", "ke", "ke_count", "flag")]
    ids1n, sc1n = ids1.cpu().numpy(), sc1.cpu().numpy()
    self_gpu = ix.export_ingest()[3].cpu().numpy()
    for x, u in enumerate(nodes):
        idl = ids1n[u]
        if x < 4:
            opm = O.pairwise(D, wv, idl)
            tol = RTOL_F32 * (np.outer(dn[idl], dn[idl]) + np.abs(opm))
            assert (np.abs(pm[x] - opm) <= tol).all(), (u, np.max(np.abs(pm[x] - opm) / tol))
        cnt, order = O.detour_sort(idl, sc1n[u], pm[x])
        assert np.array_equal(count[x], cnt) and np.array_equal(sorted_ids[x], idl[order])
        se_pos, ke_pos, fl = O.ip_prune(D, int(u), R, R // 2, idl, order, pm[x], self_gpu[idl])
        assert np.array_equal(se[x][:len(se_pos)], idl[se_pos]) and (se[x][len(se_pos):] == -1).all()
        assert ke_count[x] == len(ke_pos) and np.array_equal(ke[x][:len(ke_pos)], idl[ke_pos])
        assert np.array_equal(flag[x], fl)
    _say("full size: assemble")
    allp = ix.stage_prune(K, R, ids1, sc1, want_pm=False)
    graph = ix.stage_assemble(R, K, P, allp["se"], allp["sorted_ids"], spi1).cpu().numpy()
    ref = O.assemble(N, R, K, P, allp["se"].cpu().numpy(), allp["sorted_ids"].cpu().numpy(), spi1.cpu().numpy(), node_ids=nodes)
    assert np.array_equal(graph[nodes], ref)
    assert np.array_equal(ix.stage_entry_points(64).cpu().numpy(), O.entry_points(self_gpu, 64))


WEIGHT_SETTINGS = [(1, 0, 0), (0, 1, 0), (0, 0, 1), (0.5, 0.5, 0), (0.34, 0.33, 0.33)]


@pytest.mark.parametrize("wset", WEIGHT_SETTINGS)
def test_dynamic_fusion_sweep(full, wset):
    """Config 4: the same index, no rebuild, searched under another weight
    vector through set_weights; ground truth recomputed per setting."""
    w, docs, qs, bp, ix, D, Q = full
    nq, k = qs.n, w.k
    graph_before = ix.export_graph()[0].clone()
    ix.set_weights(wset)
    t0 = time.time()
    gt, gts = [t.cpu().numpy() for t in ix.bruteforce_topk(qs, k)]
    # the exhaustive scorer itself against the oracle on a few queries
    sample = np.arange(0, nq, nq // 6)[:6]
    wrow = np.tile(np.float32(wset), (len(sample), 1))
    oid, osc = O.bruteforce_topk(Q, sample, D, wrow, k)
    qn = row_norms(w.queries); dmax = 1.0 + 1e-6

    def oscore(r, j):
        return float(O.hybrid_block(Q, [sample[r]], D, [[j]], wrow[r])[0, 0, 3])
    assert_ranked_equiv(gt[sample], gts[sample], oid, osc, lambda r, s: RTOL_F32 * (abs(wset[0]) * qn[sample[r]] * dmax + abs(s)),
                        oscore, f"ground truth {wset}")
    res = []
    for beam in (128, 1024):
        ids, _ = ix.search_batch(qs, k, beam)            # default weights of the index
        torch.cuda.synchronize()
        t1 = time.time()
        ids, _ = ix.search_batch(qs, k, beam)
        torch.cuda.synchronize()
        dt = time.time() - t1
        rec = float(np.mean([len(set(a) & set(b)) / k for a, b in zip(ids.cpu().numpy(), gt)]))
        res.append((beam, round(rec, 4), round(nq / dt)))
    _say(f"weights {wset}: (beam, recall@10, qps) = {res}")
    assert torch.equal(graph_before, ix.export_graph()[0])          # no rebuild happened
    assert res[1][1] >= res[0][1] - 1e-9 and res[1][1] > 0.3
    ix.set_weights(w.weights)


def test_full_size_insertion_sampled(full):
    """Insertion at the size bench.py --insert measures (the last 20 % of config 2 into an index over the first
    80 %): sampled new documents are checked step by step against the oracle fed the GPU's previous step."""
    w, docs, qs, bp, ix, D, Q = full
    from paper_2511_00855_amd.synth import subset_vecset
    n1 = docs.n
    n0 = n1 - n1 // 5
    _say(f"full size: insertion of {n1 - n0} documents into {n0}")
    old_docs = B.DeviceVecs(subset_vecset(w.docs, np.arange(n0)))
    old = B.Index.build(old_docs, bp)
    t0 = time.time()
    new, tr = old.insert(docs, trace=True)
    torch.cuda.synchronize()
    _say(f"  inserted in {time.time() - t0:.2f}s {new.build_timings()}")
    tr = {k: v.cpu().numpy() for k, v in tr.items()}
    K, R, P = bp.knn_k, bp.degree, (bp.degree + 5) // 6
    wv = np.array([1, 1, 1], np.float32)
    sem_old, _, _, ent_old = [t.cpu().numpy() for t in old.export_graph()]
    g_pad = np.vstack([sem_old, np.full((n1 - n0, R), -1, np.int32)])
    sample = np.sort(np.random.default_rng(9).choice(np.arange(n0, n1), 12, replace=False))
    # the enlarged corpus is the whole of config 2, so the oracle's S0 of the fixture applies
    allc = np.tile(np.arange(n1, dtype=np.int32), (len(sample), 1))
    table = new.hybrid_scores_docs(sample.astype(np.int32), allc, wv).cpu().numpy()[:, :, 3]
    for x, u in enumerate(sample):
        j = u - n0
        oi, os_, _ = O.search(D, g_pad, ent_old, D, int(u), wv, K, 2 * K, score_table=table[x])
        assert np.array_equal(tr["cand1_ids"][j], oi) and np.array_equal(tr["cand1_sc"][j], os_), u
        mi, ms = O.merge_ranked(tr["cand1_ids"][j], tr["cand1_sc"][j], tr["cand2_ids"][j], tr["cand2_sc"][j], K)
        assert np.array_equal(tr["merged_ids"][j], mi) and np.array_equal(tr["merged_sc"][j], ms), u
        assert set(tr["knn_ids"][j].tolist()) == set(mi.tolist())
        # set two lies among the new documents and its scores are the oracle's
        c2 = tr["cand2_ids"][j]
        assert ((c2 >= n0) | (c2 < 0)).all()
        ref = O.hybrid_block(D, [int(u)], D, [np.maximum(c2, 0)], wv)[0, :, 3]
        ok = c2 >= 0
        assert np.allclose(tr["cand2_sc"][j][ok], ref[ok], rtol=1e-4, atol=1e-5), u
    # pruning of the sampled new documents replayed on the GPU's own neighbourhood similarities; assembly exact
    se, srt, spi, _ = [t.cpu().numpy() for t in new.export_build_state()]
    sem, ke, kc, ent = [t.cpu().numpy() for t in new.export_graph()]
    knn_full = torch.full((n1, K), -1, dtype=torch.int32, device=docs.device)
    knn_sc_full = torch.full((n1, K), -np.inf, dtype=torch.float32, device=docs.device)
    knn_full[n0:] = torch.from_numpy(tr["knn_ids"]).to(docs.device)
    knn_sc_full[n0:] = torch.from_numpy(tr["knn_sc"]).to(docs.device)
    g = new.stage_prune(K, R, knn_full, knn_sc_full, sample.astype(np.int32))
    pm = g["pm"].cpu().numpy()
    self_gpu = new.export_ingest()[3].cpu().numpy()
    for x, u in enumerate(sample):
        j = u - n0
        r = O.prune_node(D, int(u), wv, R, R // 2, tr["knn_ids"][j], tr["knn_sc"][j], self_all=self_gpu, Pm=pm[x])
        assert np.array_equal(se[u][:len(r.se)], r.se) and np.array_equal(srt[u], r.sorted), u
        assert kc[u] == len(r.ke) and np.array_equal(ke[u][:len(r.ke)], r.ke), u
    rows = np.concatenate([sample, np.arange(0, n0, n0 // 40)])
    assert np.array_equal(sem[rows], O.assemble(n1, R, K, P, se, srt, spi, node_ids=rows))
    assert np.array_equal(ent, O.entry_points(self_gpu, bp.n_entry))
    new.close(); old.close()


def test_bf16_corpus_at_scale_sampled():
    """150,000 documents of config 3's shape (d = 1024 stored bf16): the exact seed lists come from the thresholded
    sweep over all columns in the configuration a million-document build runs it in (19 slabs of 8,192 rows,
    256x256 tiles, inner and edge instantiations).  Sampled rows against the oracle's exhaustive top-K, the same
    rows bit for bit against the sweep over a node list (the general instantiation), and a search replay."""
    t0 = time.time()
    w = make_workload("cfg3", seed=4, n=150_000, nq=16)
    _say(f"150k bf16 documents generated in {time.time() - t0:.1f}s")
    docs = B.DeviceVecs(w.docs, bf16=True)
    qs = B.DeviceVecs(w.queries)
    bp = B.build_params(w.degree)
    K = bp.knn_k
    ix = B.Index.build(docs, bp)
    torch.cuda.synchronize()
    _say(f"built {ix.build_timings()}")
    all_ids, all_sc = [t.cpu().numpy() for t in ix.stage_seed_knn(K)]
    nodes = np.sort(np.random.default_rng(6).choice(docs.n, 48, replace=False)).astype(np.int32)
    nodes[0], nodes[-1] = 0, docs.n - 1                       # first row of the first slab, last row of the ragged last one
    sub_ids, sub_sc = [t.cpu().numpy() for t in ix.stage_seed_knn(K, nodes)]
    assert np.array_equal(sub_ids, all_ids[nodes]) and np.array_equal(sub_sc, all_sc[nodes])
    D = O.encode_docs(w.docs)
    dn = row_norms(w.docs)
    _say("oracle: exhaustive dense top-K of the sampled rows")
    oid, osc = O.seed_knn(D, nodes, K)
    assert_ranked_equiv(sub_ids, sub_sc, oid, osc, lambda r, s: RTOL_F32 * dn[nodes[r]] * dn.max(),
                        lambda r, j: float(np.dot(D.dense[nodes[r]].astype(np.float64), D.dense[j].astype(np.float64))), "bf16 seed")
    # the built index searches like the oracle on the same graph
    Q = O.VS(w.queries)
    wq = np.tile(np.float32(w.weights), (qs.n, 1))
    sem, _, _, ent = [t.cpu().numpy() for t in ix.export_graph()]
    ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, 10, 256, wq)]
    table = ix.hybrid_scores(qs, np.tile(np.arange(docs.n, dtype=np.int32), (qs.n, 1)), wq).cpu().numpy()[:, :, 3]
    for qi in range(qs.n):
        oi, os_, _ = O.search(D, sem, ent, Q, qi, wq[qi], 10, 256, score_table=table[qi])
        assert np.array_equal(ids[qi], oi) and np.array_equal(sc[qi], os_), qi
    ix.close()
