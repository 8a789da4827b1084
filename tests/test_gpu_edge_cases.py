"""GPU parity on degenerate and boundary inputs: empty lists, lists longer
than every on-chip structure (register slots, LDS tables, LDS staging),
minimal dimensions, tiny corpora, one query, k = beam, wide searches."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2511_00855_amd import binding as B
from paper_2511_00855_amd.synth import make_workload
from parity import RTOL_F32, assert_ranked_equiv, assert_scores_close, row_norms, score_tol

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _drop_lists(v, rows_sp, rows_tx):
    """Empties the sparse list of rows_sp and the text of rows_tx (CSR rebuilt)."""
    for pre, rows in (("sp", rows_sp), ("tx", rows_tx)):
        ip = getattr(v, pre + "_indptr"); idx = getattr(v, pre + "_idx"); val = getattr(v, pre + "_val")
        keep = np.ones(len(idx), bool)
        for r in rows:
            keep[ip[r]:ip[r + 1]] = False
        lens = ip[1:] - ip[:-1]
        lens[list(rows)] = 0
        setattr(v, pre + "_indptr", np.concatenate([[0], np.cumsum(lens)]).astype(np.int64))
        setattr(v, pre + "_idx", idx[keep]); setattr(v, pre + "_val", val[keep])


def _replay_search(ix, docs, qs, w, D, Q, graph, entry, wq, k, L, iters=0, width=1):
    N, nq = docs.n, qs.n
    allc = np.tile(np.arange(N, dtype=np.int32), (nq, 1))
    table = ix.hybrid_scores(qs, allc, wq).cpu().numpy()[:, :, 3]
    ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, k, L, wq, iters, width)]
    for qi in range(nq):
        oi, os_, _ = O.search(D, graph, entry, Q, qi, wq[qi], k, L, iters, width, score_table=table[qi])
        assert np.array_equal(ids[qi], oi), (qi, L, width)
        assert np.array_equal(sc[qi], os_), (qi, L, width)
    return table


@pytest.mark.parametrize("name,kw", [
    # lists beyond the register slots (128 sparse / 64 lexical entries) and the search's query tables (64 / 32)
    ("long", dict(seed=41, n=700, nq=12, dim=64, sp=("poisson", 170), tx=("lognormal", 140), qsp=("poisson", 80), qtx=("poisson", 45))),
    # lists beyond the construction tables (256 / 128) and the LDS staging of the node's lists (512)
    ("huge", dict(seed=42, n=400, nq=6, dim=32, vocab=4000, sp=("poisson", 600), tx=("lognormal", 400), qsp=("poisson", 20), qtx=("poisson", 8))),
    # smallest dense dimension, short lists, some empty ones
    ("thin", dict(seed=43, n=300, nq=10, dim=4, sp=("fixed", 3), tx=("fixed", 5), qsp=("fixed", 2), qtx=("fixed", 2))),
])
def test_boundary_list_lengths(name, kw):
    _say(f"edge case {name}")
    w = make_workload("tiny", **kw)
    if name == "thin":
        _drop_lists(w.docs, rows_sp=[0, 5, 17], rows_tx=[1, 5, 40])
        _drop_lists(w.queries, rows_sp=[0, 3], rows_tx=[1, 3])
    docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
    R, K = 8, 24
    bp = B.build_params(R, knn_k=K, nd_rounds=2, nd_sample=6, n_entry=8, sp_len=3)
    D = O.encode_docs(w.docs); Q = O.VS(w.queries)
    N, nq = docs.n, qs.n
    ix = B.Index.build(docs, bp)
    # S1 against the oracle: every query against every document
    wq = np.random.default_rng(1).uniform(0.1, 1.0, (nq, 3)).astype(np.float32)
    allc = np.tile(np.arange(N, dtype=np.int32), (nq, 1))
    got = ix.hybrid_scores(qs, allc, wq).cpu().numpy()
    ref = O.hybrid_block(Q, np.arange(nq), D, allc, wq)
    tol = score_tol(ref, wq[:, None, :], row_norms(w.queries)[:, None], row_norms(w.docs)[None, :], RTOL_F32)
    assert_scores_close(got, ref, tol, name)
    # search (tables or in-memory lists, register slots or tail loops) replayed by the oracle
    sem, kw_, kc, ent = [t.cpu().numpy() for t in ix.export_graph()]
    for (k, L, iters, width) in ((5, 16, 0, 1), (8, 8, 0, 2), (3, 40, 5, 8)):
        _replay_search(ix, docs, qs, w, D, Q, sem, ent, wq, k, L, iters, width)
    # construction: the whole build equals the chain of stages, and the prune stage replays exactly
    stage = B.Index.ingest(docs, bp)
    ids, sc = stage.stage_seed_knn(K)
    spi = torch.full((3, N, 3), -1, dtype=torch.int32, device=docs.device)
    sps = torch.full((3, N, 3), -np.inf, dtype=torch.float32, device=docs.device)
    for _ in range(2):
        ids, sc, spi, sps = stage.stage_refine(K, 6, 3, ids, spi, sps)
    g = stage.stage_prune(K, R, ids, sc)
    graph = stage.stage_assemble(R, K, 3, g["se"], g["sorted_ids"], spi).cpu().numpy()
    assert np.array_equal(graph, sem)
    pm, count, sorted_ids, se, ke, ke_count, flag = [g[n].cpu().numpy() for n in ("pm", "count", "sorted_ids", "se", "ke", "ke_count", "flag")]
    idn, scn = ids.cpu().numpy(), sc.cpu().numpy()
    self_gpu = stage.export_ingest()[3].cpu().numpy()
    wv = np.array([1, 1, 1], np.float32)
    dn = row_norms(w.docs)
    for u in range(0, N, 7):
        idl = idn[u]
        opm = O.pairwise(D, wv, idl)
        fin = np.isfinite(opm)
        tolm = RTOL_F32 * (np.outer(dn[np.maximum(idl, 0)], dn[np.maximum(idl, 0)]) + np.abs(np.where(fin, opm, 0)))
        assert np.array_equal(fin, np.isfinite(pm[u])) and (np.abs(np.where(fin, pm[u] - opm, 0)) <= tolm).all(), u
        cnt, order = O.detour_sort(idl, scn[u], pm[u])
        assert np.array_equal(count[u], cnt) and np.array_equal(sorted_ids[u], idl[order])
        self_s = np.where(idl >= 0, self_gpu[np.maximum(idl, 0)], -np.inf).astype(np.float32)
        se_pos, ke_pos, fl = O.ip_prune(D, u, R, R // 2, idl, order, pm[u], self_s)
        assert np.array_equal(se[u][:len(se_pos)], idl[se_pos]) and np.array_equal(flag[u], fl)
        assert ke_count[u] == len(ke_pos) and np.array_equal(ke[u][:len(ke_pos)], idl[ke_pos])
    # one refinement round of the oracle on the GPU's seed lists gives the GPU's lists (scores within tolerance)
    seed_ids, _ = stage.stage_seed_knn(K)
    e_i, e_s = O.empty_sp(N, 3)
    g1 = [t.cpu().numpy() for t in stage.stage_refine(K, 6, 3, seed_ids, e_i, e_s)]
    o1 = O.refine_round(D, wv, K, 6, 3, seed_ids.cpu().numpy(), e_i, e_s)
    assert_ranked_equiv(g1[0], g1[1], o1[0], o1[1], lambda r, sc_: RTOL_F32 * (dn[r] * dn.max() + abs(sc_)),
                        lambda r, j: float(O.hybrid_block(D, [r], D, [[j]], wv)[0, 0, 3]), f"{name}: refinement round")
    stage.close(); ix.close()


def test_tiny_corpora_and_single_query():
    _say("edge case: corpora of 2..40 documents")
    for n in (2, 3, 9, 40):
        w = make_workload("tiny", seed=50 + n, n=n, nq=1, dim=8, sp=("fixed", 3), tx=("fixed", 4), vocab=50)
        docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
        bp = B.build_params(4, knn_k=8, nd_rounds=1, nd_sample=4, n_entry=4, sp_len=2)
        ix = B.Index.build(docs, bp)
        sem, _, _, ent = [t.cpu().numpy() for t in ix.export_graph()]
        for u in range(n):
            row = sem[u][sem[u] >= 0]
            assert u not in row and len(set(row.tolist())) == len(row) and (row < n).all()
        D = O.encode_docs(w.docs); Q = O.VS(w.queries)
        wq = np.array([[0.3, 0.3, 0.4]], np.float32)
        for (k, L) in ((1, 1), (4, 4), (min(n, 8), 16)):
            _replay_search(ix, docs, qs, w, D, Q, sem, ent, wq, k, L)
        # with a pool larger than the corpus the search is exhaustive over what the graph reaches
        ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, 8, 64, wq)]
        gt, _ = [t.cpu().numpy() for t in ix.bruteforce_topk(qs, 8, wq)]
        reached = (ids[0] >= 0).sum()
        assert np.array_equal(ids[0][:reached], gt[0][:reached]) or reached < min(n, 8)
        ix.close()


def test_malformed_corpus_is_refused():
    """A corpus is checked once, when an index is made from it: every kernel relies on ascending ids inside the
    vocabulary, ascending row offsets and finite values."""
    _say("edge case: malformed corpora")
    base = make_workload("tiny", seed=61, n=200, nq=2, dim=16)
    bp = B.build_params(8, knn_k=16, nd_rounds=1, nd_sample=4, n_entry=4)

    def broken(change):
        w = make_workload("tiny", seed=61, n=200, nq=2, dim=16)
        change(w.docs)
        return B.DeviceVecs(w.docs)

    def swap(v):          # two neighbouring ids of one row out of order
        r = int(np.argmax(np.diff(v.sp_indptr) >= 2)); p = v.sp_indptr[r]
        v.sp_idx[p], v.sp_idx[p + 1] = v.sp_idx[p + 1], v.sp_idx[p]

    def repeat(v):        # a repeated term
        r = int(np.argmax(np.diff(v.tx_indptr) >= 2)); p = v.tx_indptr[r]
        v.tx_idx[p + 1] = v.tx_idx[p]

    def past_vocab(v): v.tx_idx[v.tx_indptr[3 + 1] - 1] = v.tx_vocab
    def negative_id(v): v.sp_idx[v.sp_indptr[7]] = -2
    def nan_value(v): v.sp_val[5] = np.nan
    def negative_count(v): v.tx_val[9] = -1.0
    def offsets_back(v): v.sp_indptr[10] = v.sp_indptr[9] - 1
    def offsets_past(v): v.tx_indptr[20] = v.tx_indptr[-1] + 3
    def offsets_start(v): v.tx_indptr[0] = 1

    for change in (swap, repeat, past_vocab, negative_id, nan_value, negative_count, offsets_back, offsets_past, offsets_start):
        with pytest.raises(RuntimeError, match="malformed"):
            B.Index.build(broken(change), bp)
        with pytest.raises(RuntimeError, match="malformed"):
            B.Index.ingest(broken(change), bp)
    # a corpus that claims 2^32 list entries or more is refused on its row offsets alone, before any kernel reads a list
    def too_many(v): v.sp_indptr[-1] = (1 << 32) - int(v.tx_indptr[-1])
    for make in (B.Index.build, B.Index.ingest):
        with pytest.raises(RuntimeError, match="fewer than 2\\^32 entries"):
            make(broken(too_many), bp)
    # the untouched corpus builds, and ids outside the corpus are holes for the explicit-pair scorer
    docs = B.DeviceVecs(base.docs); qs = B.DeviceVecs(base.queries)
    ix = B.Index.build(docs, bp)
    cand = np.array([[0, 200, -1, 199, 1 << 30], [-5, 3, 200, 4, 5]], np.int32)
    got = ix.hybrid_scores(qs, cand, np.ones((2, 3), np.float32)).cpu().numpy()
    hole = (cand < 0) | (cand >= 200)
    assert np.isneginf(got[hole]).all() and np.isfinite(got[~hole]).all()
    gd = ix.hybrid_scores_docs(np.array([5, 200, -1], np.int32), np.tile(np.arange(4, dtype=np.int32), (3, 1)),
                               np.ones(3, np.float32)).cpu().numpy()
    assert np.isfinite(gd[0]).all() and np.isneginf(gd[1:]).all()
    ix.close()


def test_pools_beyond_64_kb_of_lds():
    """Beams of 8192 and 16384 (pools of 64 and 128 KB, one workgroup per CU) replayed by the oracle, on a corpus
    larger than the pool."""
    _say("edge case: beams 8192 and 16384")
    w = make_workload("tiny", seed=71, n=24000, nq=4, dim=32)
    docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
    ix = B.Index.build(docs, B.build_params(16, knn_k=32, nd_rounds=1, nd_sample=8, n_entry=16))
    D = O.encode_docs(w.docs); Q = O.VS(w.queries)
    sem, _, _, ent = [t.cpu().numpy() for t in ix.export_graph()]
    wq = np.tile(np.float32(w.weights), (qs.n, 1))
    for (k, L, width) in ((10, 8192, 1), (100, 16384, 1), (10, 12000, 4), (10, 16384, 16)):
        _say(f"  beam {L}, width {width}")
        _replay_search(ix, docs, qs, w, D, Q, sem, ent, wq, k, L, 0, width)
    counts = ix.search_stats(qs.n)[0].cpu().numpy()
    assert (counts[:, 0] > 12000).all()          # the pool did fill
    with pytest.raises(RuntimeError, match="beam"):
        ix.search_batch(qs, 10, 16385, wq)
    ix.close()


@pytest.mark.parametrize("dim,bf16", [(1536, True), (2048, True), (1024, False), (8, True)])
def test_widest_and_narrowest_dense_rows(dim, bf16):
    """The widest rows each storage type allows (24 or 32 query values per lane), and the narrowest bf16 row: scores
    against the oracle, the build's stages chained, and the search replayed."""
    _say(f"edge case: dim {dim} bf16={bf16}")
    w = make_workload("tiny", seed=81, n=500, nq=8, dim=dim, bf16=bf16)
    docs = B.DeviceVecs(w.docs, bf16=bf16); qs = B.DeviceVecs(w.queries)
    bp = B.build_params(8, knn_k=16, nd_rounds=1, nd_sample=4, n_entry=8)
    ix = B.Index.build(docs, bp)
    D = O.encode_docs(w.docs); Q = O.VS(w.queries)
    N, nq = docs.n, qs.n
    wq = np.random.default_rng(3).uniform(0.1, 1.0, (nq, 3)).astype(np.float32)
    allc = np.tile(np.arange(N, dtype=np.int32), (nq, 1))
    got = ix.hybrid_scores(qs, allc, wq).cpu().numpy()
    ref = O.hybrid_block(Q, np.arange(nq), D, allc, wq)
    tol = score_tol(ref, wq[:, None, :], row_norms(w.queries)[:, None], row_norms(w.docs)[None, :], RTOL_F32)
    assert_scores_close(got, ref, tol, f"dim {dim}")
    sem, _, _, ent = [t.cpu().numpy() for t in ix.export_graph()]
    for (k, L, iters, width) in ((5, 16, 0, 1), (8, 64, 0, 2), (10, 300, 0, 1)):
        _replay_search(ix, docs, qs, w, D, Q, sem, ent, wq, k, L, iters, width)
    # keyword search runs another instantiation of the same kernel
    from paper_2511_00855_amd.synth import make_keywords
    kw = make_keywords(w.queries, seed=4, max_terms=2, stride=2, p_none=0.2)
    table = ix.hybrid_scores(qs, allc, wq).cpu().numpy()[:, :, 3]
    _, ke, kc, _ = [t.cpu().numpy() for t in ix.export_graph()]
    kids, ksc = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, 5, 32, kw, wq)]
    for qi in range(nq):
        terms = [int(t) for t in kw[qi] if t >= 0]
        oi, os_, _ = O.search_kw(D, sem, ke, kc, ent, Q, qi, wq[qi], 5, 32, terms, score_table=table[qi])
        assert np.array_equal(kids[qi], oi) and np.array_equal(ksc[qi], os_), qi
    gt, gts = [t.cpu().numpy() for t in ix.bruteforce_topk(qs, 5, wq)]
    ob = [O.bruteforce_topk(Q, [qi], D, wq[qi], 5) for qi in range(nq)]
    oi, osc = np.stack([b[0][0] for b in ob]), np.stack([b[1][0] for b in ob])
    qn, dn = row_norms(w.queries), row_norms(w.docs)
    assert_ranked_equiv(gt, gts, oi, osc, lambda r, sc_: RTOL_F32 * (abs(wq[r, 0]) * qn[r] * dn.max() + abs(sc_)),
                        lambda r, j: float(ref[r, j, 3]), f"dim {dim}: exhaustive top-5")
    ix.close()


@pytest.mark.parametrize("dim", [8, 64, 72, 128, 192, 200, 1024])
def test_bf16_threshold_sweep_on_ragged_shapes(dim, debug_knobs):
    """The thresholded seed sweep of bf16 rows (256x256 tiles, two LDS stages) against the score-row path (128x128
    tiles, itself checked against the oracle elsewhere): same ids and the same score bits, with a ragged last row
    tile, a ragged last column tile and a last chunk of fewer than 64 columns; also with overflowing buffers."""
    _say(f"edge case: bf16 threshold sweep, dim {dim}")
    w = make_workload("tiny", seed=91, n=777, nq=2, dim=dim, bf16=True, sp=("fixed", 4), tx=("fixed", 4))
    docs = B.DeviceVecs(w.docs, bf16=True)
    ix = B.Index.ingest(docs, B.build_params(8, knn_k=24, nd_rounds=1, nd_sample=4, n_entry=4))
    K = 24
    exact = [t.cpu().numpy() for t in ix.stage_seed_knn(K)]
    Dd = O.encode_docs(w.docs)
    oi, os_ = O.seed_knn(Dd, np.arange(docs.n), K)
    dn = row_norms(w.docs)
    assert_ranked_equiv(exact[0], exact[1], oi, os_, lambda r, sc_: RTOL_F32 * dn[r] * dn.max(),
                        lambda r, j: float(np.dot(Dd.dense[r].astype(np.float64), Dd.dense[j].astype(np.float64))), f"bf16 seed dim {dim}")
    nodes = np.arange(5, 700, 3, dtype=np.int32)
    exact_sub = [t.cpu().numpy() for t in ix.stage_seed_knn(K, nodes)]
    debug_knobs("seed_sample_cols", 128)
    for cap in (0, 32):
        debug_knobs("seed_buffer_cap", cap)
        thr = [t.cpu().numpy() for t in ix.stage_seed_knn(K)]
        assert np.array_equal(thr[0], exact[0]) and np.array_equal(thr[1], exact[1])
        thr_sub = [t.cpu().numpy() for t in ix.stage_seed_knn(K, nodes)]
        assert np.array_equal(thr_sub[0], exact_sub[0]) and np.array_equal(thr_sub[1], exact_sub[1])
    ix.close()


def test_threshold_sweep_with_more_candidates_than_a_wave_stages(debug_knobs):
    """The sweeps note a tile's candidates in LDS, a wave in its own part, before they are appended to the rows' buffers;
    what a part cannot hold is appended on the spot.  A threshold taken from very few sampled columns lets nearly half of
    every tile pass, far more than the parts hold: the lean 256x256 kernel, its ragged edge tiles and (f32 rows) the
    128x128 kernel must still give the exact lists, bit for bit."""
    _say("edge case: threshold sweeps with overflowing staging parts")
    K = 120
    for bf16 in (True, False):
        w = make_workload("tiny", seed=93, n=1100, nq=2, dim=64, bf16=bf16, sp=("fixed", 4), tx=("fixed", 4))
        docs = B.DeviceVecs(w.docs, bf16=bf16)
        ix = B.Index.ingest(docs, B.build_params(8, knn_k=K, nd_rounds=1, nd_sample=4, n_entry=4))
        exact = [t.cpu().numpy() for t in ix.stage_seed_knn(K)]
        nodes = np.arange(3, 1000, 2, dtype=np.int32)
        exact_sub = [t.cpu().numpy() for t in ix.stage_seed_knn(K, nodes)]
        debug_knobs("seed_sample_cols", 256)
        thr = [t.cpu().numpy() for t in ix.stage_seed_knn(K)]
        assert np.array_equal(thr[0], exact[0]) and np.array_equal(thr[1], exact[1]), bf16
        thr_sub = [t.cpu().numpy() for t in ix.stage_seed_knn(K, nodes)]
        assert np.array_equal(thr_sub[0], exact_sub[0]) and np.array_equal(thr_sub[1], exact_sub[1]), bf16
        debug_knobs("seed_sample_cols", 0)
        ix.close()


@pytest.mark.parametrize("bf16", [True, False])
def test_symmetric_seed_sweep_against_one_sided_and_exact(bf16, debug_knobs):
    """Whole-corpus seed lists come from a sweep over the tiles on and above the diagonal of D D^T (256x256 tiles for
    bf16 rows, 128x128 for f32 rows), every score offered to both of its documents, with thresholds that are the m-th
    best (m < K) of a column sample.  Same lists, bit for bit, as the one-sided sweep and as the exact score rows; also
    when rows overflow their buffers or fall short of K candidates and are redone.  The symmetric sweep must have
    executed well under the one-sided FLOPs."""
    _say(f"edge case: symmetric seed sweep, bf16={bf16}")
    K = 200
    w = make_workload("tiny", seed=95, n=3000, nq=2, dim=64, bf16=bf16, sp=("fixed", 4), tx=("fixed", 4))
    docs = B.DeviceVecs(w.docs, bf16=bf16)

    def lists(**knobs):
        for k, v in knobs.items():
            debug_knobs(k, v)
        ix = B.Index.ingest(docs, B.build_params(8, knn_k=K, nd_rounds=1, nd_sample=4, n_entry=4))
        out = [t.cpu().numpy() for t in ix.stage_seed_knn(K)]
        flops = ix.build_counters()["seed_flops"]
        ix.close()
        for k in knobs:
            debug_knobs(k, 0)
        return out, flops

    exact, f_exact = lists()
    sym, f_sym = lists(seed_sample_cols=256)
    one, f_one = lists(seed_sample_cols=256, seed_one_sided=1)
    ovf, _ = lists(seed_sample_cols=256, seed_buffer_cap=512)        # most rows overflow and are redone
    short, _ = lists(seed_sample_cols=256, seed_tau_ulps=1 << 22)    # thresholds far too high: rows fall short
    for name, got in (("symmetric", sym), ("one-sided", one), ("overflowing", ovf), ("short", short)):
        assert np.array_equal(got[0], exact[0]) and np.array_equal(got[1], exact[1]), name
    assert f_sym < 0.75 * f_one, (f_sym, f_one, f_exact)


def test_random_search_settings_replayed():
    """Forty seeded draws of (k, beam, parents per iteration, iteration cap) across the three workgroup sizes of the
    search (256, 512 and 1024 threads), on two graphs of different degree, each replayed by the oracle on the GPU's own
    score table: ids, scores and the number of scored documents bit for bit.  The draws include pools that never fill,
    more candidates per iteration than the workgroup has threads, and caps that stop the search mid-way."""
    rng = np.random.default_rng(2024)
    for degree, n in ((64, 20000), (24, 30000)):
        w = make_workload("tiny", seed=90 + degree, n=n, nq=3, dim=32)
        docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
        ix = B.Index.build(docs, B.build_params(degree, knn_k=2 * degree, nd_rounds=1, nd_sample=8, n_entry=32))
        D = O.encode_docs(w.docs); Q = O.VS(w.queries)
        sem, _, _, ent = [t.cpu().numpy() for t in ix.export_graph()]
        wq = rng.uniform(0.1, 1.0, (qs.n, 3)).astype(np.float32)
        allc = np.tile(np.arange(docs.n, dtype=np.int32), (qs.n, 1))
        table = ix.hybrid_scores(qs, allc, wq).cpu().numpy()[:, :, 3]
        for case in range(20):
            beam = int(rng.choice([rng.integers(1, 400), rng.integers(400, 5000), rng.integers(5000, 16385)]))
            width = int(rng.integers(1, 17))
            k = int(min(beam, rng.choice([1, 10, 100])))
            iters = int(rng.choice([0, 0, rng.integers(1, 60)]))
            try:
                ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, k, beam, wq, iters, width)]
            except B.ApError as e:   # the only admissible refusal: the setting does not fit the LDS
                assert "LDS" in str(e), (degree, beam, width, str(e))
                assert (beam + width * degree) * 8 + width * degree * 16 > 150 * 1024, (degree, beam, width)
                continue
            counts = ix.search_stats(qs.n)[0].cpu().numpy()
            _say(f"  degree {degree}: k {k} beam {beam} parents {width} cap {iters}: {counts[:, 0].mean():.0f} scored, {counts[:, 1].mean():.0f} iterations")
            for qi in range(qs.n):
                oi, os_, nv = O.search(D, sem, ent, Q, qi, wq[qi], k, beam, iters, width, score_table=table[qi])
                assert np.array_equal(ids[qi], oi), (degree, qi, k, beam, width, iters)
                assert np.array_equal(sc[qi], os_), (degree, qi, k, beam, width, iters)
                assert counts[qi, 0] == nv, (degree, qi, k, beam, width, iters, counts[qi], nv)
        ix.close()


def test_query_tables_and_query_lists_give_the_same_bits(debug_knobs):
    """The search looks a candidate's terms up in LDS tables built from the query's lists, and in the lists themselves
    when a query is too long for the tables (or no hash multiplier fits it).  The debug setting forces the second way
    on ordinary queries: answers, scores and counters must be the same bits, in all three workgroup sizes and in the
    keyword search."""
    from paper_2511_00855_amd.synth import make_keywords
    w = make_workload("tiny", seed=77, n=14000, nq=6, dim=48)
    docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
    ix = B.Index.build(docs, B.build_params(32, knn_k=64, nd_rounds=1, nd_sample=8, n_entry=16))
    wq = np.random.default_rng(3).uniform(0.1, 1.0, (qs.n, 3)).astype(np.float32)
    kw = make_keywords(w.queries, seed=5, max_terms=2, stride=2)
    got = {}
    for lists in (0, 1):
        debug_knobs("search_query_lists", lists)
        for (k, L, width) in ((10, 64, 1), (10, 700, 3), (5, 5000, 4), (10, 12000, 16)):
            ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, k, L, wq, 0, width)]
            got[(lists, "plain", L)] = (ids, sc, ix.search_stats(qs.n)[0].cpu().numpy())
        ids, sc = [t.cpu().numpy() for t in ix.search_batch_keywords(qs, 10, 300, kw, wq)]
        got[(lists, "kw", 300)] = (ids, sc, ix.search_stats(qs.n)[0].cpu().numpy())
    for (lists, kind, L), v in got.items():
        if lists == 0:
            o = got[(1, kind, L)]
            for x, y in zip(v, o):
                assert np.array_equal(x, y), (kind, L)
    ix.close()
