"""Parity at the size and in the launch configurations of the headline workload (config 3: 1,000,000 documents,
d = 1024 stored bf16, degree 64): the search at the large beams that reach the recall target there -- pools of
4096 to 16384 entries, searched by workgroups of 512 and 1024 threads with the pipelined scoring, several parents
per iteration -- replayed by the oracle bit for bit (ids, scores, number of scored documents), and every
construction stage on sampled nodes (1,000; the oracle's exhaustive seed on 100) against the oracle fed the GPU's
previous stage.  AP_TEST_MILLION_N in the environment shrinks the corpus for a quicker run of the same tests."""
import os
import time

import numpy as np
import pytest
import torch

import oracle as O
from paper_2511_00855_amd import binding as B
from paper_2511_00855_amd.synth import make_workload
from parity import RTOL_F32, assert_ranked_equiv, row_norms, score_tol

pytestmark = pytest.mark.gpu

N_DOCS = int(os.environ.get("AP_TEST_MILLION_N", "1000000"))
NQ = 32


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def million():
    t0 = time.time()
    w = make_workload("cfg3", seed=0, n=N_DOCS, nq=NQ, progress=lambda m: _say(f"  generating: {m}"))
    _say(f"cfg3 shape, {N_DOCS} documents, generated in {time.time() - t0:.1f}s")
    docs = B.DeviceVecs(w.docs, bf16=True)
    qs = B.DeviceVecs(w.queries)
    bp = B.build_params(w.degree)                      # what bench.py uses
    t0 = time.time()
    ix = B.Index.build(docs, bp)
    torch.cuda.synchronize()
    _say(f"built in {time.time() - t0:.2f}s {ix.build_timings()}")
    D = O.encode_docs(w.docs)
    Q = O.VS(w.queries)
    wq = np.tile(np.float32(w.weights), (NQ, 1))
    # fused scores of every document for every query from the pair scorer: what the oracle's replay runs on
    table = np.empty((NQ, N_DOCS), np.float32)
    allc = torch.arange(N_DOCS, dtype=torch.int32, device=docs.device).repeat(8, 1)
    for q0 in range(0, NQ, 8):
        from paper_2511_00855_amd.synth import subset_vecset
        sub = B.DeviceVecs(subset_vecset(w.queries, np.arange(q0, q0 + 8)))
        table[q0:q0 + 8] = ix.hybrid_scores(sub, allc, wq[q0:q0 + 8]).cpu().numpy()[:, :, 3]
    del allc
    sem, _, _, ent = [t.cpu().numpy() for t in ix.export_graph()]
    yield w, docs, qs, bp, ix, D, Q, wq, table, sem, ent
    ix.close()


@pytest.mark.parametrize("beam,width,nsample", [(4096, 1, 32), (4096, 4, 16), (4096, 16, 8), (8192, 8, 16), (15360, 16, 8), (16384, 1, 8), (16384, 8, 16), (16384, 16, 16), (2144, 2, 16)])
def test_million_search_replay(million, beam, width, nsample):
    """beam 4096: workgroups of 512 threads (with sixteen parents an iteration's candidates outnumber them); 8192 and beyond: 1024 threads (the pool has the CU to itself; 16384 with
    sixteen parents is the most the LDS holds, 15360 with sixteen is the setting bench.py times); 2144: the 256-thread kernel on bf16 rows.  All 32 queries are searched
    in one launch; a sample is replayed."""
    w, docs, qs, bp, ix, D, Q, wq, table, sem, ent = million
    k = w.k
    _say(f"million: search beam {beam} width {width}")
    ids, sc = [t.cpu().numpy() for t in ix.search_batch(qs, k, beam, wq, search_width=width)]
    counts, ms = ix.search_stats(NQ)
    counts = counts.cpu().numpy()
    assert (counts[:, 0] > min(beam, N_DOCS // 2)).all()            # the pool did fill
    t0 = time.time()
    for qi in range(nsample):
        oi, os_, nv = O.search(D, sem, ent, Q, qi, wq[qi], k, beam, 0, width, score_table=table[qi])
        assert np.array_equal(ids[qi], oi), (qi, beam, width)
        assert np.array_equal(sc[qi], os_), (qi, beam, width)
        assert counts[qi, 0] == nv, (qi, counts[qi], nv)
    # the scores of the answers agree with the oracle's own arithmetic (fp64 over the same bf16 values)
    rows = np.arange(nsample)
    ref = O.hybrid_block(Q, rows, D, ids[rows], wq[rows])
    qn = row_norms(w.queries)[rows][:, None]
    dn = np.linalg.norm(w.docs.dense[ids[rows].ravel()].astype(np.float64), axis=1).reshape(nsample, k)
    tol = score_tol(ref, wq[rows][:, None, :], qn, dn, RTOL_F32)[:, :, 3]
    assert (np.abs(sc[rows] - ref[:, :, 3]) <= tol).all()
    _say(f"  kernel {ms:.1f} ms for {NQ} queries, {counts[:, 0].mean():.0f} candidates/query, "
         f"{counts[:, 2].sum() / counts[:, 0].sum():.2f} without dense row; oracle replay of {nsample} in {time.time() - t0:.1f}s")


def test_million_build_stages_sampled(million):
    w, docs, qs, bp, ix, D, Q, wq, table, sem, ent = million
    N, R, K, S, P = docs.n, bp.degree, bp.knn_k, bp.nd_sample, (bp.degree + 5) // 6
    wv = np.array([1, 1, 1], np.float32)
    dn = row_norms(w.docs)
    all_nodes = np.sort(np.random.default_rng(5).choice(N, 1000, replace=False)).astype(np.int32)
    nodes = all_nodes[::10]                            # the oracle's exhaustive seed costs about a second a node here
    _say("million: seed (100 nodes)")
    ids, sc = [t.cpu().numpy() for t in ix.stage_seed_knn(K, nodes)]
    t0 = time.time()
    oid, osc = O.seed_knn(D, nodes, K)
    _say(f"  oracle seed of {len(nodes)} nodes: {time.time() - t0:.1f}s")
    assert_ranked_equiv(ids, sc, oid, osc, lambda r, s: RTOL_F32 * dn[nodes[r]] * dn.max(),
                        lambda r, j: float(np.dot(D.dense[nodes[r]].astype(np.float64), D.dense[j].astype(np.float64))), "seed")
    _say("million: refine (1000 nodes)")
    nodes = all_nodes
    seed_all, seed_sc = ix.stage_seed_knn(K)
    # the sweep over all rows (inner tiles) and the node-list sweep (general tiles) give the same bits
    assert np.array_equal(seed_all.cpu().numpy()[all_nodes[::10]], ids)
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
    _say("million: prune (1000 nodes)")
    ids1, sc1, spi1, sps1 = ix.stage_refine(K, S, P, seed_all, spi, sps)   # one full GPU round gives realistic lists
    del seed_all, seed_sc
    pr = ix.stage_prune(K, R, ids1, sc1, nodes)
    pm, count, sorted_ids, se, ke, ke_count, flag = [pr[n].cpu().numpy() for n in ("pm", "count", "sorted_ids", "se", "ke", "ke_count", "flag")]
    ids1n, sc1n = ids1.cpu().numpy(), sc1.cpu().numpy()
    self_gpu = ix.export_ingest()[3].cpu().numpy()
    for x, u in enumerate(nodes):
        idl = ids1n[u]
        if x % 100 == 0:                               # the similarities themselves on ten of the nodes
            opm = O.pairwise(D, wv, idl)
            tol = RTOL_F32 * (np.outer(dn[idl], dn[idl]) + np.abs(opm))
            assert (np.abs(pm[x] - opm) <= tol).all(), (u, np.max(np.abs(pm[x] - opm) / tol))
        cnt, order = O.detour_sort(idl, sc1n[u], pm[x])
        assert np.array_equal(count[x], cnt) and np.array_equal(sorted_ids[x], idl[order])
        se_pos, ke_pos, fl = O.ip_prune(D, int(u), R, R // 2, idl, order, pm[x], self_gpu[idl])
        assert np.array_equal(se[x][:len(se_pos)], idl[se_pos]) and (se[x][len(se_pos):] == -1).all()
        assert ke_count[x] == len(ke_pos) and np.array_equal(ke[x][:len(ke_pos)], idl[ke_pos])
        assert np.array_equal(flag[x], fl)
    _say("million: assemble")
    allp = ix.stage_prune(K, R, ids1, sc1, want_pm=False)
    graph = ix.stage_assemble(R, K, P, allp["se"], allp["sorted_ids"], spi1).cpu().numpy()
    ref = O.assemble(N, R, K, P, allp["se"].cpu().numpy(), allp["sorted_ids"].cpu().numpy(), spi1.cpu().numpy(), node_ids=nodes)
    assert np.array_equal(graph[nodes], ref)
    assert np.array_equal(ix.stage_entry_points(64).cpu().numpy(), O.entry_points(self_gpu, 64))
