"""Helpers shared by the GPU parity tests: tolerances derived from the
arithmetic, and comparison of ranked lists that tolerates only near-ties."""
import numpy as np

RTOL_F32 = 1e-5     # fp32 storage, fp32 accumulation
RTOL_BF16 = 1e-3    # bf16 dense storage (both sides read the same bf16 values)


def row_norms(v):
    return np.linalg.norm(np.asarray(v.dense, np.float64), axis=1)


def score_tol(o4, w, qn, dn, rtol):
    """Admissible |gpu - oracle| for out4 = (sim_d, sim_s, sim_f, fused).

    A length-m fp32 dot product differs from the exact one by at most about
    m*eps*sum|a_i b_i|; sum|a_i b_i| <= |a||b| for the dense part and equals the
    value itself for the sparse parts (non-negative entries).  So the bound is
    relative to  |w_d||q_d||d_d| + |w_s| sim_s + |w_f| sim_f,  not to the
    possibly cancelling sum.  o4: [..., 4] oracle values; w: [..., 3];
    qn, dn broadcastable norms of the dense parts."""
    o4 = np.asarray(o4, np.float64)
    w = np.abs(np.asarray(w, np.float64))
    dense_mag = qn * dn
    tol = np.empty_like(o4)
    tol[..., 0] = rtol * dense_mag
    tol[..., 1] = rtol * np.abs(o4[..., 1])
    tol[..., 2] = rtol * np.abs(o4[..., 2])
    tol[..., 3] = rtol * (w[..., 0] * dense_mag + w[..., 1] * np.abs(o4[..., 1]) + w[..., 2] * np.abs(o4[..., 2]))
    return tol + 1e-30


def assert_scores_close(g4, o4, tol, what=""):
    g4 = np.asarray(g4, np.float64); o4 = np.asarray(o4, np.float64)
    fin = np.isfinite(o4)
    assert np.array_equal(fin, np.isfinite(g4)), f"{what}: finite pattern differs"
    assert np.array_equal(g4[~fin], o4[~fin]), f"{what}: infinities differ"
    err = np.abs(np.where(fin, g4, 0.0) - np.where(fin, o4, 0.0))[fin]
    bad = err > tol[fin]
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} beyond tolerance, worst ratio {np.max(err / tol[fin]):.3g}"


def assert_ranked_equiv(g_ids, g_sc, o_ids, o_sc, tol_of, oracle_score, what=""):
    """Two ranked lists (score desc, id asc) of the same candidates computed in
    different precision.  Wherever they differ, the difference must be a
    near-tie: the scores at every rank agree within tolerance, and an id the
    oracle does not list must score (in the oracle) within tolerance of the
    oracle's last listed score.  Returns the number of rows with any mismatch.

    tol_of(row, score) -> admissible error; oracle_score(row, id) -> float."""
    g_ids = np.asarray(g_ids); o_ids = np.asarray(o_ids)
    g_sc = np.asarray(g_sc, np.float64); o_sc = np.asarray(o_sc, np.float64)
    assert g_ids.shape == o_ids.shape, what
    rows = np.nonzero((g_ids != o_ids).any(axis=1))[0]
    for r in rows:
        assert np.array_equal(g_ids[r] < 0, o_ids[r] < 0), f"{what}: row {r} length differs"
        m = o_ids[r] >= 0
        tol = np.array([tol_of(r, s) for s in o_sc[r][m]])
        assert (np.abs(g_sc[r][m] - o_sc[r][m]) <= 2 * tol).all(), f"{what}: row {r} scores differ"
        oset = set(o_ids[r][m].tolist())
        last = o_sc[r][m][-1]
        for pos in np.nonzero(g_ids[r] != o_ids[r])[0]:
            gid = int(g_ids[r][pos])
            if gid in oset:
                # same members, swapped order: their oracle scores must be a near-tie
                opos = int(np.nonzero(o_ids[r] == gid)[0][0])
                assert abs(o_sc[r][opos] - o_sc[r][pos]) <= 2 * tol_of(r, o_sc[r][pos]), f"{what}: row {r} order"
            else:
                s = oracle_score(r, gid)
                assert abs(s - last) <= 2 * tol_of(r, last), f"{what}: row {r} has id {gid} that is no near-tie"
    return len(rows)
