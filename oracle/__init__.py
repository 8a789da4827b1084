"""ctypes front end of the CPU oracle (``allanpoe_oracle.c``).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
CPU-baseline leg import this; the product path never does.  Argument
marshalling and the chaining of the stage functions into a whole build live
here; every number is computed by the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from types import SimpleNamespace
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "allanpoe_oracle.c")
_LIB = os.path.join(_HERE, "liballanpoe_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _VS(C.Structure):
    _fields_ = [("n", C.c_int64), ("dim", C.c_int32), ("dense", C.c_void_p),
                ("sp_indptr", C.c_void_p), ("sp_idx", C.c_void_p), ("sp_val", C.c_void_p),
                ("tx_indptr", C.c_void_p), ("tx_idx", C.c_void_p), ("tx_val", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_sparse_ip.restype = C.c_double
        _lib.orc_search.restype = C.c_int64
        _lib.orc_search_kw.restype = C.c_int64
        _lib.orc_search_kg.restype = C.c_int64
        _lib.orc_bm25_encode.restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


class VS:
    """Holds contiguous arrays of a vector set and the C struct that points at them."""

    def __init__(self, v, tx_val: Optional[np.ndarray] = None):
        self.n = int(v.n)
        self.dim = int(v.dim)
        self.dense = _c(v.dense, np.float32)
        self.sp_indptr = _c(v.sp_indptr, np.int64)
        self.sp_idx = _c(v.sp_idx, np.int32)
        self.sp_val = _c(v.sp_val, np.float32)
        self.tx_indptr = _c(v.tx_indptr, np.int64)
        self.tx_idx = _c(v.tx_idx, np.int32)
        self.tx_val = _c(v.tx_val if tx_val is None else tx_val, np.float32)
        self.s = _VS(self.n, self.dim, self.dense.ctypes.data, self.sp_indptr.ctypes.data,
                     self.sp_idx.ctypes.data, self.sp_val.ctypes.data, self.tx_indptr.ctypes.data,
                     self.tx_idx.ctypes.data, self.tx_val.ctypes.data)

    @property
    def ref(self):
        return C.byref(self.s)


# ---------------------------------------------------------------- S0
def bm25_encode(n, vocab, indptr, idx, tf, k1=1.2, b=0.75):
    indptr = _c(indptr, np.int64); idx = _c(idx, np.int32); tf = _c(tf, np.float32)
    w = np.empty(len(idx), np.float32)
    df = np.empty(vocab, np.int32)
    avg = C.c_double(0)
    rc = lib().orc_bm25_encode(C.c_int64(n), C.c_int32(vocab), _p(indptr), _p(idx), _p(tf),
                               C.c_double(k1), C.c_double(b), _p(w), _p(df), C.byref(avg))
    if rc != 0:
        raise ValueError("term id out of range")
    return w, df, avg.value


def encode_docs(docs, k1=1.2, b=0.75) -> VS:
    """Document vector set whose lexical values are BM25 weights (S0 applied)."""
    w, _, _ = bm25_encode(docs.n, docs.tx_vocab, docs.tx_indptr, docs.tx_idx, docs.tx_val, k1, b)
    return VS(docs, tx_val=w)


# ---------------------------------------------------------------- S1
def sparse_ip(ia, va, ib, vb) -> float:
    ia = _c(ia, np.int32); va = _c(va, np.float32); ib = _c(ib, np.int32); vb = _c(vb, np.float32)
    return lib().orc_sparse_ip(_p(ia), _p(va), C.c_int64(len(ia)), _p(ib), _p(vb), C.c_int64(len(ib)))


def _w_rows(w, na):
    w = np.asarray(w, np.float32)
    if w.ndim == 1:
        w = np.broadcast_to(w, (na, 3))
    return _c(w, np.float32)


def hybrid_block(A: VS, a_ids, B: VS, cand, w):
    """out[na, c, 4] = (sim_d, sim_s, sim_f, fused) for each a and each of its candidates."""
    a_ids = _c(a_ids, np.int64)
    cand = _c(cand, np.int32).reshape(len(a_ids), -1)
    na, c = cand.shape
    w = _w_rows(w, na)
    out = np.empty((na, c, 4), np.float32)
    lib().orc_hybrid_block(A.ref, C.c_int64(na), _p(a_ids), B.ref, C.c_int64(c), _p(cand), _p(w), _p(out))
    return out


def bruteforce_topk(Q: VS, q_ids, D: VS, w, k, skip_same=False):
    q_ids = _c(q_ids, np.int64)
    nq = len(q_ids)
    w = _w_rows(w, nq)
    ids = np.empty((nq, k), np.int32)
    sc = np.empty((nq, k), np.float32)
    lib().orc_bruteforce_topk(Q.ref, C.c_int64(nq), _p(q_ids), D.ref, _p(w), C.c_int32(k),
                              C.c_int32(1 if skip_same else 0), _p(ids), _p(sc))
    return ids, sc


def self_sim(D: VS, ids, w):
    ids = _c(ids, np.int64)
    w = _c(w, np.float32)
    out = np.empty(len(ids), np.float32)
    lib().orc_self_sim(D.ref, C.c_int64(len(ids)), _p(ids), _p(w), _p(out))
    return out


# ---------------------------------------------------------------- S2..S6
def seed_knn(D: VS, node_ids, K):
    node_ids = _c(node_ids, np.int64)
    ids = np.empty((len(node_ids), K), np.int32)
    sc = np.empty((len(node_ids), K), np.float32)
    lib().orc_seed_knn(D.ref, C.c_int64(len(node_ids)), _p(node_ids), C.c_int32(K), _p(ids), _p(sc))
    return ids, sc


def empty_sp(N, P):
    return np.full((3, N, P), -1, np.int32), np.full((3, N, P), -np.inf, np.float32)


def refine_round(D: VS, w, K, S, P, knn_ids, sp_ids, sp_sc, node_ids=None):
    N = D.n
    node_ids = _c(np.arange(N) if node_ids is None else node_ids, np.int64)
    nn = len(node_ids)
    knn_ids = _c(knn_ids, np.int32); sp_ids = _c(sp_ids, np.int32); sp_sc = _c(sp_sc, np.float32)
    assert knn_ids.shape == (N, K) and sp_ids.shape == (3, N, P)
    w = _c(w, np.float32)
    o_ids = np.empty((nn, K), np.int32); o_sc = np.empty((nn, K), np.float32)
    o_spi = np.empty((3, nn, P), np.int32); o_sps = np.empty((3, nn, P), np.float32)
    lib().orc_refine_round(D.ref, _p(w), C.c_int32(K), C.c_int32(S), C.c_int32(P), _p(knn_ids),
                           _p(sp_ids), _p(sp_sc), C.c_int64(nn), _p(node_ids), _p(o_ids), _p(o_sc),
                           _p(o_spi), _p(o_sps))
    return o_ids, o_sc, o_spi, o_sps


def pairwise(D: VS, w, ids):
    ids = _c(ids, np.int32)
    K = len(ids)
    w = _c(w, np.float32)
    Pm = np.empty((K, K), np.float32)
    lib().orc_pairwise(D.ref, _p(w), C.c_int32(K), _p(ids), _p(Pm))
    return Pm


def detour_sort(ids, simA, Pm):
    ids = _c(ids, np.int32); simA = _c(simA, np.float32); Pm = _c(Pm, np.float32)
    K = len(ids)
    cnt = np.empty(K, np.int32); order = np.empty(K, np.int32)
    lib().orc_detour_sort(C.c_int32(K), _p(ids), _p(simA), _p(Pm), _p(cnt), _p(order))
    return cnt, order


PRUNE_JOINT, PRUNE_RNG_ONLY, PRUNE_IP_ONLY = 0, 1, 2


def similarity_order(ids):
    """The walk order of the IP-only ablation: the list as it is ranked (holes last)."""
    ids = np.asarray(ids)
    return np.concatenate([np.nonzero(ids >= 0)[0], np.nonzero(ids < 0)[0]]).astype(np.int32)


def ip_prune(D: VS, A, R, ke_cap, ids, order, Pm, self_s, use_ip=True):
    ids = _c(ids, np.int32); order = _c(order, np.int32); Pm = _c(Pm, np.float32)
    self_s = _c(self_s, np.float32)
    K = len(ids)
    se = np.full(R, -1, np.int32); ke = np.full(max(ke_cap, 1), -1, np.int32)
    nse = C.c_int32(0); nke = C.c_int32(0)
    flag = np.zeros(K, np.int32)
    lib().orc_ip_prune(D.ref, C.c_int64(A), C.c_int32(K), C.c_int32(R), C.c_int32(ke_cap), _p(ids),
                       _p(order), _p(Pm), _p(self_s), C.c_int32(int(use_ip)), _p(se), C.byref(nse), _p(ke),
                       C.byref(nke), _p(flag))
    return se[:nse.value].copy(), ke[:nke.value].copy(), flag


def assemble(N, R, K, P, se, sorted_ids, sp_ids, node_ids=None):
    se = _c(se, np.int32); sorted_ids = _c(sorted_ids, np.int32); sp_ids = _c(sp_ids, np.int32)
    assert se.shape == (N, R) and sorted_ids.shape == (N, K) and sp_ids.shape == (3, N, P)
    node_ids = _c(np.arange(N) if node_ids is None else node_ids, np.int64)
    out = np.empty((len(node_ids), R), np.int32)
    lib().orc_assemble(C.c_int64(N), C.c_int32(R), C.c_int32(K), C.c_int32(P), _p(se), _p(sorted_ids),
                       _p(sp_ids), C.c_int64(len(node_ids)), _p(node_ids), _p(out))
    return out


def entry_points(self_s, E):
    self_s = _c(self_s, np.float32)
    out = np.empty(E, np.int32)
    lib().orc_entry_points(C.c_int64(len(self_s)), _p(self_s), C.c_int32(E), _p(out))
    return out


def prune_node(D: VS, u, w, R, ke_cap, ids, scores, self_all=None, Pm=None, mode=PRUNE_JOINT):
    """S4 + S5 for one node from its K-list (ids, scores sorted by rank).
    Returns a namespace with Pm, count, order, sorted ids, SE ids, KE ids, flags.
    mode: the joint strategy, or one of its two ablations."""
    ids = _c(ids, np.int32)
    if Pm is None:
        Pm = pairwise(D, w, ids)
    cnt, order = detour_sort(ids, scores, Pm)
    if mode == PRUNE_IP_ONLY:
        order = similarity_order(ids)
    if self_all is None:
        self_s = np.where(ids >= 0, np.diag(Pm), -np.inf).astype(np.float32)
    else:
        self_s = np.where(ids >= 0, np.asarray(self_all)[np.maximum(ids, 0)], -np.inf).astype(np.float32)
    se_pos, ke_pos, flag = ip_prune(D, u, R, ke_cap, ids, order, Pm, self_s, use_ip=mode != PRUNE_RNG_ONLY)
    return SimpleNamespace(Pm=Pm, count=cnt, order=order, sorted=ids[order], se=ids[se_pos],
                           ke=ids[ke_pos], flag=flag, se_pos=se_pos, ke_pos=ke_pos)


def default_params(R: int, **kw):
    p = dict(degree=R, knn_k=2 * R, nd_rounds=3, nd_sample=32, n_entry=64, sp_len=-(-R // 6),
             build_w=(1.0, 1.0, 1.0), bm25_k1=1.2, bm25_b=0.75, prune_mode=PRUNE_JOINT)
    p.update(kw)
    p["ke_cap"] = p["degree"] // 2
    return SimpleNamespace(**p)


def build_index(docs, params):
    """Whole construction (S0, S2..S6) by chaining the stage functions.  Returns
    a namespace with every intermediate, for stage-wise comparison."""
    D = encode_docs(docs, params.bm25_k1, params.bm25_b)
    N, R, K, P = D.n, params.degree, params.knn_k, params.sp_len
    w = np.asarray(params.build_w, np.float32)
    allv = np.arange(N, dtype=np.int64)
    self_s = self_sim(D, allv, w)
    ids, sc = seed_knn(D, allv, K)
    seed_ids = ids.copy()
    spi, sps = empty_sp(N, P)
    rounds = []
    for _ in range(params.nd_rounds):
        ids, sc, spi, sps = refine_round(D, w, K, params.nd_sample, P, ids, spi, sps)
        rounds.append((ids.copy(), sc.copy()))
    if params.nd_rounds == 0:
        # lists must carry fused scores for the pruning stage
        o = hybrid_block(D, allv, D, ids, w)
        sc = o[:, :, 3].copy()
    se = np.full((N, R), -1, np.int32)
    ke = np.full((N, max(params.ke_cap, 1)), -1, np.int32)
    ke_cnt = np.zeros(N, np.int32)
    sorted_ids = np.empty((N, K), np.int32)
    counts = np.empty((N, K), np.int32)
    for u in range(N):
        r = prune_node(D, u, w, R, params.ke_cap, ids[u], sc[u], self_all=self_s, mode=params.prune_mode)
        se[u, :len(r.se)] = r.se
        ke[u, :len(r.ke)] = r.ke
        ke_cnt[u] = len(r.ke)
        sorted_ids[u] = r.sorted
        counts[u] = r.count
    graph = assemble(N, R, K, P, se, sorted_ids, spi)
    entry = entry_points(self_s, params.n_entry)
    return SimpleNamespace(D=D, self_sim=self_s, seed_ids=seed_ids, knn_ids=ids, knn_scores=sc,
                           sp_ids=spi, sp_scores=sps, rounds=rounds, se=se, ke=ke, ke_count=ke_cnt,
                           sorted_ids=sorted_ids, counts=counts, graph=graph, entry=entry, params=params)


# ---------------------------------------------------------------- S7..S9
def _deleted_bytes(deleted, n):
    if deleted is None:
        return None
    d = np.zeros(n, np.uint8)
    d[np.asarray(deleted, np.int64)] = 1
    return d


def search(D: VS, graph, entry, Q: VS, qi, w, k, L, max_iters=0, width=1, score_table=None,
           log=False, deleted=None):
    """deleted: ids of mark-deleted documents (searched through, left out of the answer)."""
    dl = _deleted_bytes(deleted, D.n)
    graph = _c(graph, np.int32)
    entry = _c(entry, np.int32)
    R = graph.shape[1]
    w = _c(w, np.float32)
    ids = np.empty(k, np.int32); sc = np.empty(k, np.float32)
    st = None if score_table is None else _c(score_table, np.float32)
    cap = D.n if log else 0
    vl = np.empty(max(cap, 1), np.int32)
    n = lib().orc_search(D.ref, _p(graph), C.c_int32(R), _p(entry), C.c_int32(len(entry)), Q.ref,
                         C.c_int64(qi), _p(w), C.c_int32(k), C.c_int32(L), C.c_int32(max_iters),
                         C.c_int32(width), _p(st), _p(dl), _p(ids), _p(sc), _p(vl) if log else None,
                         C.c_int64(cap))
    if log:
        return ids, sc, vl[:n].copy()
    return ids, sc, int(n)


def search_batch(D: VS, graph, entry, Q: VS, q_ids: Sequence[int], w, k, L, max_iters=0, width=1):
    q_ids = list(q_ids)
    w = _w_rows(w, len(q_ids))
    ids = np.empty((len(q_ids), k), np.int32); sc = np.empty((len(q_ids), k), np.float32)
    nv = np.empty(len(q_ids), np.int64)
    for x, qi in enumerate(q_ids):
        ids[x], sc[x], nv[x] = search(D, graph, entry, Q, qi, w[x], k, L, max_iters, width)
    return ids, sc, nv


def search_kw(D: VS, graph, kw_edges, kw_count, entry, Q: VS, qi, w, k, L, kw, kw_all=False, use_kw_edges=True,
              max_iters=0, width=1, score_table=None, log=False, deleted=None):
    """Keyword-constrained search (Section 4.2.2, Algorithm 2's keyword branches) for one query.
    kw: the required term ids (empty = unconstrained)."""
    graph = _c(graph, np.int32); kw_edges = _c(kw_edges, np.int32); kw_count = _c(kw_count, np.int32)
    entry = _c(entry, np.int32)
    kw = _c(np.asarray(kw, np.int32).reshape(-1), np.int32)
    dl = _deleted_bytes(deleted, D.n)     # kept alive across the call
    w = _c(w, np.float32)
    ids = np.empty(k, np.int32); sc = np.empty(k, np.float32)
    st = None if score_table is None else _c(score_table, np.float32)
    cap = D.n if log else 0
    vl = np.empty(max(cap, 1), np.int32)
    n = lib().orc_search_kw(D.ref, _p(graph), C.c_int32(graph.shape[1]), _p(kw_edges), C.c_int32(kw_edges.shape[1]),
                            _p(kw_count), _p(entry), C.c_int32(len(entry)), Q.ref, C.c_int64(qi), _p(w), C.c_int32(k),
                            C.c_int32(L), C.c_int32(max_iters), C.c_int32(width), _p(kw), C.c_int32(len(kw)),
                            C.c_int32(int(kw_all)), C.c_int32(int(use_kw_edges)), _p(st),
                            _p(dl), _p(ids), _p(sc), _p(vl) if log else None, C.c_int64(cap))
    if log:
        return ids, sc, vl[:n].copy()
    return ids, sc, int(n)


# ---------------------------------------------------------------- updates: insertion
def rows_of(D: VS, lo: int, hi: int) -> VS:
    """Documents lo..hi-1 of an encoded vector set as a vector set of their own (values unchanged)."""
    ns = SimpleNamespace(n=hi - lo, dim=D.dim, dense=D.dense[lo:hi],
                         sp_indptr=D.sp_indptr[lo:hi + 1] - D.sp_indptr[lo],
                         sp_idx=D.sp_idx[D.sp_indptr[lo]:D.sp_indptr[hi]], sp_val=D.sp_val[D.sp_indptr[lo]:D.sp_indptr[hi]],
                         tx_indptr=D.tx_indptr[lo:hi + 1] - D.tx_indptr[lo],
                         tx_idx=D.tx_idx[D.tx_indptr[lo]:D.tx_indptr[hi]], tx_val=D.tx_val[D.tx_indptr[lo]:D.tx_indptr[hi]])
    return VS(ns)


def merge_ranked(ids_a, sc_a, ids_b, sc_b, K):
    """Best K of two ranked lists over disjoint ids, by (score descending, id ascending); -1 / -inf padded."""
    both = [(float(s), int(i)) for i, s in zip(ids_a, sc_a) if i >= 0] + [(float(s), int(i)) for i, s in zip(ids_b, sc_b) if i >= 0]
    both.sort(key=lambda t: (-t[0], t[1]))
    both = both[:K]
    ids = np.full(K, -1, np.int32); sc = np.full(K, -np.inf, np.float32)
    ids[:len(both)] = [t[1] for t in both]; sc[:len(both)] = [t[0] for t in both]
    return ids, sc


def insert_index(old, docs, beam=None):
    """Insertion of new documents (Section 4.1, updates of the hybrid index).  `docs` is the enlarged corpus: its
    first N0 documents are those of the index `old` (a build_index or insert_index result), the rest are new.
      0. S0 over the enlarged corpus (corpus statistics, hence all lexical weights, are those of the new corpus).
      1. Candidate set one: the K best old documents for each new one, found by the search of Algorithm 2 on the
         old semantic edges from the old entry points, with the new document as the query, the construction
         weights and a pool of `beam` (default 2K).
      2. Candidate set two: K-lists among the new documents alone (seed + the usual refinement rounds).
      3. The K-list of a new document = the best K of both sets; it is scored once more without 2-hop exploration
         so that its per-path lists = the best P per path among set two's per-path lists and the list's members.
      4. S4/S5 for the new documents only; S6 over all documents (old documents gain reverse neighbours among the
         new ones); entry points from all self-similarities.
    Returns a namespace like build_index's, plus the intermediates of steps 1-3 for the new documents."""
    params = old.params
    D = encode_docs(docs, params.bm25_k1, params.bm25_b)
    N0, N1 = old.graph.shape[0], D.n
    M = N1 - N0
    assert M >= 1
    R, K, P = params.degree, params.knn_k, params.sp_len
    w = np.asarray(params.build_w, np.float32)
    L = int(beam) if beam else 2 * K
    self_s = self_sim(D, np.arange(N1, dtype=np.int64), w)
    # 1: the old graph, padded with edge-less rows for the new documents (they are never reached)
    g_old = np.vstack([old.graph, np.full((M, R), -1, np.int32)])
    c1_ids = np.empty((M, K), np.int32); c1_sc = np.empty((M, K), np.float32)
    for j in range(M):
        c1_ids[j], c1_sc[j], _ = search(D, g_old, old.entry, D, N0 + j, w, K, max(L, K))
    # 2: the new documents among themselves
    Dn = rows_of(D, N0, N1)
    c2_ids, c2_sc = seed_knn(Dn, np.arange(M, dtype=np.int64), K)
    spi2, sps2 = empty_sp(M, P)
    for _ in range(params.nd_rounds):
        c2_ids, c2_sc, spi2, sps2 = refine_round(Dn, w, K, params.nd_sample, P, c2_ids, spi2, sps2)
    if params.nd_rounds == 0:
        c2_sc = hybrid_block(Dn, np.arange(M), Dn, c2_ids, w)[:, :, 3].copy()
    shift = lambda a: np.where(a >= 0, a + N0, -1).astype(np.int32)
    c2_ids, spi2 = shift(c2_ids), shift(spi2)
    # 3: merge, then per-path lists
    knn = np.full((N1, K), -1, np.int32); knn_sc = np.full((N1, K), -np.inf, np.float32)
    for j in range(M):
        knn[N0 + j], knn_sc[N0 + j] = merge_ranked(c1_ids[j], c1_sc[j], c2_ids[j], c2_sc[j], K)
    merged_ids = knn[N0:].copy(); merged_sc = knn_sc[N0:].copy()
    spi = np.full((3, N1, P), -1, np.int32); sps = np.full((3, N1, P), -np.inf, np.float32)
    spi[:, :N0], sps[:, :N0] = old.sp_ids, old.sp_scores
    spi[:, N0:], sps[:, N0:] = spi2, sps2
    newv = np.arange(N0, N1, dtype=np.int64)
    f_ids, f_sc, f_spi, f_sps = refine_round(D, w, K, 0, P, knn, spi, sps, node_ids=newv)
    knn[N0:], knn_sc[N0:] = f_ids, f_sc
    spi[:, N0:], sps[:, N0:] = f_spi, f_sps
    # 4
    se = np.vstack([old.se, np.full((M, R), -1, np.int32)])
    ke = np.vstack([old.ke, np.full((M, old.ke.shape[1]), -1, np.int32)])
    ke_cnt = np.concatenate([old.ke_count, np.zeros(M, np.int32)])
    sorted_ids = np.vstack([old.sorted_ids, np.full((M, K), -1, np.int32)])
    for u in range(N0, N1):
        r = prune_node(D, u, w, R, params.ke_cap, knn[u], knn_sc[u], self_all=self_s, mode=params.prune_mode)
        se[u, :len(r.se)] = r.se
        ke[u, :len(r.ke)] = r.ke
        ke_cnt[u] = len(r.ke)
        sorted_ids[u] = r.sorted
    graph = assemble(N1, R, K, P, se, sorted_ids, spi)
    entry = entry_points(self_s, params.n_entry)
    return SimpleNamespace(D=D, self_sim=self_s, knn_ids=knn, knn_scores=knn_sc, sp_ids=spi, sp_scores=sps, se=se, ke=ke,
                           ke_count=ke_cnt, sorted_ids=sorted_ids, graph=graph, entry=entry, params=params,
                           cand1_ids=c1_ids, cand1_scores=c1_sc, cand2_ids=c2_ids, cand2_scores=c2_sc,
                           cand2_sp_ids=spi2, cand2_sp_scores=sps2, merged_ids=merged_ids, merged_scores=merged_sc, n_old=N0)


# ---------------------------------------------------------------- logical edges (knowledge-graph augmentation)
def entity_nodes(n_ent, doc_ent_indptr, doc_ent):
    """The entity-to-document mapping (Section 3.4): CSR of the documents that mention each entity, ascending."""
    rows = [[] for _ in range(n_ent)]
    for x in range(len(doc_ent_indptr) - 1):
        for e in doc_ent[doc_ent_indptr[x]:doc_ent_indptr[x + 1]]:
            rows[int(e)].append(x)
    indptr = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int64)
    idx = np.array([x for r in rows for x in r], np.int32)
    return indptr, idx


def logical_edges(kgs, n, cap):
    """Logical edges of every document (Section 3.4; Algorithm 1's last step): triples (s, y, t) with s an entity
    of x, (s, t) a relation, t not an entity of x, y != x a document that mentions t; in ascending (s, t, y)
    order, the first `cap` of them.  Returns le [n, cap, 3] (-1 padded), le_count [n] and the entity-to-document CSR."""
    en_ip, en = entity_nodes(kgs.n_ent, kgs.doc_ent_indptr, kgs.doc_ent)
    le = np.full((n, cap, 3), -1, np.int32); cnt = np.zeros(n, np.int32)
    for x in range(n):
        mine = [int(e) for e in kgs.doc_ent[kgs.doc_ent_indptr[x]:kgs.doc_ent_indptr[x + 1]]]
        out = []
        for s in mine:
            for t in kgs.kg_idx[kgs.kg_indptr[s]:kgs.kg_indptr[s + 1]]:
                t = int(t)
                if t in mine:
                    continue
                for y in en[en_ip[t]:en_ip[t + 1]]:
                    if int(y) != x:
                        out.append((s, int(y), t))
        out = out[:cap]                      # generated in ascending (s, t, y)
        cnt[x] = len(out)
        if out:
            le[x, :len(out)] = out
    return le, cnt, en_ip, en


def search_kg(D: VS, graph, entry, Q: VS, qi, w, k, L, kgs, le, le_count, en_ip, en, q_ent, w_k, max_hops=2, max_iters=0,
              score_table=None, log=False, deleted=None):
    """Search with knowledge-graph augmentation for one query (Section 4.2.3); q_ent: the query's entities.
    deleted: ids of mark-deleted documents (Section 4.1, updates), left out of the answer."""
    graph = _c(graph, np.int32); entry = _c(entry, np.int32)
    w = _c(w, np.float32)
    de_ip = _c(kgs.doc_ent_indptr, np.int64); de = _c(kgs.doc_ent, np.int32)
    kg_ip = _c(kgs.kg_indptr, np.int64); kg = _c(kgs.kg_idx, np.int32)
    en_ip = _c(en_ip, np.int64); en = _c(en, np.int32)
    le = _c(le, np.int32); le_count = _c(le_count, np.int32)
    qe = _c(np.asarray(q_ent, np.int32).reshape(-1), np.int32)
    ids = np.empty(k, np.int32); sc = np.empty(k, np.float32)
    st = None if score_table is None else _c(score_table, np.float32)
    cap = D.n if log else 0
    vl = np.empty(max(cap, 1), np.int32); al = np.empty((max(cap, 1), 2), np.int32)
    dl = _deleted_bytes(deleted, D.n)
    n = lib().orc_search_kg(D.ref, _p(graph), C.c_int32(graph.shape[1]), _p(entry), C.c_int32(len(entry)), Q.ref,
                            C.c_int64(qi), _p(w), C.c_int32(k), C.c_int32(L), C.c_int32(max_iters), _p(de_ip), _p(de),
                            _p(kg_ip), _p(kg), _p(en_ip), _p(en), _p(le), C.c_int32(le.shape[1]), _p(le_count), _p(qe),
                            C.c_int32(len(qe)), C.c_float(w_k), C.c_int32(max_hops), _p(st), _p(dl), _p(ids), _p(sc),
                            _p(vl) if log else None, _p(al) if log else None, C.c_int64(cap))
    if log:
        return ids, sc, vl[:n].copy(), al[:n].copy()
    return ids, sc, int(n)
