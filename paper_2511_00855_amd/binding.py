"""Thin ctypes binding of ``liballanpoe.so`` (see ``include/allanpoe.h``).

Argument marshalling only: tensors are allocated with torch (device memory and
the current stream are all torch is used for), their addresses are handed to
the C ABI, and every step of the path runs in the library's HIP kernels.
There is no fallback: if the library is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ALLANPOE_LIB") or os.path.join(_HERE, "liballanpoe.so")

AP_F32, AP_BF16 = 0, 1


class ApError(RuntimeError):
    pass


class _Corpus(C.Structure):
    _fields_ = [("n", C.c_int64), ("dim", C.c_int32), ("dense_dtype", C.c_int32), ("dense", C.c_void_p),
                ("sp_indptr", C.c_void_p), ("sp_idx", C.c_void_p), ("sp_val", C.c_void_p), ("sp_vocab", C.c_int32),
                ("tx_indptr", C.c_void_p), ("tx_idx", C.c_void_p), ("tx_tf", C.c_void_p), ("tx_vocab", C.c_int32)]


class _BuildParams(C.Structure):
    _fields_ = [("degree", C.c_int32), ("knn_k", C.c_int32), ("nd_rounds", C.c_int32), ("nd_sample", C.c_int32),
                ("n_entry", C.c_int32), ("sp_len", C.c_int32), ("bm25_k1", C.c_float), ("bm25_b", C.c_float),
                ("build_w", C.c_float * 3), ("prune_mode", C.c_int32), ("seed", C.c_uint64)]


class _Queries(C.Structure):
    _fields_ = [("nq", C.c_int32), ("dense", C.c_void_p), ("sp_indptr", C.c_void_p), ("sp_idx", C.c_void_p),
                ("sp_val", C.c_void_p), ("tx_indptr", C.c_void_p), ("tx_idx", C.c_void_p), ("tx_cnt", C.c_void_p)]


class _InsertTrace(C.Structure):
    _fields_ = [(f, C.c_void_p) for f in ("cand1_ids", "cand1_sc", "cand2_ids", "cand2_sc", "cand2_sp_ids", "cand2_sp_sc",
                                          "merged_ids", "merged_sc", "knn_ids", "knn_sc")]


class _SearchParams(C.Structure):
    _fields_ = [("k", C.c_int32), ("beam", C.c_int32), ("max_iters", C.c_int32), ("search_width", C.c_int32)]


_lib = None


def lib():
    """Loads the built library; raises if it is not there (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ApError(f"{LIB_PATH} is missing: run __graft_entry__.build() (hipcc) first")
        _lib = C.CDLL(LIB_PATH)
        _lib.ap_last_error.restype = C.c_char_p
        _lib.ap_free_index.restype = None
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise ApError(f"{what} failed ({rc}): {lib().ap_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(a, dtype, device):
    if isinstance(a, torch.Tensor):
        return a.to(device=device, dtype=dtype).contiguous()
    return torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dtype).contiguous()


def _ids(a, device):
    """Optional int32 id list on the device."""
    if a is None:
        return None
    return _dev(np.asarray(a, dtype=np.int32) if not isinstance(a, torch.Tensor) else a, torch.int32, device)


def calibration_copy(dst: torch.Tensor, src: torch.Tensor):
    """Plain copy kernel of known size (see ap_calibration_copy)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    with torch.cuda.device(src.device):
        _check(lib().ap_calibration_copy(_ptr(dst), _ptr(src), C.c_size_t(nbytes), _stream()), "ap_calibration_copy")


def debug_set(name: str, value: int):
    """A debug setting of the library (see ap_debug_set); 0 restores the library's own choice."""
    _check(lib().ap_debug_set(name.encode(), C.c_int64(int(value))), "ap_debug_set")


DEBUG_NAMES = ("seed_sample_cols", "seed_buffer_cap", "seed_tau_ulps", "max_launch_threads", "search_workspace_bytes",
               "search_visited_global", "search_query_lists", "seed_one_sided")


def debug_reset():
    for name in DEBUG_NAMES:
        debug_set(name, 0)


class DeviceVecs:
    """Device copies of a vector set (documents or queries)."""

    def __init__(self, v, device="cuda:0", bf16: bool = False):
        self.device = torch.device(device)
        self.n, self.dim = int(v.n), int(v.dim)
        if bf16:
            if getattr(v, "dense_bf16", None) is None:
                raise ValueError("vector set has no bf16 dense part")
            self.dense = _dev(v.dense_bf16.view(np.int16), torch.int16, self.device)
            self.dtype = AP_BF16
        else:
            self.dense = _dev(v.dense, torch.float32, self.device)
            self.dtype = AP_F32
        self.sp_indptr = _dev(v.sp_indptr, torch.int64, self.device)
        self.sp_idx = _dev(v.sp_idx, torch.int32, self.device)
        self.sp_val = _dev(v.sp_val, torch.float32, self.device)
        self.tx_indptr = _dev(v.tx_indptr, torch.int64, self.device)
        self.tx_idx = _dev(v.tx_idx, torch.int32, self.device)
        self.tx_val = _dev(v.tx_val, torch.float32, self.device)
        self.sp_vocab = int(getattr(v, "sp_vocab", 0) or (int(self.sp_idx.max()) + 1 if len(self.sp_idx) else 1))
        self.tx_vocab = int(getattr(v, "tx_vocab", 0) or (int(self.tx_idx.max()) + 1 if len(self.tx_idx) else 1))

    def corpus_struct(self) -> _Corpus:
        return _Corpus(self.n, self.dim, self.dtype, self.dense.data_ptr(), self.sp_indptr.data_ptr(),
                       self.sp_idx.data_ptr(), self.sp_val.data_ptr(), self.sp_vocab, self.tx_indptr.data_ptr(),
                       self.tx_idx.data_ptr(), self.tx_val.data_ptr(), self.tx_vocab)

    def queries_struct(self) -> _Queries:
        if self.dtype != AP_F32:
            raise ValueError("queries are f32")
        return _Queries(self.n, self.dense.data_ptr(), self.sp_indptr.data_ptr(), self.sp_idx.data_ptr(),
                        self.sp_val.data_ptr(), self.tx_indptr.data_ptr(), self.tx_idx.data_ptr(),
                        self.tx_val.data_ptr())


def build_params(degree: int, knn_k: Optional[int] = None, nd_rounds: int = 3, nd_sample: int = 32,
                 n_entry: int = 64, sp_len: int = 0, bm25_k1: float = 1.2, bm25_b: float = 0.75,
                 build_w: Sequence[float] = (1.0, 1.0, 1.0), seed: int = 0, prune_mode: int = 0) -> _BuildParams:
    """prune_mode: 0 joint RNG-IP pruning, 1 RNG only, 2 IP only (see ap_build_params)."""
    return _BuildParams(degree, knn_k if knn_k is not None else 2 * degree, nd_rounds, nd_sample, n_entry, sp_len,
                        bm25_k1, bm25_b, (C.c_float * 3)(*build_w), prune_mode, seed)


class Index:
    """Owner of an ``ap_index`` handle.  Keeps the corpus tensors alive (the
    library borrows them)."""

    def __init__(self, handle, docs: DeviceVecs, params: _BuildParams):
        self._h = handle
        self.docs = docs
        self.params = params
        self.device = docs.device

    # -- constructors -------------------------------------------------------
    @classmethod
    def _create(cls, fn_name, docs: DeviceVecs, params: _BuildParams, *extra):
        h = C.c_void_p()
        cs = docs.corpus_struct()
        with torch.cuda.device(docs.device):
            rc = getattr(lib(), fn_name)(C.byref(cs), C.byref(params), *extra, _stream(), C.byref(h))
        _check(rc, fn_name)
        return cls(h, docs, params)

    @classmethod
    def build(cls, docs: DeviceVecs, params: _BuildParams) -> "Index":
        return cls._create("ap_build_index", docs, params)

    @classmethod
    def ingest(cls, docs: DeviceVecs, params: _BuildParams) -> "Index":
        return cls._create("ap_ingest", docs, params)

    @classmethod
    def import_graph(cls, docs: DeviceVecs, params: _BuildParams, semantic, entry, keyword=None, kw_count=None) -> "Index":
        dev = docs.device
        sem = _dev(semantic, torch.int32, dev)
        ent = _dev(entry, torch.int32, dev)
        assert sem.shape == (docs.n, params.degree) and ent.numel() == params.n_entry
        kw = None if keyword is None else _dev(keyword, torch.int32, dev)
        kc = None if kw_count is None else _dev(kw_count, torch.int32, dev)
        return cls._create("ap_import_graph", docs, params, _ptr(sem), _ptr(kw), _ptr(kc), _ptr(ent))

    def close(self):
        if self._h is not None and self._h.value:
            torch.cuda.synchronize(self.device)
            lib().ap_free_index(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the three calls -----------------------------------------------------
    def set_weights(self, w: Sequence[float]):
        _check(lib().ap_set_weights(self._h, (C.c_float * 3)(*w)), "ap_set_weights")

    def search_batch(self, queries: DeviceVecs, k: int, beam: int, per_query_w=None, max_iters: int = 0,
                     search_width: int = 1, out=None):
        nq = queries.n
        ids, sc = out if out is not None else (torch.empty((nq, k), dtype=torch.int32, device=self.device),
                                               torch.empty((nq, k), dtype=torch.float32, device=self.device))
        w = None if per_query_w is None else _dev(per_query_w, torch.float32, self.device)
        if w is not None:
            assert w.shape == (nq, 3)
        qs = queries.queries_struct()
        sp = _SearchParams(k, beam, max_iters, search_width)
        with torch.cuda.device(self.device):
            rc = lib().ap_search_batch(self._h, C.byref(qs), _ptr(w), C.byref(sp), _ptr(ids), _ptr(sc), _stream())
        _check(rc, "ap_search_batch")
        return ids, sc

    def search_batch_noalloc(self, queries: DeviceVecs, k: int, beam: int, per_query_w, out, max_iters: int = 0,
                             search_width: int = 1):
        """ap_search_batch_noalloc: the caller brings every buffer (per_query_w may be None); nothing is allocated here."""
        ids, sc = out
        qs = queries.queries_struct()
        sp = _SearchParams(k, beam, max_iters, search_width)
        with torch.cuda.device(self.device):
            rc = lib().ap_search_batch_noalloc(self._h, C.byref(qs), _ptr(per_query_w), C.byref(sp), _ptr(ids), _ptr(sc), _stream())
        _check(rc, "ap_search_batch_noalloc")
        return ids, sc

    def insert(self, enlarged: DeviceVecs, beam: int = 0, trace: bool = False):
        """A new index over `enlarged` (this index's documents first, unchanged, then the new ones); see
        ap_insert_documents.  With trace=True also returns the intermediates of the new documents."""
        n0, n1 = self.docs.n, enlarged.n
        m, K, P = n1 - n0, self.params.knn_k, self.params.sp_len or -(-self.params.degree // 6)
        dev = self.device
        tr = None
        bufs = {}
        if trace:
            def mk(shape, dt):
                return torch.empty(shape, dtype=dt, device=dev)
            bufs = dict(cand1_ids=mk((m, K), torch.int32), cand1_sc=mk((m, K), torch.float32),
                        cand2_ids=mk((m, K), torch.int32), cand2_sc=mk((m, K), torch.float32),
                        cand2_sp_ids=mk((3, m, P), torch.int32), cand2_sp_sc=mk((3, m, P), torch.float32),
                        merged_ids=mk((m, K), torch.int32), merged_sc=mk((m, K), torch.float32),
                        knn_ids=mk((m, K), torch.int32), knn_sc=mk((m, K), torch.float32))
            tr = _InsertTrace(*[_ptr(bufs[f]) for f, _ in _InsertTrace._fields_])
        h = C.c_void_p()
        cs = enlarged.corpus_struct()
        with torch.cuda.device(dev):
            rc = lib().ap_insert_documents(self._h, C.byref(cs), C.c_int32(beam), C.byref(tr) if tr is not None else None,
                                           _stream(), C.byref(h))
        _check(rc, "ap_insert_documents")
        ix = Index(h, enlarged, self.params)
        return (ix, bufs) if trace else ix

    def export_build_state(self):
        n, R, K = self.docs.n, self.params.degree, self.params.knn_k
        P = self.params.sp_len or -(-R // 6)
        dev = self.device
        se = torch.empty((n, R), dtype=torch.int32, device=dev)
        srt = torch.empty((n, K), dtype=torch.int32, device=dev)
        spi = torch.empty((3, n, P), dtype=torch.int32, device=dev)
        sps = torch.empty((3, n, P), dtype=torch.float32, device=dev)
        with torch.cuda.device(dev):
            _check(lib().ap_export_build_state(self._h, _ptr(se), _ptr(srt), _ptr(spi), _ptr(sps), _stream()), "ap_export_build_state")
        return se, srt, spi, sps

    def set_knowledge_graph(self, kgs, le_cap: int = 32):
        """kgs: namespace with n_ent, doc_ent_indptr, doc_ent, kg_indptr, kg_idx (see ap_set_knowledge_graph)."""
        dev = self.device
        self._kg = (_dev(kgs.doc_ent_indptr, torch.int64, dev), _dev(kgs.doc_ent, torch.int32, dev),
                    _dev(kgs.kg_indptr, torch.int64, dev), _dev(kgs.kg_idx, torch.int32, dev))   # kept alive: the index borrows them
        self._kg_dims = (int(kgs.n_ent), int(le_cap), int(len(kgs.doc_ent)))
        with torch.cuda.device(dev):
            _check(lib().ap_set_knowledge_graph(self._h, C.c_int32(int(kgs.n_ent)), *[_ptr(t) for t in self._kg],
                                                C.c_int32(le_cap), _stream()), "ap_set_knowledge_graph")

    def export_logical_edges(self):
        n_ent, cap, total = self._kg_dims
        dev = self.device
        le = torch.empty((self.docs.n, cap, 3), dtype=torch.int32, device=dev)
        cnt = torch.empty(self.docs.n, dtype=torch.int32, device=dev)
        en_ip = torch.empty(n_ent + 1, dtype=torch.int64, device=dev)
        en = torch.empty(max(total, 1), dtype=torch.int32, device=dev)
        with torch.cuda.device(dev):
            _check(lib().ap_export_logical_edges(self._h, _ptr(le), _ptr(cnt), _ptr(en_ip), _ptr(en), _stream()),
                   "ap_export_logical_edges")
        return le, cnt, en_ip, en[:total]

    def search_batch_entities(self, queries: DeviceVecs, k: int, beam: int, q_ent, w_k: float, max_hops: int = 2,
                              per_query_w=None, max_iters: int = 0):
        nq = queries.n
        qe = _dev(q_ent, torch.int32, self.device)
        assert qe.dim() == 2 and qe.shape[0] == nq
        ids = torch.empty((nq, k), dtype=torch.int32, device=self.device)
        sc = torch.empty((nq, k), dtype=torch.float32, device=self.device)
        w = None if per_query_w is None else _dev(per_query_w, torch.float32, self.device)
        qs = queries.queries_struct()
        sp = _SearchParams(k, beam, max_iters, 1)
        with torch.cuda.device(self.device):
            rc = lib().ap_search_batch_entities(self._h, C.byref(qs), _ptr(w), C.byref(sp), _ptr(qe), C.c_int32(qe.shape[1]),
                                                C.c_float(w_k), C.c_int32(max_hops), _ptr(ids), _ptr(sc), _stream())
        _check(rc, "ap_search_batch_entities")
        return ids, sc

    def mark_deleted(self, ids, restore: bool = False):
        """Marks documents deleted (or restores them): searched through, left out of the answers."""
        t = _dev(ids, torch.int32, self.device).reshape(-1)
        with torch.cuda.device(self.device):
            _check(lib().ap_mark_deleted(self._h, _ptr(t), C.c_int64(t.numel()), C.c_int(int(restore)), _stream()),
                   "ap_mark_deleted")

    def search_batch_keywords(self, queries: DeviceVecs, k: int, beam: int, kw_terms, per_query_w=None,
                              kw_all: bool = False, use_kw_edges: bool = True, max_iters: int = 0,
                              search_width: int = 1):
        """kw_terms: nq x stride int32 required term ids, -1 = unused slot (see ap_search_batch_keywords)."""
        nq = queries.n
        kw = _dev(kw_terms, torch.int32, self.device)
        assert kw.dim() == 2 and kw.shape[0] == nq
        ids = torch.empty((nq, k), dtype=torch.int32, device=self.device)
        sc = torch.empty((nq, k), dtype=torch.float32, device=self.device)
        w = None if per_query_w is None else _dev(per_query_w, torch.float32, self.device)
        if w is not None:
            assert w.shape == (nq, 3)
        qs = queries.queries_struct()
        sp = _SearchParams(k, beam, max_iters, search_width)
        flags = (1 if kw_all else 0) | (0 if use_kw_edges else 2)
        with torch.cuda.device(self.device):
            rc = lib().ap_search_batch_keywords(self._h, C.byref(qs), _ptr(w), C.byref(sp), _ptr(kw), C.c_int32(kw.shape[1]),
                                                C.c_uint32(flags), _ptr(ids), _ptr(sc), _stream())
        _check(rc, "ap_search_batch_keywords")
        return ids, sc

    # -- measurement / test surface -------------------------------------------
    def export_ingest(self):
        dev = self.device
        tx_w = torch.empty(self.docs.tx_idx.numel(), dtype=torch.float32, device=dev)
        df = torch.empty(self.docs.tx_vocab, dtype=torch.int32, device=dev)
        avgdl = torch.empty(1, dtype=torch.float32, device=dev)
        self_sim = torch.empty(self.docs.n, dtype=torch.float32, device=dev)
        with torch.cuda.device(dev):
            _check(lib().ap_export_ingest(self._h, _ptr(tx_w), _ptr(df), _ptr(avgdl), _ptr(self_sim), _stream()),
                   "ap_export_ingest")
        return tx_w, df, avgdl, self_sim

    def hybrid_scores(self, queries: DeviceVecs, cand_ids, per_query_w=None):
        cand = _dev(cand_ids, torch.int32, self.device).reshape(queries.n, -1)
        c = cand.shape[1]
        out = torch.empty((queries.n, c, 4), dtype=torch.float32, device=self.device)
        w = None if per_query_w is None else _dev(per_query_w, torch.float32, self.device)
        qs = queries.queries_struct()
        with torch.cuda.device(self.device):
            _check(lib().ap_hybrid_scores(self._h, C.byref(qs), _ptr(cand), C.c_int32(c), _ptr(w), _ptr(out), _stream()),
                   "ap_hybrid_scores")
        return out

    def hybrid_scores_docs(self, a_ids, cand_ids, w3):
        a = _ids(a_ids, self.device)
        cand = _dev(cand_ids, torch.int32, self.device).reshape(a.numel(), -1)
        c = cand.shape[1]
        out = torch.empty((a.numel(), c, 4), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(lib().ap_hybrid_scores_docs(self._h, _ptr(a), C.c_int32(a.numel()), _ptr(cand), C.c_int32(c),
                                               (C.c_float * 3)(*w3), _ptr(out), _stream()), "ap_hybrid_scores_docs")
        return out

    def bruteforce_topk(self, queries: DeviceVecs, k: int, per_query_w=None):
        ids = torch.empty((queries.n, k), dtype=torch.int32, device=self.device)
        sc = torch.empty((queries.n, k), dtype=torch.float32, device=self.device)
        w = None if per_query_w is None else _dev(per_query_w, torch.float32, self.device)
        qs = queries.queries_struct()
        with torch.cuda.device(self.device):
            _check(lib().ap_bruteforce_topk(self._h, C.byref(qs), _ptr(w), C.c_int32(k), _ptr(ids), _ptr(sc), _stream()),
                   "ap_bruteforce_topk")
        return ids, sc

    def stage_seed_knn(self, K: int, node_ids=None):
        nodes = _ids(node_ids, self.device)
        nn = self.docs.n if nodes is None else nodes.numel()
        ids = torch.empty((nn, K), dtype=torch.int32, device=self.device)
        sc = torch.empty((nn, K), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(lib().ap_stage_seed_knn(self._h, _ptr(nodes), C.c_int64(nn), C.c_int32(K), _ptr(ids), _ptr(sc),
                                           _stream()), "ap_stage_seed_knn")
        return ids, sc

    def stage_refine(self, K: int, S: int, P: int, knn_ids, sp_ids, sp_sc, node_ids=None):
        dev = self.device
        nodes = _ids(node_ids, dev)
        nn = self.docs.n if nodes is None else nodes.numel()
        knn_ids = _dev(knn_ids, torch.int32, dev); sp_ids = _dev(sp_ids, torch.int32, dev)
        sp_sc = _dev(sp_sc, torch.float32, dev)
        assert knn_ids.shape == (self.docs.n, K) and sp_ids.shape == (3, self.docs.n, P)
        o_ids = torch.empty((nn, K), dtype=torch.int32, device=dev)
        o_sc = torch.empty((nn, K), dtype=torch.float32, device=dev)
        o_spi = torch.empty((3, nn, P), dtype=torch.int32, device=dev)
        o_sps = torch.empty((3, nn, P), dtype=torch.float32, device=dev)
        with torch.cuda.device(dev):
            _check(lib().ap_stage_refine(self._h, C.c_int32(K), C.c_int32(S), C.c_int32(P), _ptr(knn_ids), _ptr(sp_ids),
                                         _ptr(sp_sc), _ptr(nodes), C.c_int64(nn), _ptr(o_ids), _ptr(o_sc), _ptr(o_spi),
                                         _ptr(o_sps), _stream()), "ap_stage_refine")
        return o_ids, o_sc, o_spi, o_sps

    def stage_prune(self, K: int, R: int, knn_ids, knn_sc, node_ids=None, want_pm: bool = True):
        dev = self.device
        nodes = _ids(node_ids, dev)
        nn = self.docs.n if nodes is None else nodes.numel()
        knn_ids = _dev(knn_ids, torch.int32, dev); knn_sc = _dev(knn_sc, torch.float32, dev)
        assert knn_ids.shape == (self.docs.n, K)
        pm = torch.empty((nn, K, K), dtype=torch.float32, device=dev) if want_pm else None
        count = torch.empty((nn, K), dtype=torch.int32, device=dev)
        sorted_ids = torch.empty((nn, K), dtype=torch.int32, device=dev)
        se = torch.empty((nn, R), dtype=torch.int32, device=dev)
        ke = torch.empty((nn, max(R // 2, 1)), dtype=torch.int32, device=dev)
        ke_count = torch.empty(nn, dtype=torch.int32, device=dev)
        flag = torch.empty((nn, K), dtype=torch.int32, device=dev)
        with torch.cuda.device(dev):
            _check(lib().ap_stage_prune(self._h, C.c_int32(K), C.c_int32(R), _ptr(knn_ids), _ptr(knn_sc), _ptr(nodes),
                                        C.c_int64(nn), _ptr(pm), _ptr(count), _ptr(sorted_ids), _ptr(se), _ptr(ke),
                                        _ptr(ke_count), _ptr(flag), _stream()), "ap_stage_prune")
        return dict(pm=pm, count=count, sorted_ids=sorted_ids, se=se, ke=ke, ke_count=ke_count, flag=flag)

    def stage_assemble(self, R: int, K: int, P: int, se, sorted_ids, sp_ids):
        dev = self.device
        se = _dev(se, torch.int32, dev); sorted_ids = _dev(sorted_ids, torch.int32, dev)
        sp_ids = _dev(sp_ids, torch.int32, dev)
        n = self.docs.n
        assert se.shape == (n, R) and sorted_ids.shape == (n, K) and sp_ids.shape == (3, n, P)
        out = torch.empty((n, R), dtype=torch.int32, device=dev)
        with torch.cuda.device(dev):
            _check(lib().ap_stage_assemble(self._h, C.c_int32(R), C.c_int32(K), C.c_int32(P), _ptr(se), _ptr(sorted_ids),
                                           _ptr(sp_ids), _ptr(out), _stream()), "ap_stage_assemble")
        return out

    def stage_entry_points(self, E: int):
        out = torch.empty(E, dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            _check(lib().ap_stage_entry_points(self._h, C.c_int32(E), _ptr(out), _stream()), "ap_stage_entry_points")
        return out

    def export_graph(self):
        dev = self.device
        n, R, E = self.docs.n, self.params.degree, self.params.n_entry
        sem = torch.empty((n, R), dtype=torch.int32, device=dev)
        kw = torch.empty((n, R // 2), dtype=torch.int32, device=dev)
        kc = torch.empty(n, dtype=torch.int32, device=dev)
        ent = torch.empty(E, dtype=torch.int32, device=dev)
        with torch.cuda.device(dev):
            _check(lib().ap_export_graph(self._h, _ptr(sem), _ptr(kw), _ptr(kc), _ptr(ent), _stream()), "ap_export_graph")
        return sem, kw, kc, ent

    def search_stats(self, nq: int):
        """(counts[nq, 3] = candidates scored, iterations, dense rows skipped per query; search-kernel ms) of the last search."""
        counts = torch.empty((nq, 3), dtype=torch.int32, device=self.device)
        ms = C.c_float(0)
        with torch.cuda.device(self.device):
            _check(lib().ap_search_stats(self._h, _ptr(counts), C.c_int32(nq), C.byref(ms), _stream()), "ap_search_stats")
        return counts, float(ms.value)

    def search_kernel_ms(self) -> float:
        ms = C.c_float(0)
        _check(lib().ap_search_stats(self._h, None, C.c_int32(0), C.byref(ms), None), "ap_search_stats")
        return float(ms.value)

    def build_counters(self):
        out = (C.c_uint64 * 2)()
        with torch.cuda.device(self.device):
            _check(lib().ap_build_counters(self._h, out, _stream()), "ap_build_counters")
        return dict(refine_similarities=int(out[0]), seed_flops=int(out[1]))

    def build_timings(self):
        out = (C.c_float * 6)()
        _check(lib().ap_build_timings(self._h, out), "ap_build_timings")
        return dict(zip(("ingest", "seed", "refine", "prune", "assemble", "total"), [float(x) for x in out]))
