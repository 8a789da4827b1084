"""Seeded synthetic inputs shaped like the paper's workloads (Table 1 and the
experiment settings: a dense embedding, a learned-sparse vector and a bag of
text tokens per document).

This module holds NO arithmetic of the method: it only draws random corpora and
queries.  Both the CPU oracle and the HIP path consume what it returns; BM25
weighting, scoring, graph construction and search live elsewhere.

Everything is a pure function of (config, seed), produced with
``numpy.random.default_rng``.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np


@dataclass
class VecSet:
    """A set of fused vectors: dense rows + learned-sparse CSR + text CSR.

    ``tx_val`` holds raw term counts (tf) for both documents and queries.
    ``dense_bf16`` (uint16 bit patterns) is present only when the config stores
    the dense part in bf16; then ``dense`` holds exactly those bf16 values
    widened back to fp32, so both sides of a parity test see the same numbers.
    """
    n: int
    dim: int
    dense: np.ndarray                 # float32 [n, dim]
    sp_indptr: np.ndarray             # int64 [n+1]
    sp_idx: np.ndarray                # int32 [nnz], strictly ascending per row
    sp_val: np.ndarray                # float32 [nnz]
    tx_indptr: np.ndarray             # int64 [n+1]
    tx_idx: np.ndarray                # int32 [nnz], strictly ascending per row
    tx_val: np.ndarray                # float32 [nnz] term counts
    sp_vocab: int = 0
    tx_vocab: int = 0
    dense_bf16: Optional[np.ndarray] = None


@dataclass
class Workload:
    name: str
    docs: VecSet
    queries: VecSet
    weights: Tuple[float, float, float]
    degree: int
    beam: int
    k: int
    bm25_k1: float = 1.2
    bm25_b: float = 0.75
    extra: Dict[str, object] = field(default_factory=dict)


def _zipf_cdf(vocab: int, s: float) -> np.ndarray:
    p = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(p)
    return c / c[-1]


def _draw_terms(rng: np.random.Generator, cdf: np.ndarray, perm: np.ndarray, n: int) -> np.ndarray:
    """n i.i.d. term ids: Zipf rank by inverse CDF, rank -> id by a fixed permutation."""
    r = np.searchsorted(cdf, rng.random(n), side="right")
    np.minimum(r, len(cdf) - 1, out=r)
    return perm[r]


def _say(progress, msg: str) -> None:
    if progress is not None:
        progress(msg)


_ROW_BLOCK = 1 << 19   # rows per step of the generators below (a step of a large corpus takes seconds, not minutes)


def _bags(rng, cdf, perm, counts: np.ndarray, progress=None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Token bags WITH repetition -> CSR of (term id ascending, count).  Rows are handled in blocks; the tokens of
    all rows come from one stream of draws, so the result does not depend on the block size."""
    n = len(counts)
    vocab = len(cdf)
    indptr = np.zeros(n + 1, dtype=np.int64)
    terms, tfs = [], []
    for b0 in range(0, n, _ROW_BLOCK):
        b1 = min(n, b0 + _ROW_BLOCK)
        c = counts[b0:b1]
        rows = np.repeat(np.arange(b0, b1, dtype=np.int64), c)
        toks = _draw_terms(rng, cdf, perm, int(c.sum())).astype(np.int64)
        uk, cnt = np.unique(rows * vocab + toks, return_counts=True)
        indptr[b0 + 1:b1 + 1] = np.bincount(uk // vocab - b0, minlength=b1 - b0)
        terms.append((uk % vocab).astype(np.int32)); tfs.append(cnt.astype(np.float32))
        if n > _ROW_BLOCK:
            _say(progress, f"text of rows {b0}..{b1} of {n}")
    np.cumsum(indptr, out=indptr)
    return indptr, np.concatenate(terms) if terms else np.zeros(0, np.int32), np.concatenate(tfs) if tfs else np.zeros(0, np.float32)


def _first_distinct(draws: np.ndarray, need: np.ndarray) -> np.ndarray:
    """Mask of the first need[r] distinct values of row r of `draws`, in draw order (negative = void)."""
    order = np.argsort(draws, axis=1, kind="stable")
    srt = np.take_along_axis(draws, order, axis=1)
    first_sorted = np.ones_like(srt, dtype=bool)
    first_sorted[:, 1:] = srt[:, 1:] != srt[:, :-1]
    first_sorted &= srt >= 0
    first = np.zeros_like(first_sorted)
    np.put_along_axis(first, order, first_sorted, axis=1)
    return first & (np.cumsum(first, axis=1) <= need[:, None])


def _distinct_sets(rng, cdf, perm, counts: np.ndarray, progress=None) -> Tuple[np.ndarray, np.ndarray]:
    """Per row, `counts[i]` DISTINCT Zipf term ids (keep drawing until distinct), sorted.

    Rows are handled in blocks: every row of a block draws the same number of
    candidates (enough for almost all rows) and keeps its first `counts[i]`
    distinct ones in draw order; the few rows that still lack ids keep drawing."""
    n = len(counts)
    vocab = len(cdf)
    counts = np.minimum(counts, vocab).astype(np.int64)
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=indptr[1:])
    out = np.empty(int(indptr[-1]), dtype=np.int32)
    block = 65536
    for b0 in range(0, n, block):
        b1 = min(n, b0 + block)
        need = counts[b0:b1]
        rows = np.nonzero(need > 0)[0]
        if b0 and b0 % _ROW_BLOCK == 0:
            _say(progress, f"sparse lists of rows ..{b0} of {n}")
        if not len(rows):
            continue
        m = int(need.max()) * 2 + 8
        draws = _draw_terms(rng, cdf, perm, len(rows) * m).astype(np.int32).reshape(len(rows), m)
        keep = _first_distinct(draws, need[rows])
        nk = keep.sum(axis=1)
        done = nk == need[rows]
        # complete rows: sort each row's ids and store, all at once
        kd = keep[done]
        vals = draws[done][kd]
        rid = np.repeat(np.arange(int(done.sum())), nk[done])
        o = np.lexsort((vals, rid))
        starts = indptr[b0 + rows[done]]
        seg0 = np.concatenate([[0], np.cumsum(nk[done])])[:-1]
        dest = starts[rid] + (np.arange(len(vals)) - seg0[rid])
        out[dest] = vals[o]
        # the rest keep drawing, one row at a time
        for r in np.nonzero(~done)[0]:
            i = rows[r]
            have = draws[r][keep[r]]
            while len(have) < need[i]:
                extra = _draw_terms(rng, cdf, perm, int(need[i]) * 2 + 8).astype(np.int32)
                extra = extra[~np.isin(extra, have)]
                _, f = np.unique(extra, return_index=True)
                have = np.concatenate([have, extra[np.sort(f)][: need[i] - len(have)]])
            out[indptr[b0 + i]:indptr[b0 + i + 1]] = np.sort(have)
    return indptr, out


def f32_to_bf16_rne(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round-to-nearest-even (storage format conversion only)."""
    flat = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    out = np.empty(flat.shape, dtype=np.uint16)
    step = 1 << 24
    for a in range(0, len(flat), step):
        u = flat[a:a + step].view(np.uint32).astype(np.uint64)
        out[a:a + step] = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    return out.reshape(np.shape(x))


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def _dense(rng, n: int, dim: int, bf16: bool, progress=None):
    """Unit-norm Gaussian rows, generated in row blocks out of one stream of draws (the result does not depend on
    the block size).  bf16: the rows are rounded to bf16 and `dense` holds those values widened back."""
    x = np.empty((n, dim), dtype=np.float32)
    b = np.empty((n, dim), dtype=np.uint16) if bf16 else None
    for r0 in range(0, n, _ROW_BLOCK):
        r1 = min(n, r0 + _ROW_BLOCK)
        blk = rng.standard_normal((r1 - r0, dim), dtype=np.float32)
        blk /= np.linalg.norm(blk, axis=1, keepdims=True).astype(np.float32)
        if bf16:
            b[r0:r1] = f32_to_bf16_rne(blk)
            blk = bf16_to_f32(b[r0:r1])
        x[r0:r1] = blk
        if n > _ROW_BLOCK:
            _say(progress, f"dense rows {r0}..{r1} of {n}")
    return x, b


def make_vecset(rng, n: int, dim: int, *, bf16: bool, sp_vocab: int, sp_counts: np.ndarray,
                tx_vocab: int, tx_counts: np.ndarray, sp_cdf, sp_perm, tx_cdf, tx_perm, progress=None) -> VecSet:
    dense, dense_b = _dense(rng, n, dim, bf16, progress)
    sp_indptr, sp_idx = _distinct_sets(rng, sp_cdf, sp_perm, sp_counts, progress)
    sp_val = np.abs(rng.standard_normal(len(sp_idx))).astype(np.float32)
    # a weight that rounds to 0 would make "nnz" a lie; nudge (probability ~0)
    sp_val[sp_val == 0] = np.float32(1e-3)
    tx_indptr, tx_idx, tx_val = _bags(rng, tx_cdf, tx_perm, tx_counts, progress)
    return VecSet(n=n, dim=dim, dense=dense, sp_indptr=sp_indptr, sp_idx=sp_idx, sp_val=sp_val,
                  tx_indptr=tx_indptr, tx_idx=tx_idx, tx_val=tx_val, sp_vocab=sp_vocab,
                  tx_vocab=tx_vocab, dense_bf16=dense_b)


def _lognormal_lengths(rng, n: int, mean: float, sigma: float = 0.5, lo: int = 5, hi: int = 512):
    mu = np.log(mean) - 0.5 * sigma * sigma
    return np.clip(np.rint(rng.lognormal(mu, sigma, n)), lo, hi).astype(np.int64)


def _poisson_min1(rng, lam: float, n: int):
    return np.maximum(rng.poisson(lam, n), 1).astype(np.int64)


CONFIGS = {
    # name: dict(N, nq, dim, bf16, vocab, doc sparse nnz ("fixed", v) or ("poisson", lam),
    #            doc tokens ("fixed", v) or ("lognormal", mean), query nnz, query tokens,
    #            weights, degree, beam, k)
    "tiny": dict(n=2_000, nq=100, dim=128, bf16=False, vocab=10_000, sp=("fixed", 32), tx=("fixed", 40),
                 qsp=("fixed", 8), qtx=("fixed", 6), weights=(0.5, 0.3, 0.2), degree=32, beam=64, k=10),
    "cfg2": dict(n=100_000, nq=10_000, dim=768, bf16=False, vocab=30_522, sp=("poisson", 120),
                 tx=("lognormal", 60), qsp=("poisson", 20), qtx=("poisson", 8), weights=(0.5, 0.3, 0.2),
                 degree=64, beam=128, k=10),
    "cfg3": dict(n=1_000_000, nq=10_000, dim=1024, bf16=True, vocab=250_002, sp=("poisson", 100),
                 tx=("lognormal", 60), qsp=("poisson", 20), qtx=("poisson", 8), weights=(0.4, 0.4, 0.2),
                 degree=64, beam=128, k=10),
    "cfg5": dict(n=8_800_000, nq=10_000, dim=1024, bf16=True, vocab=250_002, sp=("poisson", 80),
                 tx=("lognormal", 55), qsp=("poisson", 20), qtx=("poisson", 8), weights=(0.4, 0.4, 0.2),
                 degree=64, beam=128, k=10),
}


def _counts(rng, spec, n):
    kind, v = spec
    if kind == "fixed":
        return np.full(n, int(v), dtype=np.int64)
    if kind == "poisson":
        return _poisson_min1(rng, float(v), n)
    if kind == "lognormal":
        return _lognormal_lengths(rng, n, float(v))
    raise ValueError(kind)


def make_workload(name: str = "tiny", seed: int = 0, *, n: Optional[int] = None, nq: Optional[int] = None,
                  progress=None, **override) -> Workload:
    """Build one of the named workloads.  `n`, `nq` and any config key can be
    overridden to get a smaller case with the same distributions (used by tests
    that need several tiles and a ragged tail but not the full size).
    progress: called with a short message after every block of a large corpus."""
    c = dict(CONFIGS[name])
    c.update(override)
    if n is not None:
        c["n"] = n
    if nq is not None:
        c["nq"] = nq
    rng = np.random.default_rng(seed)
    vocab = c["vocab"]
    cdf = _zipf_cdf(vocab, 1.1)
    sp_perm = rng.permutation(vocab).astype(np.int64)
    tx_perm = rng.permutation(vocab).astype(np.int64)
    common = dict(sp_vocab=vocab, tx_vocab=vocab, sp_cdf=cdf, sp_perm=sp_perm, tx_cdf=cdf, tx_perm=tx_perm)
    docs = make_vecset(rng, c["n"], c["dim"], bf16=c["bf16"], sp_counts=_counts(rng, c["sp"], c["n"]),
                       tx_counts=_counts(rng, c["tx"], c["n"]), progress=progress, **common)
    qs = make_vecset(rng, c["nq"], c["dim"], bf16=False, sp_counts=_counts(rng, c["qsp"], c["nq"]),
                     tx_counts=np.maximum(_counts(rng, c["qtx"], c["nq"]), 1), **common)
    return Workload(name=name, docs=docs, queries=qs, weights=tuple(c["weights"]), degree=c["degree"],
                    beam=c["beam"], k=c["k"], extra=dict(seed=seed, config=c))


def make_keywords(queries: VecSet, seed: int = 0, max_terms: int = 2, stride: int = 4, p_none: float = 0.0) -> np.ndarray:
    """Required keywords for a keyword-constrained search: for each query 1..max_terms
    of its own distinct text tokens, chosen uniformly, as an nq x stride int32 array
    padded with -1.  With probability p_none a query gets no keyword at all."""
    assert 1 <= max_terms <= stride
    rng = np.random.default_rng(seed)
    out = np.full((queries.n, stride), -1, np.int32)
    for i in range(queries.n):
        terms = queries.tx_idx[queries.tx_indptr[i]:queries.tx_indptr[i + 1]]
        if len(terms) == 0 or rng.random() < p_none:
            continue
        m = min(int(rng.integers(1, max_terms + 1)), len(terms))
        out[i, :m] = rng.choice(terms, m, replace=False)
    return out


def subset_vecset(v: VecSet, rows) -> VecSet:
    """The listed rows of a vector set as a vector set of their own (CSR parts rebuilt)."""
    rows = np.asarray(rows, np.int64)
    parts = {}
    for pre in ("sp", "tx"):
        ip = getattr(v, pre + "_indptr")
        lens = (ip[1:] - ip[:-1])[rows]
        take = np.concatenate([np.arange(ip[r], ip[r + 1]) for r in rows]) if len(rows) else np.zeros(0, np.int64)
        parts[pre + "_indptr"] = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        parts[pre + "_idx"] = getattr(v, pre + "_idx")[take]
        parts[pre + "_val"] = getattr(v, pre + "_val")[take]
    bf = None if v.dense_bf16 is None else v.dense_bf16[rows]
    return dataclasses.replace(v, n=len(rows), dense=v.dense[rows], dense_bf16=bf, **parts)


def make_entity_graph(n_docs: int, nq: int, seed: int = 0, n_ent: Optional[int] = None, ents_per_doc=(1, 3),
                      kg_degree: int = 4, max_query_ents: int = 2, stride: int = 4):
    """A synthetic stand-in for a knowledge graph extracted from a corpus: every document mentions a few entities
    (distinct ids, ascending), entities are joined by undirected relations (about kg_degree per entity, no
    self-relations), and every query names 1..max_query_ents entities of one randomly chosen document.  Returns a
    namespace of CSR arrays: doc_ent_indptr / doc_ent, kg_indptr / kg_idx (symmetric), and q_ent (nq x stride, -1
    padded)."""
    from types import SimpleNamespace
    rng = np.random.default_rng(seed)
    n_ent = int(n_ent or max(8, n_docs // 8))
    counts = rng.integers(ents_per_doc[0], ents_per_doc[1] + 1, n_docs)
    indptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    ids = np.empty(indptr[-1], np.int32)
    for i in range(n_docs):
        ids[indptr[i]:indptr[i + 1]] = np.sort(rng.choice(n_ent, counts[i], replace=False))
    a = rng.integers(0, n_ent, n_ent * kg_degree // 2)
    b = rng.integers(0, n_ent, n_ent * kg_degree // 2)
    keep = a != b
    pairs = np.unique(np.concatenate([np.stack([a[keep], b[keep]], 1), np.stack([b[keep], a[keep]], 1)]), axis=0)
    kg_indptr = np.concatenate([[0], np.cumsum(np.bincount(pairs[:, 0], minlength=n_ent))]).astype(np.int64)
    kg_idx = pairs[:, 1].astype(np.int32)          # np.unique sorted the pairs: ascending targets per source
    q_ent = np.full((nq, stride), -1, np.int32)
    for q in range(nq):
        d = int(rng.integers(0, n_docs))
        mine = ids[indptr[d]:indptr[d + 1]]
        m = min(int(rng.integers(1, max_query_ents + 1)), len(mine), stride)
        q_ent[q, :m] = rng.choice(mine, m, replace=False)
    return SimpleNamespace(n_ent=n_ent, doc_ent_indptr=indptr, doc_ent=ids, kg_indptr=kg_indptr, kg_idx=kg_idx, q_ent=q_ent)
