"""The seeded input generator (shared by the oracle's tests and the GPU path; it holds none of the method's
arithmetic): the recipe's stated properties, and that generating a corpus in row blocks changes nothing."""
import numpy as np

from paper_2511_00855_amd import synth


def _equal(a, b):
    for f in ("dense", "sp_indptr", "sp_idx", "sp_val", "tx_indptr", "tx_idx", "tx_val", "dense_bf16"):
        x, y = getattr(a, f), getattr(b, f)
        if x is None or y is None:
            assert x is None and y is None, f
            continue
        assert x.dtype == y.dtype and x.shape == y.shape and np.array_equal(x.view(np.uint8), y.view(np.uint8)), f


def test_block_size_does_not_change_the_data(monkeypatch):
    cases = (("tiny", dict(n=3000)), ("cfg3", dict(n=2500, nq=10)),
             ("tiny", dict(n=2100, dim=8, bf16=True, sp=("poisson", 170), tx=("lognormal", 140))))
    whole = [synth.make_workload(name, seed=5, **kw) for name, kw in cases]
    said = []
    monkeypatch.setattr(synth, "_ROW_BLOCK", 512)
    for (name, kw), ref in zip(cases, whole):
        w = synth.make_workload(name, seed=5, progress=said.append, **kw)
        _equal(w.docs, ref.docs)
        _equal(w.queries, ref.queries)
    assert any("dense rows" in m for m in said) and any("text of rows" in m for m in said)


def test_recipe_properties():
    w = synth.make_workload("cfg2", seed=1, n=4000, nq=200)
    d, q = w.docs, w.queries
    assert np.allclose(np.linalg.norm(d.dense, axis=1), 1.0, atol=1e-5)
    for v in (d, q):
        for pre, vocab in (("sp", v.sp_vocab), ("tx", v.tx_vocab)):
            ip, idx, val = getattr(v, pre + "_indptr"), getattr(v, pre + "_idx"), getattr(v, pre + "_val")
            assert ip[0] == 0 and (np.diff(ip) >= 0).all() and ip[-1] == len(idx) == len(val)
            assert idx.min() >= 0 and idx.max() < vocab
            inner = np.ones(len(idx), bool); inner[ip[1:-1][ip[1:-1] < len(idx)]] = False; inner[0] = False
            assert (np.diff(idx)[inner[1:]] > 0).all()          # strictly ascending within every row
            assert (val > 0).all()
    assert abs(np.diff(d.sp_indptr).mean() - 120) < 3           # ~120 sparse entries per document (Poisson)
    assert 35 < np.diff(d.tx_indptr).mean() < 60                # distinct terms of ~60-token texts
    assert abs(d.tx_val.sum() / d.n - 60) < 3                   # mean text length 60 tokens
    assert abs(np.diff(q.sp_indptr).mean() - 20) < 1 and abs(q.tx_val.sum() / q.n - 8) < 0.5
    # Zipf: the most frequent term is far more frequent than the median one
    cnt = np.bincount(d.sp_idx, minlength=d.sp_vocab)
    assert cnt.max() > 50 * max(1, int(np.median(cnt[cnt > 0])))
    # same seed, same data; another seed, other data
    again = synth.make_workload("cfg2", seed=1, n=4000, nq=200)
    _equal(again.docs, d)
    other = synth.make_workload("cfg2", seed=2, n=4000, nq=200)
    assert not np.array_equal(other.docs.dense, d.dense)
