"""The search entry point that allocates nothing (ap_search_batch_noalloc: visited sets in a static device array)
against ap_search_batch, through the C ABI: same ids and scores bit for bit, on calls in a row that shrink, on
several slabs of queries, on another index right after (the array keeps the last call's contents), and with no
change in free device memory across the calls."""
import numpy as np
import pytest
import torch

from paper_2511_00855_amd import binding as B
from paper_2511_00855_amd.synth import make_workload, subset_vecset

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _out(nq, k, dev):
    # poisoned output buffers: whatever the call leaves untouched shows
    return (torch.full((nq, k), -7, dtype=torch.int32, device=dev), torch.full((nq, k), float("nan"), dtype=torch.float32, device=dev))


def test_noalloc_search_equals_search_batch(debug_knobs):
    w = make_workload("tiny", seed=33, n=3000, nq=40)
    docs = B.DeviceVecs(w.docs); qs = B.DeviceVecs(w.queries)
    ix = B.Index.build(docs, B.build_params(w.degree))
    k, dev = 10, docs.device
    wq = torch.from_numpy(np.random.default_rng(4).uniform(0.1, 1.0, (qs.n, 3)).astype(np.float32)).to(dev)
    small = B.DeviceVecs(subset_vecset(w.queries, np.arange(13)))
    w2 = make_workload("tiny", seed=34, n=700, nq=9, dim=64)
    docs2 = B.DeviceVecs(w2.docs); qs2 = B.DeviceVecs(w2.queries)
    ix2 = B.Index.build(docs2, B.build_params(16, nd_rounds=2, n_entry=16))
    # references from the existing entry point, and every buffer the calls below need, before the memory reading
    ref = {}
    for name, (q, beam, width, pw) in dict(first=(qs, 96, 2, wq), second=(small, 64, 1, wq[:13].contiguous()),
                                           default_w=(qs, 48, 1, None)).items():
        ref[name] = [t.clone() for t in ix.search_batch(q, k, beam, pw, search_width=width)]
    ref2 = [t.clone() for t in ix2.search_batch(qs2, 5, 32, None)]
    bufs = {name: _out(n, kk, dev) for name, (n, kk) in dict(first=(40, k), second=(13, k), default_w=(40, k), slabs=(40, k),
                                                             other=(9, 5), again=(40, k)).items()}
    wq13 = wq[:13].contiguous()
    # corpora this small would keep their visited sets in LDS: hold them in the workspace, which is what this entry
    # point is about (the references above ran with the sets in LDS: same bits either way)
    debug_knobs("search_visited_global", 1)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]

    _say("no-alloc search: 40 queries, beam 96, two parents per iteration")
    ix.search_batch_noalloc(qs, k, 96, wq, bufs["first"], search_width=2)
    _say("no-alloc search: the next call, 13 queries, beam 64")
    ix.search_batch_noalloc(small, k, 64, wq13, bufs["second"])
    ix.search_batch_noalloc(qs, k, 48, None, bufs["default_w"])
    _say("no-alloc search: another index right after")
    ix2.search_batch_noalloc(qs2, 5, 32, None, bufs["other"])
    _say("no-alloc search: slabs of seven queries")
    debug_knobs("search_workspace_bytes", 7 * ((docs.n + 31) // 32) * 4)
    ix.search_batch_noalloc(qs, k, 96, wq, bufs["slabs"], search_width=2)
    debug_knobs("search_workspace_bytes", 0)
    debug_knobs("search_visited_global", 0)     # and once with the library's own choice (LDS here)
    ix.search_batch_noalloc(qs, k, 96, wq, bufs["again"], search_width=2)
    debug_knobs("search_visited_global", 1)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0, "device memory changed across calls that must not allocate"

    for name, want in (("first", ref["first"]), ("second", ref["second"]), ("default_w", ref["default_w"]), ("other", ref2),
                       ("slabs", ref["first"]), ("again", ref["first"])):
        assert torch.equal(bufs[name][0], want[0]), name
        assert torch.equal(bufs[name][1], want[1]), name

    # a workspace too small for one query's visited bits is refused, with the limit in the message
    debug_knobs("search_workspace_bytes", 64)
    with pytest.raises(RuntimeError, match="static workspace of 64 bytes"):
        ix.search_batch_noalloc(qs, k, 96, wq, bufs["again"])
    debug_knobs("search_workspace_bytes", 0)
    # argument checks of the existing entry point hold here too
    with pytest.raises(RuntimeError, match="beam"):
        ix.search_batch_noalloc(qs, k, 5, wq, bufs["again"])
    ix.close(); ix2.close()
