#!/usr/bin/env python3
"""Benchmark of the hybrid-index hot path on one MI355X.

One "step" = one batched search (S7-S9) of all queries of the workload on an
index that this same run built on the GPU (S0-S6; build time reported beside
it).  The headline value is queries per second at the first setting of the
sweep (pool size `beam`, parents per iteration `width`) whose recall@10 against
exact hybrid top-10 reaches 0.95.  The headline workload is config 3 (one
million documents, d = 1024 stored bf16); config 2 (100,000 documents, f32) is
measured first, briefly, and reported as the `cfg2` object of the same line.
Inputs are seeded synthetic data resident in HBM before any timed region.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E data-sheet peak
MFMA_PEAK_TFLOPS = {True: 2500.0, False: 157.3}   # dense bf16 / fp32 matrix peaks (bf16 rows / f32 rows)

# (beam, width) settings tried in order until the recall target is met
SWEEPS = {
    "tiny": "64,128,256,512",
    "cfg2": "128,512,1024,1536,2048:16,2080:16,2112:16,2144:16,2176:16,2240:16,2304:16,2560,3072,4096:4,6144:4,8192:16,12288:16,16384:16",
    "cfg3": "128,1024,4096:4,8192:16,12288:16,14336:16,15360:16,16384:16",
    "cfg5": "128,1024,4096:4,16384:16",
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def recall_at_k(ids, gt):
    import numpy as np
    return float(np.mean([len(set(a.tolist()) & set(b.tolist())) / float(len(b)) for a, b in zip(ids, gt)]))


def parse_sweep(text):
    out = []
    for item in text.split(","):
        beam, _, width = item.partition(":")
        out.append((int(beam), int(width or 1)))
    return out


def keyword_ground_truth(w, ix, wq, kw, sample, k):
    """Exact top-k among the documents that hold at least one of a query's required terms, for the sampled queries:
    exhaustive scores from ap_hybrid_scores; filter and top-k in torch (measurement only; ties by lower id as torch
    returns them is not relied on: tests compare it with a brute force on the oracle's scores up to near-ties).
    Returns (ids [len(sample), k] with -1 where fewer than k documents satisfy, scores)."""
    import numpy as np
    import scipy.sparse as sps
    import torch
    from paper_2511_00855_amd import binding as B
    from paper_2511_00855_amd.synth import subset_vecset
    n = w.docs.n
    inv = sps.csr_matrix((np.ones(len(w.docs.tx_idx), np.int8), w.docs.tx_idx, w.docs.tx_indptr),
                         shape=(n, w.docs.tx_vocab)).tocsc()
    gt, gs = [], []
    for c0 in range(0, len(sample), 250):
        rows = sample[c0:c0 + 250]
        sub = B.DeviceVecs(subset_vecset(w.queries, rows), "cuda:0")
        allc = torch.arange(n, dtype=torch.int32, device="cuda:0").repeat(len(rows), 1)
        sc = ix.hybrid_scores(sub, allc, wq[torch.from_numpy(rows).to("cuda:0")])[:, :, 3]
        rr, cc = [np.zeros(0, np.int64)], [np.zeros(0, np.int64)]
        for x, qi in enumerate(rows):
            for t in kw[qi][kw[qi] >= 0]:
                d = inv.indices[inv.indptr[t]:inv.indptr[t + 1]]
                rr.append(np.full(len(d), x, np.int64)); cc.append(d.astype(np.int64))
        mask = torch.zeros(sc.shape, dtype=torch.bool, device="cuda:0")
        mask[torch.from_numpy(np.concatenate(rr)).to("cuda:0"), torch.from_numpy(np.concatenate(cc)).to("cuda:0")] = True
        top = sc.masked_fill(~mask, float("-inf")).topk(k, dim=1)
        ids = torch.where(torch.isinf(top.values), torch.full_like(top.indices, -1), top.indices)
        gt.append(ids.cpu().numpy()); gs.append(top.values.cpu().numpy())
        del sc, mask, allc
    return np.concatenate(gt), np.concatenate(gs)


def keyword_leg(args, w, ix, qs, wq, k, chosen):
    """Keyword-constrained search (Section 4.2.2): every query requires 1-2 of its own text tokens.  Ground truth
    = exact top-k among the documents holding a required term, on up to 1000 sampled queries."""
    import numpy as np
    import torch
    from paper_2511_00855_amd.synth import make_keywords
    nq = qs.n
    kw = make_keywords(w.queries, seed=1, max_terms=2, stride=2)
    sample = np.arange(0, nq, max(1, nq // 1000))[:1000]
    gt, _ = keyword_ground_truth(w, ix, wq, kw, sample, k)
    out = []
    for beam in sorted({w.beam, 512, chosen}):
        for edges in (True, False):
            ix.search_batch_keywords(qs, k, beam, kw, wq, use_kw_edges=edges)
            torch.cuda.synchronize()
            t1 = time.time()
            ids, _ = ix.search_batch_keywords(qs, k, beam, kw, wq, use_kw_edges=edges)
            torch.cuda.synchronize()
            dt = time.time() - t1
            counts, kms = ix.search_stats(nq)
            got = ids.cpu().numpy()[sample]
            rec = float(np.mean([len(set(a[a >= 0].tolist()) & set(b[b >= 0].tolist())) / max(1, int((b >= 0).sum()))
                                 for a, b in zip(got, gt)]))
            out.append(dict(beam=beam, keyword_edges=edges, recall=round(rec, 4), qps=round(nq / dt, 1), kernel_ms=round(kms, 3),
                            dists_per_query=round(float(counts[:, 0].float().mean().item()), 1)))
            log(f"[bench] keywords beam {beam} edges {edges}: recall@{k} {rec:.4f} (on {len(sample)} sampled queries)  "
                f"{nq / dt:,.0f} qps  kernel {kms:.2f} ms  {out[-1]['dists_per_query']:.0f} dists/query")
    return dict(required_terms="1-2 of each query's own text tokens, any-match", sampled_queries=len(sample), sweep=out)


def entities_leg(args, w, ix, qs, wq, k):
    """Search with entities (Sections 3.4 and 4.2.3) on a synthetic entity graph over this corpus (every document
    mentions 1-3 entities, about four relations per entity, every query names 1-2 entities of one document): what
    the augmentation costs against the plain search of the same index at the same beam, and how often it changes the
    answer.  The paper applies the knowledge graph to small shards; so should --n."""
    import numpy as np
    import torch
    from paper_2511_00855_amd.synth import make_entity_graph
    nq = qs.n
    kgs = make_entity_graph(w.docs.n, nq, seed=5)
    ix.set_knowledge_graph(kgs, le_cap=16)
    out = []
    for beam in (64, 128, 512):
        row = dict(beam=beam)
        ans = {}
        for name, fn in (("plain", lambda: ix.search_batch(qs, k, beam, wq)),
                         ("entities", lambda: ix.search_batch_entities(qs, k, beam, kgs.q_ent, 0.5, 2, wq))):
            fn(); torch.cuda.synchronize()
            t1 = time.time()
            ids, _ = fn()
            torch.cuda.synchronize()
            row[name + "_qps"] = round(nq / (time.time() - t1), 1)
            row[name + "_kernel_ms"] = round(ix.search_kernel_ms(), 3)
            ans[name] = ids.cpu().numpy()
        row["qps_ratio"] = round(row["entities_qps"] / row["plain_qps"], 3)
        row["queries_whose_answer_changed"] = round(float((ans["plain"] != ans["entities"]).any(axis=1).mean()), 4)
        out.append(row)
        log(f"[bench] entities beam {beam}: plain {row['plain_qps']:,.0f} qps, with entities {row['entities_qps']:,.0f} qps "
            f"({row['qps_ratio']:.2f}x), answers changed for {100 * row['queries_whose_answer_changed']:.1f}% of the queries")
    return dict(entity_graph=f"{kgs.n_ent} entities, {len(kgs.doc_ent)} mentions, {len(kgs.kg_idx) // 2} relations; reward 0.5, 2 hops", sweep=out)


WEIGHT_SETTINGS = ((1.0, 0.0, 0.0), (0.0, 1.0, 0.0), (0.0, 0.0, 1.0), (0.5, 0.5, 0.0), (0.34, 0.33, 0.33))


def weights_leg(args, ix, qs, k):
    """Dynamic fusion (Theorem 1; Section 4.2.1): the same index, never rebuilt, searched under five other weight
    settings; per setting the exact top-k under those weights, then beams upward until the recall target."""
    import numpy as np
    import torch
    nq = qs.n
    out = []
    for wv in WEIGHT_SETTINGS:
        wq = torch.from_numpy(np.tile(np.float32(wv), (nq, 1))).to("cuda:0")
        gt = ix.bruteforce_topk(qs, k, wq)[0].cpu().numpy()
        rows, hit = [], None
        for beam in sorted(int(b) for b in args.weight_beams.split(",")):
            ix.search_batch(qs, k, beam, wq)
            torch.cuda.synchronize()
            t1 = time.time()
            ids, _ = ix.search_batch(qs, k, beam, wq)
            torch.cuda.synchronize()
            dt = time.time() - t1
            rec = recall_at_k(ids.cpu().numpy(), gt)
            counts, kms = ix.search_stats(nq)
            rows.append(dict(beam=beam, recall=round(rec, 4), qps=round(nq / dt, 1), kernel_ms=round(kms, 3),
                             dists_per_query=round(int(counts[:, 0].sum().item()) / nq, 1)))
            if rec >= args.target_recall:
                hit = rows[-1]
                break
        out.append(dict(weights=wv, at_target=hit, sweep=rows))
        last = rows[-1]
        log(f"[bench] weights {wv}: " + (f"recall {hit['recall']:.4f} at beam {hit['beam']}, {hit['qps']:,.0f} qps" if hit else
                                         f"target not reached; beam {last['beam']}: recall {last['recall']:.4f}, {last['qps']:,.0f} qps"))
    return out


def insert_leg(args, w, bp, docs, qs, wq, k, gt, sweep, build_s, bf16):
    """Insertion (Section 4.1, updates): an index over the first (1-f) of the corpus receives the last f; the
    updated index is searched at the settings of the main sweep, against the same ground truth as the rebuild."""
    import numpy as np
    import torch
    from paper_2511_00855_amd import binding as B
    from paper_2511_00855_amd.synth import subset_vecset
    n = w.docs.n
    out = []
    for f in sorted({args.insert, args.insert / 2, args.insert / 4}):
        n0 = n - int(round(n * f))
        old_docs = B.DeviceVecs(subset_vecset(w.docs, np.arange(n0)), "cuda:0", bf16=bf16)
        old = B.Index.build(old_docs, bp)
        torch.cuda.synchronize()
        t0 = time.time()
        new = old.insert(docs)
        torch.cuda.synchronize()
        dt = time.time() - t0
        st = dict(zip(("ingest", "candidate_sets", "merge_and_rescore", "prune", "assemble", "total"), new.build_timings().values()))
        rows = []
        for sw in sweep:
            beam, width = sw["beam"], sw["width"]
            new.search_batch(qs, k, beam, wq, search_width=width)
            torch.cuda.synchronize()
            t1 = time.time()
            ids, _ = new.search_batch(qs, k, beam, wq, search_width=width)
            torch.cuda.synchronize()
            qps = qs.n / (time.time() - t1)
            rows.append(dict(beam=beam, width=width, recall=round(recall_at_k(ids.cpu().numpy(), gt), 4), qps=round(qps, 1),
                             rebuilt_recall=sw["recall"], rebuilt_qps=sw["qps"]))
        out.append(dict(fraction=f, inserted=n - n0, seconds=round(dt, 3), rebuild_seconds=round(build_s, 3),
                        share_of_rebuild=round(dt / build_s, 3), stages_s={a: round(b, 3) for a, b in st.items()}, search=rows))
        log(f"[bench] insert {100 * f:.0f}% ({n - n0} docs): {dt:.3f}s = {100 * dt / build_s:.1f}% of the rebuild ({build_s:.2f}s); "
            + "; ".join(f"beam {r['beam']}: recall {r['recall']:.4f} (rebuilt {r['rebuilt_recall']:.4f})" for r in rows[:1] + rows[-1:]))
        new.close(); old.close()
        del old_docs
    return out


def graph_quality_leg(w, docs, ix, bp, rounds, nodes_wanted, bf16):
    """How good the construction's lists are (measured, not checked): for sampled nodes, the overlap of the K-list
    after the seed stage and after each refinement round with the exact K nearest documents under the construction's
    fused similarity (exhaustive document-document scores from ap_hybrid_scores_docs; top-K in torch: measurement
    only), and how often the inner-product rule of the joint pruning rejected a neighbour."""
    import numpy as np
    import torch
    N, K, R, S = docs.n, bp.knn_k, bp.degree, bp.nd_sample
    P = bp.sp_len or -(-R // 6)
    nodes = np.sort(np.random.default_rng(11).choice(N, min(nodes_wanted, N), replace=False)).astype(np.int32)
    wv = tuple(float(x) for x in bp.build_w)
    exact = []
    chunk = max(1, min(len(nodes), (1 << 28) // N))       # at most 4 GiB of scores at a time
    allc = torch.arange(N, dtype=torch.int32, device="cuda:0")
    for c0 in range(0, len(nodes), chunk):
        part = nodes[c0:c0 + chunk]
        sc = ix.hybrid_scores_docs(part, allc.repeat(len(part), 1), wv)[:, :, 3]
        sc[torch.arange(len(part), device="cuda:0"), torch.from_numpy(part.astype(np.int64)).to("cuda:0")] = float("-inf")
        exact.append(sc.topk(K, dim=1).indices.cpu().numpy())
        del sc
    exact = np.concatenate(exact)

    def overlap(lists):
        got = lists[torch.from_numpy(nodes.astype(np.int64)).to(lists.device)].cpu().numpy()
        return float(np.mean([len(set(a.tolist()) & set(b.tolist())) / float(K) for a, b in zip(got, exact)]))
    ids, sc = ix.stage_seed_knn(K)
    per_round = [round(overlap(ids), 4)]
    spi = torch.full((3, N, P), -1, dtype=torch.int32, device="cuda:0")
    sps = torch.full((3, N, P), float("-inf"), dtype=torch.float32, device="cuda:0")
    for _ in range(rounds):
        ids, sc, spi, sps = ix.stage_refine(K, S, P, ids, spi, sps)
        per_round.append(round(overlap(ids), 4))
    pr = ix.stage_prune(K, R, ids, sc, nodes, want_pm=False)
    se, srt = pr["se"].cpu().numpy(), pr["sorted_ids"].cpu().numpy()
    ip_fired = float(np.mean([not np.array_equal(a, b[:R]) for a, b in zip(se, srt)]))
    del ids, sc, spi, sps
    return dict(sampled_nodes=int(len(nodes)), knn_k=K,
                klist_recall_vs_exact_fused_knn=dict(seed=per_round[0], after_round=per_round[1:]),
                nodes_where_ip_rule_rejected_a_neighbour=round(ip_fired, 4))


def run_workload(args, name, *, n, nq, steps, warmup, sweep_text, cpu_seconds, graph_nodes, extra_legs):
    """Generates the workload, builds its index, finds the first sweep setting that reaches the recall target, times
    `steps` searches there, and returns everything the JSON line reports about it."""
    import numpy as np
    import torch
    from paper_2511_00855_amd import binding as B
    from paper_2511_00855_amd.synth import make_workload

    t0 = time.time()
    w = make_workload(name, seed=0, n=n, nq=nq, progress=lambda m: log(f"[bench] {name} generating: {m}"))
    cfg = w.extra["config"]
    bf16 = bool(cfg["bf16"])
    log(f"[bench] workload {name}: n={w.docs.n} nq={w.queries.n} dim={w.docs.dim} bf16={bf16} generated in {time.time() - t0:.1f}s")
    docs = B.DeviceVecs(w.docs, "cuda:0", bf16=bf16)
    qs = B.DeviceVecs(w.queries, "cuda:0")
    nq, k, N = qs.n, w.k, w.docs.n
    wq = torch.from_numpy(np.tile(np.float32(w.weights), (nq, 1))).to("cuda:0")
    torch.cuda.synchronize()

    # ---- build on the GPU (S0-S6), timed to stream sync with data resident
    bp = B.build_params(w.degree, nd_rounds=args.rounds, prune_mode=args.prune_mode)
    t0 = time.time()
    ix = B.Index.build(docs, bp)
    torch.cuda.synchronize()
    build_s = time.time() - t0
    bt = ix.build_timings()
    refine_sims = ix.build_counters()["refine_similarities"]
    log(f"[bench] {name} build {build_s:.2f}s stages {bt}")

    sp_nnz = float(w.docs.sp_indptr[-1]) / N
    tx_nnz = float(w.docs.tx_indptr[-1]) / N
    dense_bytes = w.docs.dim * (2 if bf16 else 4)
    bytes_per_dist = dense_bytes + 8.0 * sp_nnz + 8.0 * tx_nnz + 32.0   # rows + descriptor and offsets
    partial_bytes = bytes_per_dist - dense_bytes

    # what bounds each construction stage, against its own peak: the exact dense seed product (MFMA), the refinement
    # rounds (one full similarity per candidate: HBM), the neighbourhood phase (pair similarities per second)
    K = bp.knn_k
    seed_flops = float(ix.build_counters()["seed_flops"]) or 2.0 * N * N * w.docs.dim   # what the stage's MFMA products executed
    seed_tflops = seed_flops / max(bt["seed"], 1e-9) / 1e12
    refine_gbs = refine_sims * bytes_per_dist / max(bt["refine"], 1e-9) / 1e9
    build_roofline = dict(
        seed=dict(bound="mfma", achieved=round(seed_tflops, 1), peak=MFMA_PEAK_TFLOPS[bf16], unit="TFLOP/s",
                  frac=round(seed_tflops / MFMA_PEAK_TFLOPS[bf16], 4), flops=seed_flops,
                  full_product_flops=2.0 * N * N * w.docs.dim,
                  full_product_equivalent_TFLOPs=round(2.0 * N * N * w.docs.dim / max(bt["seed"], 1e-9) / 1e12, 1),
                  note="FLOPs the stage's dense products executed (sampled columns + sweep, padded tiles included; bf16 rows: only the "
                       "tiles on and above the diagonal of D D^T) over the whole stage's time (products, selections)"),
        refine=dict(bound="hbm", achieved=round(refine_gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s", frac=round(refine_gbs / HBM_PEAK_GBS, 4),
                    similarities=refine_sims, bytes_per_similarity=round(bytes_per_dist, 1),
                    similarities_per_s=round(refine_sims / max(bt["refine"], 1e-9), 1)),
        prune=dict(bound="alu", pair_similarities=N * K * (K - 1) // 2,
                   pair_similarities_per_s=round(N * K * (K - 1) / 2 / max(bt["prune"], 1e-9), 1),
                   note="dense Gram (MFMA) + list merges + detour sort + prune walk; one pair = both sparse parts merged"))

    # ---- ground truth: exact hybrid top-k under the same weights
    t0 = time.time()
    gt, _ = ix.bruteforce_topk(qs, k, wq)
    torch.cuda.synchronize()
    gt_s = time.time() - t0
    gt = gt.cpu().numpy()
    log(f"[bench] {name} exhaustive top-{k} of {nq} queries: {gt_s:.2f}s")

    gq = graph_quality_leg(w, docs, ix, bp, args.rounds, graph_nodes, bf16) if graph_nodes > 0 else None
    if gq:
        log(f"[bench] {name} graph quality: {gq}")

    # ---- sweep: the nominal beam, then upward until the recall target
    settings = [(args.beam, args.width)] if args.beam else parse_sweep(sweep_text)
    if not args.beam and (w.beam, 1) not in settings:
        settings = sorted(set(settings) | {(w.beam, 1)})
    sweep = []
    chosen = None
    for beam, width in settings:
        ix.search_batch(qs, k, beam, wq, search_width=width)
        torch.cuda.synchronize()
        t1 = time.time()
        ids, _ = ix.search_batch(qs, k, beam, wq, search_width=width)
        torch.cuda.synchronize()
        dt = time.time() - t1
        rec = recall_at_k(ids.cpu().numpy(), gt)
        counts, kms = ix.search_stats(nq)
        nd = int(counts[:, 0].sum().item())
        nsk = int(counts[:, 2].sum().item())
        sweep.append(dict(beam=beam, width=width, recall=round(rec, 4), qps=round(nq / dt, 1), kernel_ms=round(kms, 3),
                          dists_per_query=round(nd / nq, 1), dense_skipped_frac=round(nsk / max(nd, 1), 3)))
        log(f"[bench] {name} beam {beam} width {width}: recall@{k} {rec:.4f}  {nq / dt:,.0f} qps  kernel {kms:.2f} ms  {nd / nq:.0f} dists/query "
            f"({100.0 * nsk / max(nd, 1):.1f}% without the dense row)")
        if chosen is None and rec >= args.target_recall:
            chosen = (beam, width)
        if chosen is not None and beam >= w.beam:
            break
    reached = chosen is not None
    if chosen is None:
        chosen = settings[-1]
    beam, width = chosen

    # ---- timed region: exactly `steps` searches at the chosen setting
    out = (torch.empty((nq, k), dtype=torch.int32, device="cuda:0"), torch.empty((nq, k), dtype=torch.float32, device="cuda:0"))
    for _ in range(warmup):
        ix.search_batch(qs, k, beam, wq, out=out, search_width=width)
    torch.cuda.synchronize()
    kernel_ms = []
    t1 = time.time()
    for _ in range(steps):
        ix.search_batch(qs, k, beam, wq, out=out, search_width=width)
        kernel_ms.append(ix.search_kernel_ms())   # events recorded around the kernel on its own stream
    torch.cuda.synchronize()
    elapsed = time.time() - t1
    ms_per_step = elapsed * 1e3 / steps
    qps = nq * steps / elapsed
    rec = recall_at_k(out[0].cpu().numpy(), gt)
    counts, _ = ix.search_stats(nq)
    counts = counts.cpu().numpy().astype(np.int64)
    n_dist, n_iter, n_skip = int(counts[:, 0].sum()), int(counts[:, 1].sum()), int(counts[:, 2].sum())

    # ---- roofline of the search kernel: algorithmic bytes / measured kernel time.  Units per launch: full similarities
    # (descriptor + lists + dense row), partial ones (the candidate provably cannot enter the pool: no dense row), and
    # one adjacency row per iteration (at least one parent is expanded in every iteration).
    bytes_per_launch = (n_dist - n_skip) * bytes_per_dist + n_skip * partial_bytes + n_iter * w.degree * 4.0
    bytes_if_all_full = n_dist * bytes_per_dist + n_iter * w.degree * 4.0
    k_ms = float(np.mean(kernel_ms))
    achieved = bytes_per_launch / (k_ms * 1e-3) / 1e9
    traffic = None
    tfile = os.path.join(ROOT, "profiles", f"k_search_{name}_beam{beam}_w{width}_traffic.json")
    if os.path.exists(tfile) and N == cfg["n"] and nq == cfg["nq"]:
        t = json.load(open(tfile))     # HBM-side bytes per launch from the committed rocprofv3 --pmc summary of this same configuration
        traffic = round(t["fetch_bytes_per_launch"] + t["write_bytes_per_launch"])
    roofline = dict(bound="hbm", kernel="k_search", achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4), traffic=traffic, kernel_ms=round(k_ms, 3),
                    bytes_per_full_similarity=round(bytes_per_dist, 1), bytes_per_partial_similarity=round(partial_bytes, 1),
                    similarities_per_launch=n_dist, partial_similarities_per_launch=n_skip,
                    algorithmic_bytes_per_launch=round(bytes_per_launch),
                    GBps_if_every_similarity_were_full=round(bytes_if_all_full / (k_ms * 1e-3) / 1e9, 1),
                    dists_per_s=round(n_dist / (k_ms * 1e-3), 1),
                    traffic_GBps=None if traffic is None else round(traffic / (k_ms * 1e-3) / 1e9, 1),
                    frac_of_traffic=None if traffic is None else round(traffic / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))

    res = dict(workload=name, N=N, nq=nq, k=k, beam=beam, width=width, reached=reached, recall=rec, qps=qps, ms_per_step=ms_per_step,
               build_s=build_s, build_stages=bt, build_roofline=build_roofline, gt_s=gt_s, graph_quality=gq, sweep=sweep,
               roofline=roofline, bf16=bf16, sp_nnz=sp_nnz, tx_nnz=tx_nnz, exhaustive_qps=round(nq / gt_s, 1))
    for leg in extra_legs:
        if leg == "keywords":
            res["keyword_search"] = keyword_leg(args, w, ix, qs, wq, k, beam)
        elif leg == "insert":
            res["insertion"] = insert_leg(args, w, bp, docs, qs, wq, k, gt, sweep, build_s, bf16)
        elif leg == "weights":
            res["dynamic_fusion"] = weights_leg(args, ix, qs, k)
        elif leg == "entities":
            res["entity_search"] = entities_leg(args, w, ix, qs, wq, k)

    # ---- CPU baseline: the oracle as it stands, one thread, bounded samples of the same work
    if cpu_seconds > 0:
        import oracle as O
        sem, _, _, ent = [t.cpu().numpy() for t in ix.export_graph()]
        D = O.encode_docs(w.docs)
        Q = O.VS(w.queries)
        t2 = time.time()
        O.search(D, sem, ent, Q, 0, w.weights, k, beam, 0, width)
        per_q = max(time.time() - t2, 1e-4)
        sample = int(max(2, min(nq, 0.5 * cpu_seconds / per_q)))   # the search leg takes half the budget, the construction leg the rest and a little more
        t2 = time.time()
        oi, _, nv = O.search_batch(D, sem, ent, Q, range(sample), w.weights, k, beam, 0, width)
        dt = time.time() - t2
        agree = recall_at_k(out[0].cpu().numpy()[:sample], oi)
        cpu = dict(value=round(sample / dt, 3), unit="queries/s", cores=1, kind="oracle",
                   sample=f"first {sample} of {nq} queries of {name}, beam {beam}, {width} parent(s) per iteration, same GPU-built graph; "
                          f"{int(nv.sum())} hybrid similarities in {dt:.1f}s; top-{k} overlap with GPU {agree:.3f}",
                   hybrid_dists_per_s=round(float(nv.sum()) / dt, 1))
        log(f"[bench] {name} oracle: {sample} queries in {dt:.1f}s = {sample / dt:.2f} qps on 1 core ({os.cpu_count()} visible)")
        # construction: the oracle's refinement round and prune stage on sampled nodes (time-boxed), scaled to the corpus
        P = bp.sp_len or -(-w.degree // 6)
        knn_gpu, _ = [t.cpu().numpy() for t in ix.stage_seed_knn(K)]
        e_i, e_s = O.empty_sp(N, P)
        wv = np.float32([1, 1, 1])
        nodes = np.linspace(0, N - 1, 1000).astype(np.int64)
        done, t_ref, t_pr, box = 0, 0.0, 0.0, max(2.0, 1.5 * cpu_seconds)   # all 1000 sampled nodes on the headline workload (about 28 s)
        while done < len(nodes) and (t_ref + t_pr < box or done < 100):
            part = nodes[done:done + 25]
            t2 = time.time()
            r_ids, r_sc, _, _ = O.refine_round(D, wv, K, bp.nd_sample, P, knn_gpu, e_i, e_s, node_ids=part)
            t_ref += time.time() - t2
            t2 = time.time()
            for x, u in enumerate(part):
                O.prune_node(D, int(u), wv, w.degree, w.degree // 2, r_ids[x], r_sc[x])
            t_pr += time.time() - t2
            done += len(part)
        est = N * (args.rounds * t_ref + t_pr) / done
        cpu["build_extrapolated_s"] = round(est, 1)
        cpu["build_sample"] = (f"{done} nodes: one refinement round {t_ref / done:.4f}s/node, neighbourhood similarities + prune "
                               f"{t_pr / done:.4f}s/node; x {N} nodes, {args.rounds} rounds, seed stage not counted (extrapolation)")
        log(f"[bench] {name} oracle build, extrapolated from {done} nodes: {est:,.0f}s on 1 core (GPU {build_s:.2f}s)")
        res["cpu_baseline"] = cpu
    else:
        res["cpu_baseline"] = None
    ix.close()
    del docs, qs, wq
    torch.cuda.empty_cache()
    return res


def describe(res, weights):
    return (f"{res['workload']}: N={res['N']} docs, dense d={res['dim']} {'bf16' if res['bf16'] else 'f32'}, "
            f"sparse ~{res['sp_nnz']:.0f} nnz/doc, text ~{res['tx_nnz']:.0f} distinct terms/doc, {res['nq']} queries, "
            f"weights {weights}, degree {res['degree']}, k={res['k']}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg3", help="cfg3 (default), cfg2, tiny, cfg5")
    ap.add_argument("--n", type=int, default=None, help="override the number of documents (smaller rehearsal)")
    ap.add_argument("--nq", type=int, default=None)
    ap.add_argument("--rounds", type=int, default=3)
    ap.add_argument("--beams", default=None, help="sweep settings 'beam[:width],...' (default: per workload)")
    ap.add_argument("--weight-sweep", action="store_true",
                    help="also search the same index under five other weight settings (dynamic fusion, no rebuild)")
    ap.add_argument("--weight-beams", default="128,512,1024,1536,2048,2304,2560,2816,3072,3584,4096,4608,5120,5632,6144,8192,12288,16384")
    ap.add_argument("--beam", type=int, default=0, help="fix the beam (skips the sweep; for profiling runs)")
    ap.add_argument("--width", type=int, default=1, help="parents per iteration with --beam")
    ap.add_argument("--target-recall", type=float, default=0.95)
    ap.add_argument("--prune-mode", type=int, default=0,
                    help="0 = joint RNG-IP pruning (the method), 1 = RNG only, 2 = IP only (the paper's pruning ablation)")
    ap.add_argument("--insert", type=float, default=0.0,
                    help="also measure insertion: build on the first (1-f) of the corpus, insert the last f "
                         "(e.g. 0.2), report seconds next to the rebuild and recall/QPS of the updated index")
    ap.add_argument("--keywords", action="store_true",
                    help="also measure the keyword-constrained search (1-2 required terms per query, with and "
                         "without keyword edges) and add a keyword_search object to the line")
    ap.add_argument("--entities", action="store_true",
                    help="also time the search with entities (Section 4.2.3) on a synthetic entity graph over the corpus")
    ap.add_argument("--no-cfg2", action="store_true", help="skip the brief config-2 leg that precedes a larger headline workload")
    ap.add_argument("--graph-nodes", type=int, default=500, help="nodes sampled for the graph-quality figures (0 = skip)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="budget of the oracle's search timing leg")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2511_00855_amd import binding as B
    from paper_2511_00855_amd.synth import CONFIGS

    os.environ.setdefault("ALLANPOE_PROGRESS", "1")   # a build of millions of documents reports on stderr as it goes
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()   # fail loudly if the HIP library is not built

    # ---- a plain 1 GiB copy: what this machine streams (read + write), and the yardstick of the profiler's byte counters
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
    b = torch.empty_like(a)
    B.calibration_copy(b, a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(2):
        B.calibration_copy(b, a)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * 2.0 * a.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    log(f"[bench] streaming copy of 1 GiB: {copy_gbs:,.0f} GB/s (read + write)")
    del a, b

    legs = [x for x, on in (("keywords", args.keywords), ("insert", args.insert > 0), ("weights", args.weight_sweep),
                                ("entities", args.entities)) if on]
    side = None
    if args.workload in ("cfg3", "cfg5") and not args.no_cfg2 and not args.beam:
        # config 2 first, briefly: its own sweep to the recall target and a short timed run
        side = run_workload(args, "cfg2", n=None, nq=None, steps=3, warmup=1, sweep_text=SWEEPS["cfg2"],
                            cpu_seconds=0.0 if args.no_cpu_baseline else 5.0, graph_nodes=args.graph_nodes, extra_legs=[])
    main_res = run_workload(args, args.workload, n=args.n, nq=args.nq, steps=args.steps, warmup=args.warmup,
                            sweep_text=args.beams or SWEEPS[args.workload],
                            cpu_seconds=0.0 if args.no_cpu_baseline else args.cpu_seconds, graph_nodes=args.graph_nodes,
                            extra_legs=legs)

    def pack(res):
        cfg = CONFIGS[res["workload"]]
        res["dim"], res["degree"] = cfg["dim"], cfg["degree"]
        rf = dict(res["roofline"])
        rf["streaming_copy_GBps"] = round(copy_gbs, 1)
        rf["frac_of_streaming_copy"] = round(rf["achieved"] / copy_gbs, 4)
        return dict(
            value=round(res["qps"], 1), ms_per_step=round(res["ms_per_step"], 3),
            config={"workload": describe(res, tuple(cfg["weights"])), "beam": res["beam"], "search_width": res["width"],
                    "recall_at_10": round(res["recall"], 4), "recall_target_reached": res["reached"],
                    "nominal_beam": cfg["beam"], "refine_rounds": args.rounds,
                    "pruning": ("joint RNG-IP", "RNG only", "IP only")[args.prune_mode]},
            build_s=round(res["build_s"], 3), build_stages_s={x: round(y, 3) for x, y in res["build_stages"].items()},
            build_roofline=res["build_roofline"], graph_quality=res["graph_quality"],
            exhaustive_scan_qps=res["exhaustive_qps"], hybrid_dists_per_s=rf["dists_per_s"], beam_sweep=res["sweep"],
            roofline=rf, cpu_baseline=res["cpu_baseline"])

    m = pack(main_res)
    line = {
        "metric": "hybrid-search QPS at recall@10=0.95", "value": m["value"], "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": m["ms_per_step"],
        "higher_is_better": True, "vs_baseline": None,
        "dtype": "bf16-storage/f32-accumulate" if main_res["bf16"] else "f32", "data": "synthetic",
    }
    line.update({x: y for x, y in m.items() if x not in ("value", "ms_per_step")})
    for extra in ("keyword_search", "insertion", "dynamic_fusion", "entity_search"):
        if extra in main_res:
            line[extra] = main_res[extra]
    if side is not None:
        s = pack(side)
        s["steps"], s["warmup"] = 3, 1
        s["dtype"] = "f32"
        line["cfg2"] = s
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
