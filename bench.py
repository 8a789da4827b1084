#!/usr/bin/env python3
"""Benchmark of the hybrid-index hot path on one MI355X.

One "step" = one batched search (S7-S9) of all queries of the workload on an
index that this same run built on the GPU (S0-S6; build time reported beside
it).  The headline value is queries per second at the smallest beam whose
recall@10 against exact hybrid top-10 reaches 0.95.  Inputs are seeded
synthetic data resident in HBM before the timed region.  Prints ONE JSON line.
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

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E data-sheet peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def recall_at_k(ids, gt):
    import numpy as np
    return float(np.mean([len(set(a.tolist()) & set(b.tolist())) / float(len(b)) for a, b in zip(ids, gt)]))


def keyword_leg(args, w, ix, qs, wq, k, chosen):
    """Keyword-constrained search (Section 4.2.2): every query requires 1-2 of its own text tokens.  Ground truth
    = exact top-k among the documents holding a required term, on up to 1000 sampled queries (exhaustive scores
    from ap_hybrid_scores, filter and top-k in torch: measurement only)."""
    import numpy as np
    import scipy.sparse as sps
    import torch
    from paper_2511_00855_amd import binding as B
    from paper_2511_00855_amd.synth import make_keywords, subset_vecset
    nq, n = qs.n, w.docs.n
    kw = make_keywords(w.queries, seed=1, max_terms=2, stride=2)
    sample = np.arange(0, nq, max(1, nq // 1000))[:1000]
    inv = sps.csr_matrix((np.ones(len(w.docs.tx_idx), np.int8), w.docs.tx_idx, w.docs.tx_indptr),
                         shape=(n, w.docs.tx_vocab)).tocsc()
    gt = []
    for c0 in range(0, len(sample), 250):
        rows = sample[c0:c0 + 250]
        sub = B.DeviceVecs(subset_vecset(w.queries, rows), "cuda:0")
        allc = torch.arange(n, dtype=torch.int32, device="cuda:0").repeat(len(rows), 1)
        sc = ix.hybrid_scores(sub, allc, wq[torch.from_numpy(rows).to("cuda:0")])[:, :, 3]
        rr, cc = [], []
        for x, qi in enumerate(rows):
            for t in kw[qi][kw[qi] >= 0]:
                d = inv.indices[inv.indptr[t]:inv.indptr[t + 1]]
                rr.append(np.full(len(d), x, np.int64)); cc.append(d.astype(np.int64))
        mask = torch.zeros(sc.shape, dtype=torch.bool, device="cuda:0")
        mask[torch.from_numpy(np.concatenate(rr)).to("cuda:0"), torch.from_numpy(np.concatenate(cc)).to("cuda:0")] = True
        top = sc.masked_fill(~mask, float("-inf")).topk(k, dim=1)
        ids = torch.where(torch.isinf(top.values), torch.full_like(top.indices, -1), top.indices)
        gt.append(ids.cpu().numpy())
        del sc, mask, allc
    gt = np.concatenate(gt)
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
    updated index is searched at the beams of the main sweep, against the same ground truth as the rebuild."""
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
            beam = sw["beam"]
            new.search_batch(qs, k, beam, wq)
            torch.cuda.synchronize()
            t1 = time.time()
            ids, _ = new.search_batch(qs, k, beam, wq)
            torch.cuda.synchronize()
            qps = qs.n / (time.time() - t1)
            rows.append(dict(beam=beam, recall=round(recall_at_k(ids.cpu().numpy(), gt), 4), qps=round(qps, 1),
                             rebuilt_recall=sw["recall"], rebuilt_qps=sw["qps"]))
        out.append(dict(fraction=f, inserted=n - n0, seconds=round(dt, 3), rebuild_seconds=round(build_s, 3),
                        share_of_rebuild=round(dt / build_s, 3), stages_s={a: round(b, 3) for a, b in st.items()}, search=rows))
        log(f"[bench] insert {100 * f:.0f}% ({n - n0} docs): {dt:.3f}s = {100 * dt / build_s:.1f}% of the rebuild ({build_s:.2f}s); "
            + "; ".join(f"beam {r['beam']}: recall {r['recall']:.4f} (rebuilt {r['rebuilt_recall']:.4f})" for r in rows[:1] + rows[-1:]))
        new.close(); old.close()
        del old_docs
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg2", help="cfg2 (default), tiny, cfg3, cfg5")
    ap.add_argument("--n", type=int, default=None, help="override the number of documents (smaller rehearsal)")
    ap.add_argument("--nq", type=int, default=None)
    ap.add_argument("--rounds", type=int, default=3)
    ap.add_argument("--beams", default="128,256,512,1024,1536,2048,2112,2144,2176,2240,2304,2560,3072,4096,6144,8192,12288,16384")
    ap.add_argument("--weight-sweep", action="store_true",
                    help="also search the same index under five other weight settings (dynamic fusion, no rebuild)")
    ap.add_argument("--weight-beams", default="128,512,1024,1536,2048,2304,2560,2816,3072,3584,4096,4608,5120,5632,6144,8192,12288,16384")
    ap.add_argument("--beam", type=int, default=0, help="fix the beam (skips the sweep; for profiling runs)")
    ap.add_argument("--target-recall", type=float, default=0.95)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="kept for older command lines: the 1 GiB plain copy kernel (yardstick for profiler byte "
                         "counters and for the streaming rate of this box) always runs three times")
    ap.add_argument("--prune-mode", type=int, default=0,
                    help="0 = joint RNG-IP pruning (the method), 1 = RNG only, 2 = IP only (the paper's pruning ablation)")
    ap.add_argument("--insert", type=float, default=0.0,
                    help="also measure insertion: build on the first (1-f) of the corpus, insert the last f "
                         "(e.g. 0.2), report seconds next to the rebuild and recall/QPS of the updated index")
    ap.add_argument("--keywords", action="store_true",
                    help="also measure the keyword-constrained search (1-2 required terms per query, with and "
                         "without keyword edges) and add a keyword_search object to the line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the oracle timing leg")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_00855_amd import binding as B
    from paper_2511_00855_amd.synth import make_workload

    os.environ.setdefault("ALLANPOE_PROGRESS", "1")   # a build of millions of documents reports on stderr as it goes
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()   # fail loudly if the HIP library is not built

    t0 = time.time()
    w = make_workload(args.workload, seed=0, n=args.n, nq=args.nq, progress=lambda m: log(f"[bench] generating: {m}"))
    cfg = w.extra["config"]
    bf16 = bool(cfg["bf16"])
    log(f"[bench] workload {args.workload}: n={w.docs.n} nq={w.queries.n} dim={w.docs.dim} bf16={bf16} "
        f"generated in {time.time() - t0:.1f}s")
    docs = B.DeviceVecs(w.docs, "cuda:0", bf16=bf16)
    qs = B.DeviceVecs(w.queries, "cuda:0")
    nq, k = qs.n, w.k
    wq = torch.from_numpy(np.tile(np.float32(w.weights), (nq, 1))).to("cuda:0")
    torch.cuda.synchronize()

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

    # ---- build on the GPU (S0-S6), timed to stream sync with data resident
    bp = B.build_params(w.degree, nd_rounds=args.rounds, prune_mode=args.prune_mode)
    t0 = time.time()
    ix = B.Index.build(docs, bp)
    torch.cuda.synchronize()
    build_s = time.time() - t0
    bt = ix.build_timings()
    log(f"[bench] build {build_s:.2f}s stages {bt}")

    # ---- ground truth: exact hybrid top-k under the same weights
    t0 = time.time()
    gt, _ = ix.bruteforce_topk(qs, k, wq)
    torch.cuda.synchronize()
    gt = gt.cpu().numpy()
    log(f"[bench] exhaustive top-{k} of {nq} queries: {time.time() - t0:.2f}s")

    # ---- beam sweep: nominal beam, then upward until the recall target
    def run_once(beam):
        ids, sc = ix.search_batch(qs, k, beam, wq)
        return ids

    sweep = []
    chosen = None
    beams = [args.beam] if args.beam else sorted(set(int(b) for b in args.beams.split(",")) | {w.beam})
    for beam in beams:
        ids = run_once(beam)
        torch.cuda.synchronize()
        t1 = time.time()
        ids = run_once(beam)
        torch.cuda.synchronize()
        dt = time.time() - t1
        rec = recall_at_k(ids.cpu().numpy(), gt)
        counts, kms = ix.search_stats(nq)
        nd = int(counts[:, 0].sum().item())
        nsk = int(counts[:, 2].sum().item())
        sweep.append(dict(beam=beam, recall=round(rec, 4), qps=round(nq / dt, 1), kernel_ms=round(kms, 3),
                          dists_per_query=round(nd / nq, 1), dense_skipped_frac=round(nsk / max(nd, 1), 3)))
        log(f"[bench] beam {beam}: recall@{k} {rec:.4f}  {nq / dt:,.0f} qps  kernel {kms:.2f} ms  {nd / nq:.0f} dists/query "
            f"({100.0 * nsk / max(nd, 1):.1f}% without the dense row)")
        if chosen is None and rec >= args.target_recall:
            chosen = beam
        if chosen is not None and beam >= w.beam:
            break
    reached = chosen is not None
    if chosen is None:
        chosen = beams[-1]

    # ---- timed region: exactly `steps` searches at the chosen beam
    out = (torch.empty((nq, k), dtype=torch.int32, device="cuda:0"), torch.empty((nq, k), dtype=torch.float32, device="cuda:0"))
    for _ in range(args.warmup):
        ix.search_batch(qs, k, chosen, wq, out=out)
    torch.cuda.synchronize()
    kernel_ms = []
    t1 = time.time()
    for _ in range(args.steps):
        ix.search_batch(qs, k, chosen, wq, out=out)
        kernel_ms.append(ix.search_kernel_ms())   # events recorded around the kernel on its own stream
    torch.cuda.synchronize()
    elapsed = time.time() - t1
    ms_per_step = elapsed * 1e3 / args.steps
    qps = nq * args.steps / elapsed
    rec = recall_at_k(out[0].cpu().numpy(), gt)
    counts, _ = ix.search_stats(nq)
    counts = counts.cpu().numpy().astype(np.int64)
    n_dist, n_iter, n_skip = int(counts[:, 0].sum()), int(counts[:, 1].sum()), int(counts[:, 2].sum())

    # ---- roofline of the search kernel: algorithmic bytes / measured kernel time
    sp_nnz = float(w.docs.sp_indptr[-1]) / w.docs.n
    tx_nnz = float(w.docs.tx_indptr[-1]) / w.docs.n
    dense_bytes = w.docs.dim * (2 if bf16 else 4)
    bytes_per_dist = dense_bytes + 8.0 * sp_nnz + 8.0 * tx_nnz + 32.0   # rows + 4 offsets
    # algorithmic bytes per launch = units x per-unit figure, for the two kinds of unit the kernel counts:
    #   a full similarity (descriptor + lists + dense row) and a partial one (the candidate provably cannot
    #   enter the pool, so its dense row is not needed: descriptor + lists only), plus the edge rows.
    partial_bytes = bytes_per_dist - dense_bytes
    bytes_per_launch = (n_dist - n_skip) * bytes_per_dist + n_skip * partial_bytes + n_iter * w.degree * 4.0
    bytes_if_all_full = n_dist * bytes_per_dist + n_iter * w.degree * 4.0
    k_ms = float(np.mean(kernel_ms))
    achieved = bytes_per_launch / (k_ms * 1e-3) / 1e9
    traffic = None
    tfile = os.path.join(ROOT, "profiles", f"k_search_{args.workload}_beam{chosen}_traffic.json")
    if os.path.exists(tfile):      # HBM-side bytes per launch from the committed rocprofv3 --pmc summary of this same configuration
        t = json.load(open(tfile))
        traffic = round(t["fetch_bytes_per_launch"] + t["write_bytes_per_launch"])
    roofline = dict(bound="hbm", kernel="k_search", achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4), traffic=traffic, kernel_ms=round(k_ms, 3),
                    bytes_per_full_similarity=round(bytes_per_dist, 1), bytes_per_partial_similarity=round(partial_bytes, 1),
                    similarities_per_launch=n_dist, partial_similarities_per_launch=n_skip,
                    algorithmic_bytes_per_launch=round(bytes_per_launch),
                    GBps_if_every_similarity_were_full=round(bytes_if_all_full / (k_ms * 1e-3) / 1e9, 1),
                    dists_per_s=round(n_dist / (k_ms * 1e-3), 1),
                    streaming_copy_GBps=round(copy_gbs, 1),
                    traffic_GBps=None if traffic is None else round(traffic / (k_ms * 1e-3) / 1e9, 1))

    kw_report = keyword_leg(args, w, ix, qs, wq, k, chosen) if args.keywords else None
    ins_report = insert_leg(args, w, bp, docs, qs, wq, k, gt, sweep, build_s, bf16) if args.insert > 0 else None
    ws_report = weights_leg(args, ix, qs, k) if args.weight_sweep else None

    # ---- CPU baseline: the oracle as it stands, one thread, bounded sample of the same searches
    cpu = None
    if not args.no_cpu_baseline:
        import oracle as O
        sem, _, _, ent = [t.cpu().numpy() for t in ix.export_graph()]
        D = O.encode_docs(w.docs)
        Q = O.VS(w.queries)
        t2 = time.time()
        O.search(D, sem, ent, Q, 0, w.weights, k, chosen)
        per_q = max(time.time() - t2, 1e-4)
        sample = int(max(4, min(nq, args.cpu_seconds / per_q)))
        t2 = time.time()
        oi, _, nv = O.search_batch(D, sem, ent, Q, range(sample), w.weights, k, chosen)
        dt = time.time() - t2
        agree = recall_at_k(out[0].cpu().numpy()[:sample], oi)
        cpu = dict(value=round(sample / dt, 2), unit="queries/s", cores=1, kind="oracle",
                   sample=f"first {sample} of {nq} queries, beam {chosen}, same GPU-built graph; "
                          f"{int(nv.sum())} hybrid similarities in {dt:.1f}s; top-{k} overlap with GPU {agree:.3f}",
                   hybrid_dists_per_s=round(float(nv.sum()) / dt, 1))
        log(f"[bench] oracle: {sample} queries in {dt:.1f}s = {sample / dt:.1f} qps on 1 core ({os.cpu_count()} visible)")
        # construction: the oracle's refinement round and prune stage on a few nodes, extrapolated to the corpus
        nodes = np.linspace(0, w.docs.n - 1, 6).astype(np.int64)
        K, P = bp.knn_k, bp.sp_len or -(-w.degree // 6)
        knn_gpu, knn_sc_gpu = [t.cpu().numpy() for t in ix.stage_seed_knn(K)]
        e_i, e_s = O.empty_sp(w.docs.n, P)
        wv = np.float32([1, 1, 1])
        t2 = time.time()
        r_ids, r_sc, _, _ = O.refine_round(D, wv, K, bp.nd_sample, P, knn_gpu, e_i, e_s, node_ids=nodes)
        t_ref = (time.time() - t2) / len(nodes)
        t2 = time.time()
        for x, u in enumerate(nodes):
            O.prune_node(D, int(u), wv, w.degree, w.degree // 2, r_ids[x], r_sc[x])
        t_pr = (time.time() - t2) / len(nodes)
        est = w.docs.n * (args.rounds * t_ref + t_pr)
        cpu["build_extrapolated_s"] = round(est, 1)
        cpu["build_sample"] = (f"{len(nodes)} nodes: one refinement round {t_ref:.3f}s/node, neighbourhood similarities + prune "
                               f"{t_pr:.3f}s/node; x {w.docs.n} nodes, {args.rounds} rounds, seed stage not counted (extrapolation)")
        log(f"[bench] oracle build, extrapolated from {len(nodes)} nodes: {est:,.0f}s on 1 core (GPU {build_s:.2f}s)")

    line = {
        "metric": "hybrid-search QPS at recall@10=0.95", "value": round(qps, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16-storage/f32-accumulate" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: N={w.docs.n} docs, dense d={w.docs.dim} {'bf16' if bf16 else 'f32'}, "
                               f"sparse ~{sp_nnz:.0f} nnz/doc, text ~{tx_nnz:.0f} distinct terms/doc, {nq} queries, "
                               f"weights {tuple(w.weights)}, degree {w.degree}, k={k}",
                   "beam": chosen, "recall_at_10": round(rec, 4), "recall_target_reached": reached,
                   "nominal_beam": w.beam, "refine_rounds": args.rounds,
                   "pruning": ("joint RNG-IP", "RNG only", "IP only")[args.prune_mode]},
        "build_s": round(build_s, 3), "build_stages_s": {a: round(b, 3) for a, b in bt.items()},
        "hybrid_dists_per_s": roofline["dists_per_s"], "beam_sweep": sweep,
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if kw_report is not None:
        line["keyword_search"] = kw_report
    if ins_report is not None:
        line["insertion"] = ins_report
    if ws_report is not None:
        line["dynamic_fusion"] = ws_report
    print(json.dumps(line), flush=True)
    ix.close()


if __name__ == "__main__":
    main()
