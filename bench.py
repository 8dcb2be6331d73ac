#!/usr/bin/env python3
"""Throughput benchmark of the label-filtered search hot path on one MI355X.

One "step" = one vf_search call over the whole query batch of the workload
(route + IVF-BFS scan + IVF-Graph beam search + AND predicate + finalise), with the
index, the queries and the outputs already resident in HBM.  The default workload is
the SIFT-1M-like configuration the metric is quoted on: N = 1e6 float32 vectors of
dim 128, 1,000 Zipf labels, T = 10,000, graph degree 32, 10,000 single-label
queries, k = 10 (a seeded synthetic stand-in for the paper's dataset).

Prints ONE JSON line.  `value` is queries/s at the fastest setting of a grid of
(itopk, width, iters, n_seeds) whose recall@10, measured in this run against exact
filtered ground truth, is >= 0.90; the >= 0.99 operating point is reported beside it.
`roofline` prices the kernel with the longest launches in the timed region against
the roof that bounds it, from the algorithmic bytes / flops its work counters imply and
its duration from HIP events; `cpu_baseline` times the CPU oracle on a bounded sample
of the same queries.  --latency, --multi, --sweep, --workload c3|c5 add further
measurements to `config`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X fp32 vector, published (256 CUs x 2.4 GHz x 256 flop/clk)
SCAN_KERNELS = ("scan_topk_kernel", "scan_topk16_kernel", "scan_valu_kernel", "scan_bf16_kernel")   # vf_profile.scan_kernel

# (itopk, width, iters, n_seeds) settings tried, cheapest first within each group.  Recall on this
# workload is governed by the number of seeds (per-list graphs over separated clusters are
# disconnected), then by the iteration count.
CANDIDATES = sorted({(itopk, 1, iters, ns)
                     for itopk in (32,)
                     for iters in (6, 8, 12, 16, 24, 32)
                     for ns in (1536, 2048, 2560, 3072, 4096, 5120, 6144, 8192, 12288)}
                    | {(32, wd, iters, ns) for wd, its in ((2, (4, 6, 12, 16)), (4, (3, 8, 12))) for iters in its
                       for ns in (2560, 3072, 4096, 6144, 8192)}
                    | {(64, 1, 24, 8192), (64, 2, 24, 8192), (128, 2, 32, 12288)},
                    key=lambda c: (c[3] + c[2] * c[1] * 32) * (1.0 + c[0] / 256.0))


def committed_traffic(kernel, workload, params):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled), if it was taken at these parameters; else None."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}.txt")
    try:
        text = open(path).read()
    except OSError:
        return None
    want = "params = " + repr(dict(zip(("itopk", "width", "iters", "n_seeds"), params)))
    if want not in text:
        return None
    import re
    vals = re.findall(kernel + r", \d+ timed-region launches: raw [0-9.]+ -> ([0-9.]+) GB per launch", text)
    if len(vals) != 2:
        return None
    return int(round((float(vals[0]) + float(vals[1])) * 1e9))


def committed_params(workload):
    """(itopk, width, iters, n_seeds) the committed counter summary was taken at, or None."""
    import re
    try:
        text = open(os.path.join(ROOT, "profiles", f"bench_{workload}.txt")).read()
    except OSError:
        return None
    m = re.search(r"params = \{'itopk': (\d+), 'width': (\d+), 'iters': (\d+), 'n_seeds': (\d+)\}", text)
    return tuple(int(g) for g in m.groups()) if m else None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def recall_at_k(found, truth):
    """Eq. (1) of the paper with |GT| in the denominator when fewer than K vectors match."""
    num = den = 0
    for f, t in zip(found, truth):
        t = t[t >= 0]
        if len(t) == 0:
            continue
        num += np.isin(f[f >= 0], t).sum()
        den += len(t)
    return float(num) / max(den, 1)


def time_search(vf, ix, Q, qoff, qids, k, params, steps, warmup, out_ids, out_dists):
    import torch
    itopk, width, iters, n_seeds = params
    for _ in range(warmup):
        vf.search(ix, Q, qoff, qids, k, itopk, width, iters, n_seeds, out_ids, out_dists)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        vf.search(ix, Q, qoff, qids, k, itopk, width, iters, n_seeds, out_ids, out_dists)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--n", type=int, default=None, help="override the number of vectors (testing only)")
    ap.add_argument("--nq", type=int, default=None)
    ap.add_argument("--T", type=int, default=None)
    ap.add_argument("--sweep", action="store_true", help="print recall/QPS of every candidate setting to stderr")
    ap.add_argument("--graph", choices=("knn", "pruned"), default="knn",
                    help="per-list graphs: exact kNN (the configuration the oracle baseline can follow at full size) "
                         "or degree-2R kNN reduced by rank-based pruning and reverse edges (implies --no-cpu)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-sample", type=int, default=1024)
    ap.add_argument("--params", default=None,
                    help="itopk,width,iters,n_seeds of the point to time (default: the fastest grid point with recall >= 0.90)")
    ap.add_argument("--gt-sample", type=int, default=0,
                    help="measure recall on this many randomly chosen queries (ground truth of the full set "
                         "of a 10M-vector workload would take many minutes)")
    ap.add_argument("--compare-graphs", action="store_true",
                    help="also build the index with exact kNN and with pruned graphs and report recall by list size")
    ap.add_argument("--multi", action="store_true",
                    help="also measure two-label AND (greedy and parallel policy) and OR queries on the same index")
    ap.add_argument("--latency", action="store_true",
                    help="also measure small-batch latency (batches of 1, 8 and 64 queries, half graph / half scan labels)")
    ap.add_argument("--and-scan-limit", type=int, default=0,
                    help="selectivity-aware routing (vf_search_ex): AND queries whose smallest list is a graph list of at "
                         "most this many vectors are answered by the exact predicate scan of that list; 0 = the paper's routing")
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE",
                    help="set an experiment switch of the library (vf_tune) before the index is built; repeatable")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run three 1 GiB device-to-device copies (scale reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_00812_amd import binding as vf
    from paper_2506_00812_amd.workloads import make_workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    vf.load_library()
    if args.and_scan_limit:
        # every vf.search call of this run goes through vf_search_ex with the limit (single-label queries and AND
        # queries on long lists are routed as before)
        plain_search = vf.search
        vf.search = lambda *a, **kw: plain_search(*a, and_scan_limit=args.and_scan_limit, **kw)

    t0 = time.time()
    log(f"[bench] generating workload {args.workload} ...")
    w = make_workload(args.workload, n=args.n, nq=args.nq, T=args.T)
    s = w.spec
    log(f"[bench] workload {s.name}: n={s.n} dim={s.dim} {s.dtype} labels={s.n_labels} T={s.T} R={s.graph_degree} "
        f"nq={s.nq} generated in {time.time() - t0:.1f}s")
    X = torch.from_numpy(w.vectors).cuda()
    Q = torch.from_numpy(w.queries).cuda()
    for kv in args.tune:
        name, _, value = kv.partition("=")
        vf.tune_defaults(name.strip(), float(value))
        log(f"[bench] switch {name.strip()} = {float(value):g}")
    t0 = time.time()
    log("[bench] building the index ...")
    pruned = args.graph == "pruned"
    if pruned:
        args.no_cpu = True   # the oracle cannot build whole pruned graphs of this size in bounded time
    ix = vf.build_index(X, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree,
                        graph_kind=vf.GRAPH_PRUNED if pruned else vf.GRAPH_KNN)
    torch.cuda.synchronize()
    build_s = time.time() - t0
    st = ix.stats()
    log(f"[bench] index built in {build_s:.1f}s: {st['n_graph_labels']} graph labels ({st['n_HS']} postings), "
        f"{st['n_scan_labels']} scan labels ({st['n_LS']} postings), {st['bytes_total'] / 2**20:.0f} MiB")

    k = s.k
    out_ids = torch.empty((s.nq, k), dtype=torch.int64, device="cuda")
    out_dists = torch.empty((s.nq, k), dtype=torch.float32, device="cuda")
    # untimed: a burst of back-to-back calls.  The first time several calls are in flight the HIP
    # runtime grows its pools (a 5 ms stall, once per process); that belongs to start-up, not to a step.
    for _ in range(12):
        vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, k, 32, 1, 4, 256, out_ids, out_dists)
    torch.cuda.synchronize()
    t0 = time.time()
    ix.profile_enable(True)
    gt_rows = None        # recall is measured on these query rows (all of them unless --gt-sample)
    if args.gt_sample and args.gt_sample < s.nq:
        gt_rows = np.sort(np.random.default_rng(97531).choice(s.nq, size=args.gt_sample, replace=False))
        cnt = np.diff(w.qlabel_offsets)[gt_rows]
        sub_off = np.zeros(len(gt_rows) + 1, dtype=np.int64)
        np.cumsum(cnt, out=sub_off[1:])
        sub_ids = np.concatenate([w.qlabel_ids[w.qlabel_offsets[j]:w.qlabel_offsets[j + 1]] for j in gt_rows])
        gt_ids, _ = vf.search_exact(ix, Q[torch.from_numpy(gt_rows).cuda()].contiguous(), sub_off, sub_ids, k)
    else:
        gt_ids, _ = vf.search_exact(ix, Q, w.qlabel_offsets, w.qlabel_ids, k)
    gt = gt_ids.cpu().numpy()
    pfe = ix.profile_read()
    ix.profile_enable(False)

    def recall_of(found):
        return recall_at_k(found if gt_rows is None else found[gt_rows], gt)
    # the dense invocations of the contraction kernel: ground truth (hundreds of queries share the
    # popular lists) and the per-list kNN self-joins of the index build (every vertex is a query)
    flops_per_pair = 2 * s.dim
    S_all = ix.export("S").astype(np.float64)
    knn_flops = float((S_all[S_all >= s.T] ** 2).sum()) * flops_per_pair
    mfma_peak = FP32_VECTOR_PEAK_TFLOPS if s.dtype == "float32" else 5000.0
    dense = {
        "unit": "TFLOP/s" if s.dtype == "float32" else "TOP/s", "peak": mfma_peak,
        "ground_truth": {"pairs": int(pfe["scan_pairs"]), "ms": round(pfe["scan_ms"], 3),
                         "achieved": round(pfe["scan_pairs"] * flops_per_pair / (pfe["scan_ms"] * 1e-3) / 1e12, 1)},
        "index_build_knn": {"pairs": int(knn_flops / flops_per_pair), "s": round(build_s, 3),
                            "achieved_lower_bound": round(knn_flops / build_s / 1e12, 1),
                            "note": "whole vf_build_index call, host work included"},
    }
    dense["ground_truth"]["frac"] = round(dense["ground_truth"]["achieved"] / mfma_peak, 4)
    dense["index_build_knn"]["frac"] = round(dense["index_build_knn"]["achieved_lower_bound"] / mfma_peak, 4)
    log(f"[bench] exact filtered ground truth in {time.time() - t0:.1f}s")


    # strata of the batch: single label / AND, graph-routed / scan-routed (on the rows recall is measured on)
    rows = np.arange(s.nq) if gt_rows is None else gt_rows
    S_host = ix.export("S")
    nlab = np.diff(w.qlabel_offsets)[rows]
    smallest = np.array([S_host[w.qlabel_ids[w.qlabel_offsets[j]:w.qlabel_offsets[j + 1]]].min() for j in rows])
    strata_masks = {name: mask for name, mask in (("single_graph", (nlab == 1) & (smallest >= s.T)),
                                                  ("single_scan", (nlab == 1) & (smallest < s.T)),
                                                  ("and_graph", (nlab > 1) & (smallest >= s.T)),
                                                  ("and_scan", (nlab > 1) & (smallest < s.T))) if mask.any()}

    def strata_recall(found):
        return {name: recall_at_k(found[rows[mask]], gt[mask]) for name, mask in strata_masks.items()}

    # ---- pick the operating points: cheapest candidates reaching recall 0.90 and 0.99
    table = []
    worst_stratum = {}
    cands = CANDIDATES
    if s.n > 2_000_000:   # long lists need more seeds: a coarser grid reaching further
        cands = sorted({(itopk, 1, iters, ns) for itopk in (32, 64) for iters in (8, 16, 32)
                        for ns in (2048, 4096, 8192, 16384, 32768)}, key=lambda c: c[3] + c[2] * 32)
    if pruned:   # pruned graphs are connected far better: a fraction of the seeds suffices
        cands = sorted({(32, wd, iters, ns) for wd in (1, 2) for iters in (3, 4, 6, 8, 12, 16, 24)
                        for ns in (64, 128, 256, 384, 512, 768, 1024, 1536, 2048, 4096)},
                       key=lambda c: c[3] + c[2] * c[1] * 32)
        if s.n > 2_000_000:
            cands = sorted({(itopk, 1, iters, ns) for itopk in (32, 64) for iters in (8, 16, 32)
                            for ns in (256, 512, 1024, 2048, 4096, 8192)}, key=lambda c: c[3] + c[2] * 32)
    for params in cands:
        if params[1] * s.graph_degree > 128:
            continue
        ms = time_search(vf, ix, Q, w.qlabel_offsets, w.qlabel_ids, k, params, 10 if s.nq <= 20000 else 3, 2, out_ids, out_dists)
        found = out_ids.cpu().numpy()
        rec = recall_of(found)
        table.append((params, rec, s.nq / ms * 1e3))
        worst_stratum[params] = min(strata_recall(found).values())
        if args.sweep:
            log(f"[sweep] itopk={params[0]:3d} width={params[1]} iters={params[2]:2d} n_seeds={params[3]:5d} "
                f"recall@{k}={rec:.4f} qps={s.nq / ms * 1e3:,.0f}")

    def best(th):
        ok = [t for t in table if t[1] >= th]
        return max(ok, key=lambda t: t[2]) if ok else None

    p90, p99 = best(0.90), best(0.99)
    # the fastest setting at which EVERY stratum reaches 0.90 (the blended figure leans on the scan-routed
    # queries, whose answers are exact)
    ok_all = [t for t in table if worst_stratum[t[0]] >= 0.90]
    p90_all = max(ok_all, key=lambda t: t[2]) if ok_all else None
    # several settings are within measurement noise of one another (ten timed steps each); among those
    # within 10 % of the fastest, the one the committed rocprofv3 counters were taken at is preferred, so
    # that the `traffic` figure applies to the run
    pref = committed_params(s.name)
    if p90 is not None and pref is not None:
        for t in table:
            if t[0] == pref and t[1] >= 0.90 and t[2] >= 0.90 * p90[2]:
                p90 = t
    if args.params:
        forced = tuple(int(v) for v in args.params.split(","))
        p90 = next(t for t in table if t[0] == forced)
    headline = p90 or max(table, key=lambda t: t[1])

    # ---- timed region: exactly K steps at the recall >= 0.90 operating point, profiling events on
    # (the interpreter's cyclic garbage collector is switched off for the timed loops: a collection
    # in the middle of one costs tens of milliseconds of host time)
    import gc
    gc.collect()
    gc.disable()
    ix.profile_enable(True)
    itopk, width, iters, n_seeds = headline[0]
    # untimed, like the burst after the index build: one pass over the library's ring of 64 timing-event sets.
    # While events are recorded for the first time the HIP runtime stalls once more for about 5 ms at some
    # point (seen in one run out of four when only the W warm-up steps preceded the timed region: 20 steps
    # then took 12.8 ms instead of 7.8 ms)
    for _ in range(72):
        vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, k, itopk, width, iters, n_seeds, out_ids, out_dists)
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, k, itopk, width, iters, n_seeds, out_ids, out_dists)
    torch.cuda.synchronize()
    ix.profile_enable(True)      # resets the duration sums: warm-up steps are not counted
    t0 = time.perf_counter()
    dbg = []
    for _ in range(args.steps):
        tt = time.perf_counter()
        vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, k, itopk, width, iters, n_seeds, out_ids, out_dists)
        dbg.append((time.perf_counter() - tt) * 1e3)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    if os.environ.get("VF_BENCH_DEBUG"):
        log("[debug] per-call host ms: " + " ".join(f"{t:.2f}" for t in dbg))
    pf = ix.profile_read()
    assert pf["calls"] == args.steps
    beam_avg_ms = pf["beam_ms_sum"] / pf["calls"]
    scan_avg_ms = pf["scan_ms_sum"] / pf["calls"]
    seed_avg_ms = pf["seed_ms_sum"] / pf["calls"]
    ix.profile_enable(False)
    found_head = out_ids.cpu().numpy()
    recall_head = recall_of(found_head)

    # recall per stratum at the headline point; for AND workloads also per decade of the intersection's
    # selectivity |C_a ∩ C_b| / N (sampled rows only)
    strata = {name: {"queries": int(mask.sum()), "recall_at_10": round(recall_at_k(found_head[rows[mask]], gt[mask]), 4)}
              for name, mask in strata_masks.items()}
    if s.query_mode == "and2" and len(rows) <= 5000:
        M_HS, M_LS, O_HS, O_LS = ix.export("M_HS"), ix.export("M_LS"), ix.export("O_HS"), ix.export("O_LS")

        def plist(l):
            return M_HS[O_HS[l]:O_HS[l] + S_host[l]] if O_HS[l] >= 0 else M_LS[O_LS[l]:O_LS[l] + S_host[l]]
        sel = np.empty(len(rows))
        for t, j in enumerate(rows):
            a, b = w.qlabel_ids[w.qlabel_offsets[j]:w.qlabel_offsets[j] + 2]
            sel[t] = len(np.intersect1d(plist(a), plist(b), assume_unique=True)) / s.n
        dec = np.floor(np.log10(np.maximum(sel, 1e-12))).astype(int)
        strata["by_selectivity_decade"] = {
            f"1e{d}": {"queries": int((dec == d).sum()),
                       "recall_at_10": round(recall_at_k(found_head[rows[dec == d]], gt[dec == d]), 4)}
            for d in sorted(set(dec.tolist()))}

    # ---- the same K steps once more with the launches serialised on one stream: in the timed
    # region the IVF-BFS kernel runs beside the IVF-Graph kernels and each shares the chip;
    # here every kernel has it to itself (reported next to the timed-region figures)
    for _ in range(args.warmup):
        vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, k, itopk, width, iters, n_seeds, out_ids, out_dists)
    torch.cuda.synchronize()
    ix.profile_enable(True, serial=True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, k, itopk, width, iters, n_seeds, out_ids, out_dists)
    torch.cuda.synchronize()
    ms_per_step_serial = (time.perf_counter() - t0) * 1e3 / args.steps
    pfs = ix.profile_read()
    def seed_kernel_name(p):
        return "seed_select_kernel" if p["seed_selected"] else ("seed_mfma_kernel" if p["seeds_on_matrix_cores"] else "seed_dist_kernel")
    alone_ms = {"beam_kernel": pfs["beam_ms_sum"] / pfs["calls"],
                seed_kernel_name(pfs): pfs["seed_ms_sum"] / pfs["calls"],
                SCAN_KERNELS[pfs["scan_kernel"]]: pfs["scan_ms_sum"] / pfs["calls"]}
    ix.profile_enable(False)

    eb = 1 if s.dtype == "uint8" else 4
    vec_bytes = s.dim * eb
    n_gq = pf["n_graph_queries"]
    # algorithmic work of each kernel of one step (one vf_search call)
    # distances whose vector the beam kernel gathers itself (counted by the kernel): children, and, when
    # float32 seeds went through the matrix cores, the best approximate seeds it re-scores
    gathered = pf["beam_gathered"]
    seed_kernel = seed_kernel_name(pf)
    # what passes from the seed kernel to the beam kernel: every distance (4 bytes a pair), or, when the seed kernel
    # selects, a few 8-byte keys per query and seed segment
    seed_handover = pf["seed_run_keys"] * 8 if pf["seed_selected"] else pf["seed_pairs"] * 4
    scan_kernel = SCAN_KERNELS[pf["scan_kernel"]]
    # the filtering kernel streams the bfloat16 copy of the lists (half the bytes per component) and leaves
    # k + margin candidates per query and list segment for the re-ranking kernel
    scan_vec_bytes = vec_bytes // 2 if pf["scan_kernel"] == 3 else vec_bytes
    kernels = {
        "beam_kernel": {
            "ms": beam_avg_ms, "bound": "hbm",
            "bytes": gathered * (vec_bytes + 4) + seed_handover + pf["beam_expanded"] * s.graph_degree * 4
                     + pf["beam_tested"] * 4 + n_gq * (vec_bytes + k * 12),
            "flops": 3 * gathered * s.dim},
        seed_kernel: {
            # matrix-core seed scoring moves more bytes than its flops are worth on this chip (operands in, the
            # distance matrix out): its binding roof is HBM; the exact ordered-distance kernel is ALU work
            # (with the selection fused in, only a few keys per query leave the kernel: back on the matrix-core roof)
            "ms": seed_avg_ms, "bound": ("mfma" if pf["seed_selected"] else "hbm") if pf["seeds_on_matrix_cores"] else "alu",
            # 2: float32 data scored from the bfloat16 copy of the seeds (two bfloat16 products per component:
            # the query's high and low part)
            "peak": ((2500.0 if pf["seeds_on_matrix_cores"] == 2 else FP32_VECTOR_PEAK_TFLOPS)
                     if s.dtype == "float32" else 5000.0) if pf["seeds_on_matrix_cores"] else FP32_VECTOR_PEAK_TFLOPS,
            "bytes": pf["seed_tile_seeds"] * ((vec_bytes // 2 if pf["seeds_on_matrix_cores"] == 2 else vec_bytes) + 4)
                     + n_gq * vec_bytes + seed_handover,
            # matrix cores: one multiply-add per element of q.x; vector ALU: one subtract + one fused multiply-add
            "flops": ({0: 3, 1: 2, 2: 4}[int(pf["seeds_on_matrix_cores"])]) * pf["seed_pairs"] * s.dim},
        scan_kernel: {
            "ms": scan_avg_ms, "bound": "hbm",
            "bytes": pf["scan_list_entries"] * (scan_vec_bytes + 4) + pf["n_scan_queries"] * (vec_bytes + k * 12),
            "flops": 2 * pf["scan_pairs"] * s.dim},
    }
    # the dominant kernel: the one with the longest average launch duration in the timed region
    dom = max(kernels, key=lambda n: kernels[n]["ms"])
    kd = kernels[dom]
    if kd["bound"] == "hbm":
        achieved, peak, unit = kd["bytes"] / (kd["ms"] * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
    else:   # fp32 vector ALU and fp32 dense MFMA have the same published peak; int8 MFMA 5 POP/s
        achieved, peak, unit = kd["flops"] / (kd["ms"] * 1e-3) / 1e12, kd.get("peak", FP32_VECTOR_PEAK_TFLOPS), \
            ("TFLOP/s" if s.dtype == "float32" else "TOP/s")
    roofline = {
        "kernel": dom, "bound": kd["bound"], "achieved": round(achieved, 2), "peak": peak, "unit": unit,
        "frac": round(achieved / peak, 4),
        "traffic": committed_traffic(dom, s.name, headline[0]),
        "algorithmic_bytes_per_launch": int(kd["bytes"]), "algorithmic_flops_per_launch": int(kd["flops"]),
        "avg_launch_ms": round(kd["ms"], 4),
        "alone": {"avg_launch_ms": round(alone_ms[dom], 4),
                  "achieved": round((kd["bytes"] / 1e9 if kd["bound"] == "hbm" else kd["flops"] / 1e12) / (alone_ms[dom] * 1e-3), 2),
                  "frac": round((kd["bytes"] / 1e9 if kd["bound"] == "hbm" else kd["flops"] / 1e12) / (alone_ms[dom] * 1e-3) / peak, 4),
                  "ms_per_step_serialised": round(ms_per_step_serial, 4)},
        # the whole graph path priced as the gathers of the paper's formulation (every query fetches every
        # vector it scores): bytes per query = scored (D b + 4) + expanded R 4 + tested 4 + D b + k 12
        "graph_search_as_gathers": (lambda b, ms: {"bytes_per_launch": int(b), "ms_alone": round(ms, 4),
                                                   "achieved": round(b / (ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                                                   "frac_of_hbm_peak": round(b / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 3)})(
            pf["beam_scored"] * (vec_bytes + 4) + pf["beam_expanded"] * s.graph_degree * 4 + pf["beam_tested"] * 4
            + n_gq * (vec_bytes + k * 12), alone_ms["beam_kernel"] + alone_ms[seed_kernel]),
        # the beam kernel priced on the search proper alone: children gathered, rows, predicate words, query in,
        # results out -- without the seeds it re-scores and without what the seed kernel hands over
        "beam_children_only": (lambda b: {"bytes_per_launch": int(b),
                                          "frac": round(b / (kernels["beam_kernel"]["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                          "frac_alone": round(b / (alone_ms["beam_kernel"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})(
            (gathered - pf["seed_rescored"]) * (vec_bytes + 4) + pf["beam_expanded"] * s.graph_degree * 4
            + pf["beam_tested"] * 4 + n_gq * (vec_bytes + k * 12)),
        "dense_contraction": dense,
        "graph_queries_per_launch": int(n_gq), "scan_queries_per_launch": int(pf["n_scan_queries"]),
        "scan_queries_rescanned_exactly": int(pf["scan_fallbacks"]),
        "distances_per_graph_query": round(pf["beam_scored"] / max(n_gq, 1), 1),
        "all_kernels": {n: {"avg_launch_ms": round(v["ms"], 4), "avg_launch_ms_alone": round(alone_ms[n], 4), "bound": v["bound"],
                            "algorithmic_bytes_per_launch": int(v["bytes"]), "flops_per_launch": int(v["flops"]),
                            "GBs": round(v["bytes"] / (max(v["ms"], 1e-6) * 1e-3) / 1e9, 1),
                            "TFLOPs": round(v["flops"] / (max(v["ms"], 1e-6) * 1e-3) / 1e12, 2)}
                        for n, v in kernels.items()},
    }

    if args.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # second operating point, timed the plain way
    extra = {}
    if p99 is not None:
        ms99 = time_search(vf, ix, Q, w.qlabel_offsets, w.qlabel_ids, k, p99[0], args.steps, args.warmup + 12, out_ids,
                           out_dists)
        extra = {"qps_at_recall_0.99": round(s.nq / ms99 * 1e3, 1), "recall_0.99_measured": round(p99[1], 4),
                 "params_0.99": dict(zip(("itopk", "width", "iters", "n_seeds"), p99[0]))}
    else:
        extra = {"qps_at_recall_0.99": None, "recall_0.99": "not reached on this grid",
                 "recall_ceiling": round(max(t[1] for t in table), 4)}
    if p90_all is not None:
        ms_all = time_search(vf, ix, Q, w.qlabel_offsets, w.qlabel_ids, k, p90_all[0], args.steps, args.warmup + 12, out_ids,
                             out_dists)
        sr = strata_recall(out_ids.cpu().numpy())
        extra["every_stratum_0.90"] = {"qps": round(s.nq / ms_all * 1e3, 1), "recall_at_10": round(p90_all[1], 4),
                                       "params": dict(zip(("itopk", "width", "iters", "n_seeds"), p90_all[0])),
                                       "recall_by_stratum": {n: round(v, 4) for n, v in sr.items()}}
    else:
        extra["every_stratum_0.90"] = {"qps": None, "note": "no setting of the grid reaches 0.90 on every stratum",
                                       "best_worst_stratum_recall": round(max(worst_stratum.values()), 4)}

    # ---- two-label queries on the same index: greedy AND, parallel AND policy, OR
    if args.multi:
        rng = np.random.default_rng(2468)
        cnt = np.diff(w.label_offsets)
        multi = np.flatnonzero(cnt >= 2)
        pick = rng.choice(multi, size=s.nq, replace=True)          # both labels of a pair occur on one data point
        qids2 = np.empty((s.nq, 2), dtype=np.int32)
        for t, v in enumerate(pick):
            labs = np.unique(w.label_ids[w.label_offsets[v]:w.label_offsets[v + 1]])
            if len(labs) < 2:
                labs = np.array([labs[0], (labs[0] + 1) % s.n_labels])
            qids2[t] = rng.choice(labs, size=2, replace=False)
        qoff2 = np.arange(0, 2 * s.nq + 1, 2, dtype=np.int64)
        qids2 = qids2.reshape(-1)
        res = {}
        for name, mode in (("and_greedy", vf.AND_GREEDY), ("and_parallel", vf.AND_PARALLEL), ("or", vf.OR)):
            gi, _ = vf.search_multi(ix, Q, qoff2, qids2, mode | vf.MULTI_EXACT, k)
            gtm = gi.cpu().numpy()
            row = {}
            for tag, prm in (("p90", headline[0]), ("p99", (p99 or headline)[0])):
                for _ in range(args.warmup + 12):   # a new call shape: the runtime's one-time stall again (see above)
                    vf.search_multi(ix, Q, qoff2, qids2, mode, k, *prm, out_ids, out_dists)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    vf.search_multi(ix, Q, qoff2, qids2, mode, k, *prm, out_ids, out_dists)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) * 1e3 / args.steps
                row[tag] = {"params": list(prm), "qps": round(s.nq / ms * 1e3, 1),
                            "recall_at_10": round(recall_at_k(out_ids.cpu().numpy(), gtm), 4)}
            res[name] = row
        extra["two_label_queries"] = res

    # ---- exact kNN graphs against pruned graphs (rank-based pruning + reverse edges): recall of the graph-routed
    # queries by list size at fixed search parameters, and the build time of either kind
    if args.compare_graphs:
        S_host = ix.export("S")
        first_label = w.qlabel_ids[w.qlabel_offsets[:-1]]
        single = np.diff(w.qlabel_offsets) == 1
        rows_all = np.arange(s.nq) if gt_rows is None else gt_rows
        gt_full = {int(r): gt[t] for t, r in enumerate(rows_all)}
        settings = [(32, 1, 8, 256), (32, 1, 8, 1024), tuple(headline[0]), tuple((p99 or headline)[0])]
        buckets = [(s.T, 2 * s.T), (2 * s.T, 5 * s.T), (5 * s.T, 15 * s.T), (15 * s.T, 1 << 62)]
        cmp_out = {"settings": [list(p) for p in settings], "index_build_s": {}, "recall_at_10": {}}
        for kind_name, kind in (("knn", vf.GRAPH_KNN), ("pruned", vf.GRAPH_PRUNED)):
            torch.cuda.synchronize()
            tb = time.time()
            ix2 = vf.build_index(X, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree, graph_kind=kind)
            torch.cuda.synchronize()
            cmp_out["index_build_s"][kind_name] = round(time.time() - tb, 3)
            for prm in settings:
                vf.search(ix2, Q, w.qlabel_offsets, w.qlabel_ids, k, *prm, out_ids, out_dists)
                found = out_ids.cpu().numpy()
                for lo, hi in buckets:
                    sel = [r for r in rows_all if single[r] and lo <= S_host[first_label[r]] < hi]
                    if not sel:
                        continue
                    rec = recall_at_k(found[sel], np.stack([gt_full[int(r)] for r in sel]))
                    key = f"list size [{lo}, {hi if hi < (1 << 61) else 'inf'})"
                    cmp_out["recall_at_10"].setdefault(key, {"queries": len(sel)}).setdefault(kind_name, []).append(round(rec, 4))
            del ix2
        extra["graph_comparison"] = cmp_out

    # ---- small-batch latency on the same index (batches of 1, 8, 64; labels half graph lists, half scan lists)
    if args.latency:
        S_host = ix.export("S")
        lab = w.qlabel_ids[w.qlabel_offsets[:-1]]
        gq_idx = np.flatnonzero(S_host[lab] >= s.T)
        sq_idx = np.flatnonzero((S_host[lab] < s.T) & (S_host[lab] > 0))
        rng = np.random.default_rng(4321)
        lat = {}
        p_lat = (p99 or headline)[0]
        for bs in (1, 8, 64):
            times = []
            n_batches = 1200
            for b in range(n_batches):
                ng = bs // 2 if bs > 1 else (b % 2)
                pick = np.concatenate([rng.choice(gq_idx, size=ng, replace=False),
                                       rng.choice(sq_idx, size=bs - ng, replace=False)])
                Qb = Q[torch.from_numpy(pick).cuda()].contiguous()
                qo = np.arange(bs + 1, dtype=np.int64)
                ql = np.ascontiguousarray(lab[pick])
                oi = out_ids[:bs]; od = out_dists[:bs]
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                vf.search(ix, Qb, qo, ql, k, *p_lat, oi, od)
                torch.cuda.synchronize()
                times.append((time.perf_counter() - t0) * 1e3)
            t = np.sort(np.array(times[200:]))      # first 200 batches are warm-up
            lat[f"batch_{bs}"] = {"p50_ms": round(float(t[len(t) // 2]), 4), "p99_ms": round(float(t[int(len(t) * 0.99)]), 4),
                                  "qps": round(bs / float(np.mean(t)) * 1e3, 1)}
        # throughput of small batches that arrive faster than one call completes: the same calls issued
        # round-robin on 1 and on 4 streams without waiting in between (every stream has a workspace of its
        # own inside the index, so calls on different streams overlap on the GPU)
        streams = [torch.cuda.Stream() for _ in range(4)]
        for bs in (1, 8, 64):
            batches = []
            for b in range(64):
                ng = bs // 2 if bs > 1 else (b % 2)
                pick = np.concatenate([rng.choice(gq_idx, size=ng, replace=False),
                                       rng.choice(sq_idx, size=bs - ng, replace=False)])
                batches.append((Q[torch.from_numpy(pick).cuda()].contiguous(), np.arange(bs + 1, dtype=np.int64),
                                np.ascontiguousarray(lab[pick]),
                                torch.empty((bs, k), dtype=torch.int64, device="cuda"),
                                torch.empty((bs, k), dtype=torch.float32, device="cuda")))
            torch.cuda.synchronize()
            for n_streams in (1, 4):
                rates = []
                for rep in range(6):
                    t0 = time.perf_counter()
                    for r in range(8):
                        for i, (Qb, qo, ql, oi, od) in enumerate(batches):
                            with torch.cuda.stream(streams[i % n_streams]):
                                vf.search(ix, Qb, qo, ql, k, *p_lat, oi, od)
                    torch.cuda.synchronize()
                    rates.append(8 * len(batches) * bs / (time.perf_counter() - t0))
                lat[f"batch_{bs}"][f"pipelined_qps_{n_streams}_stream{'s' if n_streams > 1 else ''}"] = round(float(np.median(rates[1:])), 1)
        # the same kind of traffic through a serving session (one resident kernel, a job ring, one wave per query):
        # single queries submitted from the host with 1, 8, 64 and 240 of them in flight.  A worker wave scores its
        # query's seeds by itself, so sessions are measured at the operating point's parameters and at a moderate
        # seed count
        served = {}
        n_serve = 4000
        pick = np.concatenate([rng.choice(gq_idx, size=n_serve // 2, replace=True), rng.choice(sq_idx, size=n_serve // 2, replace=True)])
        rng.shuffle(pick)
        qs_host = np.ascontiguousarray(w.queries[pick])
        qo_s = np.arange(n_serve + 1, dtype=np.int64)
        ql_s = np.ascontiguousarray(lab[pick])
        gt_s = gt if gt_rows is None else None
        for tag, prm in (("operating_point", p_lat), ("512_seeds", (p_lat[0], p_lat[1], p_lat[2], 512))):
            if prm[0] > 64:
                continue
            srv = vf.Server(ix, k, *prm, n_workers=240, ring_slots=1024)
            try:
                srv.run(qs_host[:512], qo_s[:513], ql_s[:512], in_flight=64)        # warm-up
                row = {"params": list(prm)}
                for fl in (1, 8, 64, 240):
                    t0 = time.perf_counter()
                    ids_s, _, lat_us = srv.run(qs_host, qo_s, ql_s, in_flight=fl)
                    dt = time.perf_counter() - t0
                    ls = np.sort(lat_us)
                    row[f"in_flight_{fl}"] = {"qps": round(n_serve / dt, 1), "p50_ms": round(float(ls[len(ls) // 2]) / 1e3, 4),
                                              "p99_ms": round(float(ls[int(len(ls) * 0.99)]) / 1e3, 4)}
                if gt_s is not None:
                    row["recall_at_10"] = round(recall_at_k(ids_s, gt_s[pick]), 4)
            finally:
                srv.end()
            served[tag] = row
        lat["served_session"] = served
        extra["latency"] = {"params": dict(zip(("itopk", "width", "iters", "n_seeds"), p_lat)), **lat}

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same queries
    cpu = None
    if not args.no_cpu:
        from oracle import OracleIndex
        rng = np.random.default_rng(12345)
        sample = np.sort(rng.choice(s.nq, size=min(args.cpu_sample, s.nq), replace=False))
        # threads: the host cores this job may use -- the box's own limit (OMP_NUM_THREADS) when it sets one,
        # else every core the interpreter sees
        seen = os.cpu_count() or 1
        limit = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
        cores = min(seen, limit) if limit > 0 else seen
        qs = np.ascontiguousarray(w.queries[sample])
        cnt = np.diff(w.qlabel_offsets)[sample]
        qo = np.zeros(len(sample) + 1, dtype=np.int64)
        np.cumsum(cnt, out=qo[1:])
        ql = np.concatenate([w.qlabel_ids[w.qlabel_offsets[j]:w.qlabel_offsets[j + 1]] for j in sample]).astype(np.int32)
        t0 = time.time()
        ixo = OracleIndex(w.vectors, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree, lazy_graph=True,
                          n_threads=cores)
        okw = dict(and_scan_limit=args.and_scan_limit)
        ids_o, d_o = ixo.search(qs, qo, ql, k, itopk, width, iters, n_seeds, **okw)   # untimed: builds the graph rows it touches
        log(f"[bench] oracle index (lazy graph rows) + first pass over {len(sample)} queries on {cores} threads: "
            f"{time.time() - t0:.1f}s")

        def timed(n_threads, budget_s, max_reps):
            reps, spent = 0, 0.0
            t0 = time.perf_counter()
            while spent < budget_s and reps < max_reps:
                ixo.search(qs, qo, ql, k, itopk, width, iters, n_seeds, n_threads=n_threads, **okw)
                reps += 1
                spent = time.perf_counter() - t0
            return reps * len(sample) / spent, reps
        cpu_qps, reps = timed(cores, 4.0, 200)
        one_qps, reps1 = timed(1, 6.0, 50)
        vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, k, itopk, width, iters, n_seeds, out_ids, out_dists)
        torch.cuda.synchronize()
        gpu_rows = out_ids.cpu().numpy()[sample]     # same parameters as the timed region
        agree = float(np.mean([np.array_equal(a, b) for a, b in zip(gpu_rows, ids_o)]))
        cpu = {"value": round(cpu_qps, 1), "unit": "queries/s", "cores": cores, "kind": "oracle",
               "sample": f"{len(sample)} of the {s.nq} queries (seeded random sample), same parameters as the timed "
                         f"region, {reps} timed passes on {cores} threads after one untimed pass that builds the graph "
                         f"rows touched; single_core: {reps1} passes on one thread",
               "single_core": round(one_qps, 1), "cpu_count_seen": seen,
               "rows_identical_to_gpu": round(agree, 4)}

    line = {
        "metric": "filtered QPS at recall@10 >= 0.90", "value": round(s.nq / ms_per_step * 1e3, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if s.dtype == "float32" else "u8", "data": "synthetic",
        "config": {"workload": f"{s.name}: N={s.n} dim={s.dim} {s.dtype}, {s.n_clusters} Gaussian clusters, "
                               f"{s.n_labels} Zipf({s.zipf_alpha}) labels, T={s.T}, R={s.graph_degree}, "
                               f"{s.nq} queries ({s.query_mode}), k={k}, seed {s.seed}",
                   "graphs": "pruned (degree-2R kNN, rank-based pruning, reverse edges)" if pruned else "exact kNN",
                   "and_scan_limit": args.and_scan_limit,
                   "params": dict(zip(("itopk", "width", "iters", "n_seeds"), headline[0])),
                   "recall_at_10": round(recall_head, 4), "reached_0.90": p90 is not None,
                   "recall_by_stratum": strata,
                   "index_build_s": round(build_s, 2), **extra},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
