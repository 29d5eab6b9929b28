#!/usr/bin/env python3
"""Benchmark of the QuIVer query hot path on one MI355X.

A "step" is one batch through qv_search (query encode -> code-space beam search -> float32 cosine
rerank) for all queries of the workload, inputs resident in HBM.  The default workload is the 768-d,
1M-vector, ef=64 configuration the metric is quoted on.  Prints ONE JSON line on stdout; progress
goes to stderr.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def log(msg: str) -> None:
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def kernel_source_digest() -> str:
    """sha256 over the sources the search kernel is compiled from: a counter file taken on other code is stale."""
    h = hashlib.sha256()
    for name in ("search.hip", "kernels.h"):
        with open(os.path.join(ROOT, "paper_2605_02171_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def mean_lines_per_row(row_bytes: int, stride_bytes: int) -> float:
    """128-byte lines a code row touches on average when rows start at multiples of stride_bytes."""
    starts = {(i * stride_bytes) % 128 for i in range(128)}
    return float(np.mean([(s + row_bytes + 127) // 128 for s in starts]))


def ground_truth(xd, qd, k, metric):
    """Exact float32 top-k on the GPU (chunked matmul; the only dense contraction in this repo)."""
    import torch
    n = xd.shape[0]
    best_v = torch.full((qd.shape[0], k), -float("inf"), device=qd.device)
    best_i = torch.zeros((qd.shape[0], k), dtype=torch.int64, device=qd.device)
    qn = qd / qd.norm(dim=1, keepdim=True).clamp_min(1e-30) if metric == "cosine" else qd
    q2 = (qd * qd).sum(1, keepdim=True)
    for s in range(0, n, 131072):
        xb = xd[s:s + 131072]
        if metric == "cosine":
            sim = qn @ (xb / xb.norm(dim=1, keepdim=True).clamp_min(1e-30)).T
        else:
            sim = -(q2 - 2.0 * (qd @ xb.T) + (xb * xb).sum(1)[None, :])
        v, i = sim.topk(k, dim=1)
        cat_v = torch.cat([best_v, v], 1)
        cat_i = torch.cat([best_i, i + s], 1)
        best_v, sel = cat_v.topk(k, dim=1)
        best_i = cat_i.gather(1, sel)
    return best_i.cpu().numpy()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)   # ~5 s of search: long enough for an outside sampler to see
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--n", type=int, default=0, help="override the number of base vectors (for quick runs)")
    ap.add_argument("--nq", type=int, default=0)
    ap.add_argument("--ef", type=int, default=64)
    ap.add_argument("--visited-slots", type=int, default=0)
    ap.add_argument("--lanes-per-row", type=int, default=0)
    ap.add_argument("--table-format", type=int, default=0)
    ap.add_argument("--visited-mode", type=int, default=0, help="0 default, 1 exact table, 2 cache")
    ap.add_argument("--rerank-mode", type=int, default=0, help="0 default, 1 a kernel of its own, 2 inside the search kernel")
    ap.add_argument("--gpu-build", action="store_true",
                    help="also build the graph on the GPU (qv_build_graph), time it and search it")
    ap.add_argument("--graph", choices=("host", "gpu"), default="host",
                    help="host: the input graph comes from the host generator (default; the only choice the CPU "
                         "oracle leg accepts); gpu: built by qv_build_graph (no CPU leg: nothing the library "
                         "produced is ever an oracle input)")
    ap.add_argument("--encoding", choices=("sm", "sign1", "sq2"), default="sm",
                    help="sm: the method; sign1 / sq2: the paper's ablation encodings (graph built on the GPU in that "
                         "encoding's own distance, so --graph gpu is implied and there is no CPU leg)")
    ap.add_argument("--index-layout", choices=("dense", "recommended", "split"), default="recommended",
                    help="recommended (default): the index's code rows in the layout qv_code_layout names (planes padded "
                         "to a compiled kernel width, rows aligned to 128-byte lines); differs from dense rows only at "
                         "some widths, e.g. 384-d and 960-d, not at 768-d.  split: sign plane first, the rest of the magnitude "
                         "plane in a second array that is read only for neighbours the sign-plane bound lets through "
                         "(768-d, 1024-d, 1536-d)")
    ap.add_argument("--cold-host", action="store_true",
                    help="keep the float32 vectors in pinned host memory (rerank reads them over PCIe)")
    ap.add_argument("--no-scan", action="store_true", help="skip the brute-force code scan / overlap probe")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one elementwise copy kernel (1 GiB read + 1 GiB write) to calibrate byte counters")
    ap.add_argument("--cpu-sample", type=int, default=10000, help="queries the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-companion", action="store_true",
                    help="skip the companion figure (default run only): the same path on the low-rank 768-d workload H2, "
                         "the regime the paper calls compatible, where Recall@10 means something")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (on several, the queries would be sharded over replicas "
              "of the index). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    import paper_2605_02171_amd as qv
    from workloads import datagen, graph

    torch.cuda.set_device(0)
    enc = {"sm": qv.ENC_SM, "sign1": qv.ENC_SIGN1, "sq2": qv.ENC_SQ2}[args.encoding]
    if enc != qv.ENC_SM:
        args.graph = "gpu"
    w = datagen.scaled(args.workload, n=args.n or None, nq=args.nq or None)
    ef, k = args.ef, w.k
    t0 = time.time()
    x = datagen.make_base(w)
    q = datagen.make_queries(w)
    log(f"workload {w.name}: n={w.n} d={w.d} nq={w.nq} generated in {time.time() - t0:.1f}s")
    os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
    xd = torch.from_numpy(x).cuda()
    qd = torch.from_numpy(q).cuda()
    t0 = time.time()
    if args.graph == "host":
        adj, entry = graph.cached_graph(f"{w.name}_{w.n}", x, w.R, w.L, w.alpha,
                                        progress_path=os.path.join(ROOT, "gpurun_out", "bench_progress.log"))
        adjd = qv.from_numpy_u32(adj)
    else:
        # entry = the node whose code is nearest to the code of the float32 centroid (ties: smallest id), as the
        # host generator picks it; graph by the library's own construction
        args.cpu_sample = 0
        c0 = qv.encode(xd, enc=enc)
        cen = torch.zeros((1, w.d), dtype=torch.float64, device="cuda")
        for s0 in range(0, w.n, 1 << 18):
            cen += xd[s0:s0 + (1 << 18)].sum(0, keepdim=True, dtype=torch.float64)
        eid, _ = qv.bq_scan(c0, qv.encode((cen / w.n).float(), enc=enc), w.d, 1, enc=enc)
        entry = int(qv.to_numpy_u32(eid)[0, 0])
        adjd = qv.build_graph(c0, w.d, w.R, w.L, w.alpha, entry, enc=enc)
        torch.cuda.synchronize()
        adj = None
        del c0
    t_graph = time.time() - t0
    log(f"graph R={w.R} L={w.L} alpha={w.alpha} ready in {t_graph:.1f}s "
        f"({'host, %d threads' % graph.host_threads() if args.graph == 'host' else 'GPU, entry %d' % entry})")

    # base encode (index-build side of the hot path): timed on its own
    codes = qv.encode(xd, enc=enc)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        codes = qv.encode(xd, enc=enc)
    e1.record()
    torch.cuda.synchronize()
    enc_ms = e0.elapsed_time(e1) / 5
    enc_bytes = w.n * (4 * w.d + 8 * qv.code_words(w.d, enc))
    log(f"encode base: {enc_ms:.3f} ms, {enc_bytes / enc_ms / 1e6:.0f} GB/s")

    x_cold = None
    if args.cold_host:
        x_cold = torch.empty(x.shape, dtype=torch.float32, pin_memory=True)
        x_cold.copy_(torch.from_numpy(x))
    dense_layout = ((w.d + 63) // 64, qv.code_words(w.d, enc))
    layout = qv.code_layout(w.d, enc) if args.index_layout == "recommended" else dense_layout
    split = qv.split_codes(codes, w.d) if args.index_layout == "split" else None
    index_codes = qv.pad_codes(codes, w.d, layout, enc=enc) if layout != dense_layout else codes
    index = qv.Index(adjd, index_codes, x_cold if args.cold_host else xd, entry, enc=enc,
                     layout=layout if layout != dense_layout else None)
    if split is not None:
        index.set_split_codes(split)
    ws = torch.empty((qv.search_workspace_bytes(w.nq, w.d, k, ef),), dtype=torch.uint8, device="cuda")

    # Counters for the algorithmic-byte model: one traced pass with the visited set that never forgets, which
    # evaluates every node at most once, as the algorithm states it (queries whose table still filled up are
    # counted as they ran and reported).
    index.set_tuning(0, args.lanes_per_row, args.table_format, qv.VISITED_EXACT)
    exact = qv.search(index, qd, k, ef, trace=True, workspace=ws)
    torch.cuda.synchronize()
    n_exp = qv.to_numpy_u32(exact.n_expanded).astype(np.int64)
    n_eval = qv.to_numpy_u32(exact.n_dist_evals).astype(np.int64)
    n_cand = qv.to_numpy_u32(exact.n_cand).astype(np.int64)
    n_overflow = int((qv.to_numpy_u32(exact.status) & 2 != 0).sum())
    del exact
    # the configuration that is timed (default: visited set as a small cache): results for recall / parity
    index.set_tuning(args.visited_slots, args.lanes_per_row, args.table_format, args.visited_mode, args.rerank_mode)
    traced = qv.search(index, qd, k, ef, trace=True, workspace=ws)
    torch.cuda.synchronize()
    n_eval_run = qv.to_numpy_u32(traced.n_dist_evals).astype(np.int64)
    status = qv.to_numpy_u32(traced.status)
    ids_gpu = qv.to_numpy_u32(traced.ids)
    assert (qv.to_numpy_u32(traced.n_expanded) == n_exp).all()
    code_b = 8 * qv.code_words(w.d, enc)
    search_bytes = int(4 * w.R * n_exp.sum() + code_b * n_eval.sum() + code_b * w.nq + 8 * ef * w.nq)
    rerank_bytes = int(4 * w.d * n_cand.sum() + 4 * w.d * w.nq + 8 * k * w.nq)
    encq_bytes = int(w.nq * (4 * w.d + code_b))
    log(f"per query: expanded {n_exp.mean():.1f}, distance evals {n_eval.mean():.0f} (max {n_eval.max()}; "
        f"{n_overflow} queries overflowed the exact table); as timed: {n_eval_run.mean():.0f} evals "
        f"({n_eval_run.sum() / n_eval.sum() - 1:+.1%}); expanded p50/p90/p99/max = "
        f"{np.percentile(n_exp, 50):.0f}/{np.percentile(n_exp, 90):.0f}/{np.percentile(n_exp, 99):.0f}/{n_exp.max()}; "
        f"evals p50/p90/p99 = {np.percentile(n_eval, 50):.0f}/{np.percentile(n_eval, 90):.0f}/{np.percentile(n_eval, 99):.0f}")

    # timed region
    out = qv.SearchOutput(traced.ids, traced.scores)
    for _ in range(args.warmup):
        qv.search(index, qd, k, ef, workspace=ws, out=out)
    timer = qv.Timer(args.steps)
    index.set_timer(timer)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        qv.search(index, qd, k, ef, workspace=ws, out=out)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    stage_ms = timer.read()
    index.set_timer(None)
    ms_per_step = wall * 1e3 / args.steps
    qps = w.nq / (wall / args.steps)
    search_ms = float(stage_ms[:, 1].mean())
    log(f"{ms_per_step:.3f} ms/step, {qps:.0f} QPS; stages (ms): encode {stage_ms[:, 0].mean():.3f}, "
        f"search {search_ms:.3f}, rerank {stage_ms[:, 2].mean():.3f}")

    # ceiling of the memory system for the search kernel's gather pattern: as many random code rows as the
    # batch evaluates, no arithmetic
    gather_gbps = gather_line_gbps = None
    n_rows = int(n_eval.sum()) // 64 * 64
    if n_rows >= 64 and enc == qv.ENC_SM:      # the probe reads rows of two planes
        rid = torch.randint(0, w.n, (n_rows,), device="cuda", dtype=torch.int32)
        qv.gather_probe(codes, w.d, rid)
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(3):
            qv.gather_probe(codes, w.d, rid)
        g1.record()
        torch.cuda.synchronize()
        probe_s = g0.elapsed_time(g1) / 3 * 1e-3
        gather_gbps = n_rows * (code_b + 4) / probe_s / 1e9
        gather_line_gbps = n_rows * mean_lines_per_row(code_b, code_b) * 128 / probe_s / 1e9
        log(f"random code-row gather ceiling: {gather_gbps:.0f} GB/s of rows, {gather_line_gbps:.0f} GB/s of 128-byte lines")
        del rid

    if args.calib_copy:
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.add(a, 1.0, out=b)  # one vectorized elementwise kernel: reads 2^30 B, writes 2^30 B
        torch.cuda.synchronize()
        del a, b

    gt = ground_truth(xd, qd, k, w.metric)
    recall = float(np.mean([len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ids_gpu, gt)]) / k)
    log(f"Recall@{k} = {recall:.4f}")

    # brute-force scan in code space (all queries x all base codes) and the overlap probe against exact top-10
    scan = None
    if not args.no_scan:
        qcodes_d = qv.encode(qd, enc=enc)
        sid, sdist = qv.bq_scan(codes, qcodes_d, w.d, k, enc=enc)
        torch.cuda.synchronize()
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s0.record()
        sid, sdist = qv.bq_scan(codes, qcodes_d, w.d, k, enc=enc)
        s1.record()
        torch.cuda.synchronize()
        scan_ms = s0.elapsed_time(s1)
        hits = qv.topk_overlap(sid, torch.from_numpy(gt.astype(np.uint32).view(np.int32)).cuda())
        overlap = float(qv.to_numpy_u32(hits).sum()) / (w.nq * k)
        found = qv.topk_overlap(sid, qv.from_numpy_u32(np.ascontiguousarray(qv.to_numpy_u32(traced.cand_ids)[:, :k])))
        # per 32 dims: xor, 2 three-input ops, 3 popcount-adds (2-bit encodings); xor + popcount-add (1-bit sign)
        lane_ops = (2.0 if enc == qv.ENC_SIGN1 else 6.0) * ((w.d + 31) // 32) * w.nq * w.n
        alu_peak = 256 * 64 * 2.4e9
        scan = {"ms": scan_ms, "dist_evals_per_s": w.nq * w.n / (scan_ms * 1e-3),
                "top10_overlap_code_vs_exact": overlap,
                "graph_search_finds_code_top10": float(qv.to_numpy_u32(found).sum()) / (w.nq * k),
                "roofline": {"kernel": "bq_scan_kernel", "bound": "alu", "achieved": lane_ops / (scan_ms * 1e-3) / 1e12,
                             "peak": alu_peak / 1e12, "unit": "T lane-ops/s (int32 VALU)",
                             "frac": lane_ops / (scan_ms * 1e-3) / alu_peak}}
        log(f"code scan {w.nq} x {w.n}: {scan_ms:.1f} ms, {scan['dist_evals_per_s'] / 1e9:.1f} G dist/s, "
            f"{scan['roofline']['frac']:.2f} of VALU peak; top-10 overlap code vs exact {overlap:.3f}; "
            f"beam search finds {scan['graph_search_finds_code_top10']:.3f} of the code-space top-10")

    # graph construction on the GPU (same reading as the oracle's orc_build_graph), timed, then searched
    gpu_build = None
    if args.gpu_build:
        adj_g = qv.build_graph(codes, w.d, w.R, w.L, w.alpha, entry, enc=enc)      # warm-up (first launches, allocator)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        adj_g = qv.build_graph(codes, w.d, w.R, w.L, w.alpha, entry, enc=enc)
        torch.cuda.synchronize()
        t_gb = time.perf_counter() - t0
        index_g = qv.Index(adj_g, codes, xd, entry, enc=enc)
        og = qv.search(index_g, qd, k, ef, workspace=ws)
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(5):
            og = qv.search(index_g, qd, k, ef, workspace=ws)
        g1.record()
        torch.cuda.synchronize()
        rec_g = float(np.mean([len(set(a.tolist()) & set(b.tolist())) for a, b in zip(qv.to_numpy_u32(og.ids), gt)]) / k)
        deg_g = (qv.to_numpy_u32(adj_g) != 0xFFFFFFFF).sum(1)
        gpu_build = {"seconds": t_gb, "nodes_per_s": w.n / t_gb, "mean_degree": float(deg_g.mean()),
                     "recall_at_10_on_it": rec_g, "qps_on_it": w.nq / (g0.elapsed_time(g1) / 5 * 1e-3),
                     "host_generator_seconds": t_graph}
        log(f"GPU graph construction: {t_gb:.2f} s ({w.n / t_gb / 1e3:.0f} k nodes/s), mean degree {deg_g.mean():.1f}; "
            f"search on it: recall {rec_g:.4f}, {gpu_build['qps_on_it']:.0f} QPS")
        del index_g, adj_g

    # CPU oracle on a bounded sample of the same queries, all host threads
    cpu = None
    parity = None
    if args.cpu_sample > 0:
        import oracle
        threads = graph.host_threads()
        ns = min(args.cpu_sample, w.nq)
        t0 = time.time()
        ocodes = oracle.encode(x, threads=threads)
        t_enc = time.time() - t0
        t0 = time.time()
        ref = oracle.search(q[:ns], adj, ocodes, x, entry, k, ef, threads=threads)
        t_cpu = time.time() - t0
        kept_all = (status[:ns] & 2) == 0       # queries whose visited set forgot nothing in the timed configuration
        parity = bool((ref.cand_ids == qv.to_numpy_u32(traced.cand_ids)[:ns]).all() and
                      (ref.cand_dist == qv.to_numpy_u32(traced.cand_dist)[:ns]).all() and
                      (ref.n_expanded == n_exp[:ns]).all() and
                      (ref.n_dist_evals[kept_all] == n_eval_run[:ns][kept_all]).all() and
                      (ref.n_dist_evals <= n_eval_run[:ns]).all() and
                      (n_overflow > 0 or (ref.n_dist_evals == n_eval[:ns]).all()) and
                      (ocodes == qv.to_numpy_u64(codes)).all() and
                      np.allclose(ref.scores, traced.scores.cpu().numpy()[:ns], rtol=1e-5, atol=1e-7))
        orecall = float(np.mean([len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ref.ids, gt[:ns])]) / k)
        n1 = min(200, ns)
        t0 = time.time()
        oracle.search(q[:n1], adj, ocodes, x, entry, k, ef, threads=1)
        t_1t = time.time() - t0
        cpu_model = "unknown"
        try:
            with open("/proc/cpuinfo") as f:
                cpu_model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "unknown")
        except OSError:
            pass
        cpu = {"value": ns / t_cpu, "single_thread_value": n1 / t_1t, "unit": "queries/s", "cores": threads, "kind": "oracle",
               "cpu_model": cpu_model, "host_cpus_visible": os.cpu_count(),
               "sample": f"first {ns} of the {w.nq} queries, same graph/codes/vectors; search+rerank wall time "
                         f"{t_cpu:.2f}s ({threads} threads); base encode by the oracle took {t_enc:.1f}s (not included)",
               "recall_at_10": orecall}
        log(f"oracle: {n1 / t_1t:.0f} QPS on 1 thread ({n1} queries), {ns / t_cpu:.0f} QPS on {threads} threads, recall {orecall:.4f}, parity with GPU: {parity}")

    # Companion figure for the default run: the same shapes (1M x 768, 10,000 queries, ef as given) on the low-rank
    # workload H2, where code ranking and exact ranking agree well enough for Recall@10 to mean something (the
    # prescribed generator of the headline workload is outside that regime).  Graph by qv_build_graph; no CPU leg.
    companion = None
    if w.name == "C2" and not (args.n or args.nq or args.no_companion) and enc == qv.ENC_SM:
        hw = datagen.scaled("H2")
        hx = torch.from_numpy(datagen.make_base(hw)).cuda()
        hq = torch.from_numpy(datagen.make_queries(hw)).cuda()
        hcodes = qv.encode(hx)
        cen = torch.zeros((1, hw.d), dtype=torch.float64, device="cuda")
        for s0 in range(0, hw.n, 1 << 18):
            cen += hx[s0:s0 + (1 << 18)].sum(0, keepdim=True, dtype=torch.float64)
        eid, _ = qv.bq_scan(hcodes, qv.encode((cen / hw.n).float()), hw.d, 1)
        hentry = int(qv.to_numpy_u32(eid)[0, 0])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        hadj = qv.build_graph(hcodes, hw.d, hw.R, hw.L, hw.alpha, hentry)
        torch.cuda.synchronize()
        t_hb = time.perf_counter() - t0
        hindex = qv.Index(hadj, hcodes, hx, hentry)
        hgt = ground_truth(hx, hq, k, hw.metric)
        companion = {"workload": f"H2: {hw.n} x {hw.d} low-rank unit-norm vectors (ours), {hw.nq} queries, graph R={hw.R} "
                                 f"L={hw.L} alpha={hw.alpha} by qv_build_graph in {t_hb:.2f} s, k={k}, ef={ef}"}
        for lay in ("dense", "split"):
            hindex.set_split_codes(qv.split_codes(hcodes, hw.d) if lay == "split" else None)
            ho = qv.search(hindex, hq, k, ef, workspace=ws)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            h_steps = min(args.steps, 500)
            for _ in range(h_steps):
                ho = qv.search(hindex, hq, k, ef, workspace=ws)
            torch.cuda.synchronize()
            h_ms = (time.perf_counter() - t0) * 1e3 / h_steps
            h_rec = float(np.mean([len(set(a.tolist()) & set(b.tolist())) for a, b in zip(qv.to_numpy_u32(ho.ids), hgt)]) / k)
            companion[f"{lay}_code_rows"] = {"queries_per_s": hw.nq / (h_ms * 1e-3), "ms_per_step": h_ms, "recall_at_10": h_rec}
            log(f"companion H2, {lay} code rows: {h_ms:.3f} ms/step, {hw.nq / (h_ms * 1e-3):.0f} QPS, Recall@{k} = {h_rec:.4f}")
        del hindex, hadj, hcodes, hx, hq

    # counter-measured traffic of the search kernel for this workload, from the committed rocprofv3 summary of this
    # same command; a file taken on other kernel sources is ignored and reported as stale
    traffic = l2_hit = traffic_commit = None
    traffic_stale = False
    tpath = os.path.join(ROOT, "profiles", f"traffic_{w.name}_ef{ef}.json")
    default_run = not (args.n or args.nq or args.visited_slots or args.lanes_per_row or args.table_format or
                       args.visited_mode or args.rerank_mode or args.cold_host) and args.graph == "host" and enc == qv.ENC_SM
    if split is not None:
        tpath = tpath.replace(".json", "_split.json")
    if os.path.exists(tpath) and default_run and args.index_layout != "dense":
        with open(tpath) as f:
            tj = json.load(f)
        if tj.get("kernel_source_sha256") == kernel_source_digest():
            traffic = tj.get("search_kernel_hbm_bytes_per_launch")
            l2_hit = tj.get("l2_hit_rate")
            traffic_commit = tj.get("commit")
        else:
            traffic_stale = True
            log(f"{os.path.basename(tpath)} was taken on other kernel sources: ignored")

    # with Stage 2 inside the search kernel that kernel's bytes are those of both stages
    fused = index.rerank_fused(ef)
    kernel_bytes = search_bytes + (rerank_bytes if fused else 0)
    algorithmic_gbps = kernel_bytes / (search_ms * 1e-3) / 1e9
    traffic_gbps = traffic / (search_ms * 1e-3) / 1e9 if traffic else None
    # The fraction of the HBM roofline is taken from the bytes the fabric moved (counters) when a current counter file
    # exists: rows that several queries share (the start of every search, hub nodes) are served by L2, so the bytes the
    # algorithm asks for can exceed both what moved and what HBM could move.  Without counters the algorithmic
    # figure is all there is, and `basis` says so.
    achieved = traffic_gbps if traffic_gbps else algorithmic_gbps
    line = {
        "metric": "QPS at Recall@10 (ef=%d), 1M x 768 on 1 MI355X" % ef if w.name == "C2" and not args.n
                  else f"QPS at Recall@10 (ef={ef})",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64 popcount (search), f64-accumulated f32 (rerank)", "data": "synthetic",
        "cold_store": "pinned host memory" if args.cold_host else "HBM",
        "config": {"workload": f"{w.name}: {w.n} x {w.d} {w.kind} unit-norm vectors, {w.nq} queries, "
                               f"graph R={w.R} L={w.L} alpha={w.alpha}, k={k}, ef={ef}"},
        "recall_at_10": recall,
        "bq_dist_evals_per_s": float(n_eval.sum() / (search_ms * 1e-3)),
        "dist_evals_per_query": {"algorithm": float(n_eval.mean()), "as_timed": float(n_eval_run.mean())},
        "stage_ms": {"query_encode": float(stage_ms[:, 0].mean()), "beam_search": search_ms,
                     "rerank": float(stage_ms[:, 2].mean())},
        "algorithmic_bytes_per_step": {"query_encode": encq_bytes, "beam_search": search_bytes,
                                       "rerank": rerank_bytes},
        "whole_path_GBps": (encq_bytes + search_bytes + rerank_bytes) / (ms_per_step * 1e-3) / 1e9,
        "encode_base": {"ms": enc_ms, "GBps": enc_bytes / enc_ms / 1e6},
        "index_code_layout": {"plane_words": layout[0], "row_stride_words": layout[1], "split": split is not None}, "graph_build_s": t_graph, "graph_from": args.graph, "encoding": args.encoding,
        "random_row_gather_ceiling_GBps": gather_gbps,
        "search_bytes_line_granular": int(4 * w.R * n_exp.sum() + (2 * 128 if code_b % 128 else code_b) * n_eval.sum())
        if code_b <= 256 else None,
        "parity_with_oracle_on_sample": parity,
        "rerank_inside_search_kernel": fused,
        "random_line_gather_ceiling_GBps": gather_line_gbps,
        "roofline": {"kernel": "beam_search_kernel (search + rerank)" if fused else "beam_search_kernel", "bound": "hbm",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "basis": "counter traffic (L2-to-fabric bytes) / kernel time" if traffic_gbps
                              else "algorithmic bytes / kernel time (no current counter file for this run)",
                     "traffic": traffic, "traffic_GBps": traffic_gbps, "traffic_commit": traffic_commit,
                     "traffic_file_stale": traffic_stale,
                     "algorithmic_bytes": kernel_bytes, "algorithmic_GBps": algorithmic_gbps,
                     "algorithmic_frac": algorithmic_gbps / HBM_PEAK_GBPS, "l2_hit_rate": l2_hit,
                     "line_rate_frac_of_probe": traffic_gbps / gather_line_gbps if traffic_gbps and gather_line_gbps else None,
                     "kernel_ms": search_ms},
        "cpu_baseline": cpu,
        "bq_scan": scan,
        "gpu_graph_build": gpu_build,
        "compatible_regime_companion": companion,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
