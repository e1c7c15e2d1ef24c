#!/usr/bin/env python3
"""Benchmark of the CTkvr decode hot path on one MI355X.

A "step" is one pass of the whole path -- centroid scoring, top-C' probe,
list gather + dedup, exact q.K over the recalled keys, top-rho' rerank, sparse
attention -- over one batch of decode queries of the named synthetic workload,
with the index, the paged KV cache and all queries already resident in HBM.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg3|cfg4|cfg1]

prints ONE JSON line.  The CPU oracle is timed beside it on a bounded sample
(reported baseline, not the target).  Everything is single-GPU: --gpus above 1
exits with a message.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def step_bytes(wl, C, L_sum_per_seq, e):
    """Algorithmic bytes one decode step must move for one sequence: centroid table
    and inverse norms, the probed lists, each recalled key row once per KV head,
    block-table entries, the selected value rows, q in and o out."""
    h, g, d = wl.h, wl.g, wl.d
    return (h * C * d * e + h * C * 4 + g * wl.n_probe * wl.list_len * 4 + L_sum_per_seq * d * e
            + (L_sum_per_seq + g * wl.top_k) * 4 + g * wl.top_k * d * e + 2 * h * d * 4)


def bench_build(args, wl, emit=True):
    """Index build only (Algorithm 1 lines 1-4): a "step" is one complete build."""
    import torch
    import paper_2512_15550_amd as ck
    from ctkvr_inputs import gen_batch
    from ctkvr_inputs import device as H
    K = args.steps if args.steps is not None else 3
    W = min(args.warmup, 1)
    bt = gen_batch(wl, n_decode=1, full_walk=bool(args.kmeans))
    db = H.device_batch(bt)
    res = {}
    if args.kmeans:   # k-means centroid mode: 10 Lloyd iterations from k-means++ positions (drawn on the host, untimed)
        from ctkvr_inputs.kmeans_init import centroid_positions, kmeanspp_for_sequence
        t0 = time.time()
        if emit:
            init = np.stack([kmeanspp_for_sequence(sq.q_full, wl.g, wl.centroids_of(sq.s), seed=sq.seed) for sq in bt.seqs])
        else:   # riding along in the default line: seeded random start positions (k-means++ takes minutes on the host
                # and is outside the timed region either way; the Lloyd iterations cost the same from any start)
            init = np.stack([centroid_positions("random", sq.s, wl.centroids_of(sq.s), wl.g, seed=sq.seed) for sq in bt.seqs])
        t_pp = time.time() - t0
        qf, cu = H.device_full_queries(bt)
        ip = torch.from_numpy(np.ascontiguousarray(init, np.int32)).cuda()
        for iters in (0, 10):
            p = H.params_of(wl, build_algo=ck.BUILD_MFMA, centroid_mode=ck.KMEANS, kmeans_iters=iters)
            ck.ctkvr_free(ck.ctkvr_build_index(p, qf, cu, False, db.k_pages, db.block_table, db.ctx_lens, init_pos=ip))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(K):
                ck.ctkvr_free(ck.ctkvr_build_index(p, qf, cu, False, db.k_pages, db.block_table, db.ctx_lens, init_pos=ip))
            torch.cuda.synchronize()
            res[f"kmeans{iters}"] = (time.perf_counter() - t0) / K * 1e3
        lloyd_ms = res["kmeans10"] - res["kmeans0"]
        lloyd_flops = sum(10 * 2.0 * s * wl.centroids_of(s) * wl.h * wl.d for s in wl.ctx_lens)
        res["kmeans"] = {"build_ms_with_10_lloyd_iterations": res["kmeans10"], "lloyd_ms": lloyd_ms,
                         "assignment_gemm_flops": lloyd_flops, "lloyd_TFLOPs": lloyd_flops / (lloyd_ms * 1e-3) / 1e12,
                         "lloyd_mfma_frac": lloyd_flops / (lloyd_ms * 1e-3) / 1e12 / 2500.0,
                         "start_positions": "k-means++ (host)" if emit else "seeded random", "start_positions_host_s": t_pp}
    for name, algo in (("mfma", ck.BUILD_MFMA), ("exact", ck.BUILD_EXACT)):
        p = H.params_of(wl, build_algo=algo)
        for _ in range(W):
            ck.ctkvr_free(ck.ctkvr_build_index(p, db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            ck.ctkvr_free(ck.ctkvr_build_index(p, db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens))
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) / K * 1e3
        if name == "mfma":   # which way the lists were chosen (untimed extra build)
            probe = ck.ctkvr_build_index(p, db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens)
            by_cand, redone = ck.ctkvr_index_build_route(probe)
            res["route"] = {"by_candidates": by_cand, "chunks_redone": redone}
            ck.ctkvr_free(probe)
    flops = sum(2.0 * wl.h * wl.centroids_of(s) * s * wl.d for s in wl.ctx_lens)
    tf = flops / (res["mfma"] * 1e-3) / 1e12
    rec = {"metric": "index build ms (centroid table + top-rho inverted lists)", "value": res["mfma"], "unit": "ms",
           "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": res["mfma"], "higher_is_better": False, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": wl.name, "ctx_lens": wl.ctx_lens, "q_heads": wl.h, "kv_heads": wl.g,
                      "centroids": wl.n_centroids, "list_len": wl.list_len, "build_algo": "mfma"},
           "exact_build_ms": res["exact"], "score_gemm_flops": flops, "mfma_build_route": res["route"], "kmeans": res.get("kmeans"),
           "roofline": ({"kernel": "Lloyd iterations (kmeans_assign_kernel GEMM + counting-sort update)", "bound": "mfma",
                         "achieved": res["kmeans"]["lloyd_TFLOPs"], "peak": 2500.0, "unit": "TFLOP/s",
                         "frac": res["kmeans"]["lloyd_TFLOPs"] / 2500.0, "traffic": None} if args.kmeans else
                        {"kernel": "whole build (score GEMM + denominators + selection)", "bound": "mfma", "achieved": tf,
                         "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0, "traffic": None}),
           "cpu_baseline": None}
    if not emit:
        return {"mfma_build_ms": res["mfma"], "exact_build_ms": res["exact"], "score_gemm_flops": flops,
                "mfma_build_route": res["route"], "whole_build_TFLOPs": tf, "whole_build_mfma_frac": tf / 2500.0, "kmeans": res.get("kmeans"),
                "config": rec["config"]}
    print(json.dumps(rec))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"])
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain device copy of known size instead (scale for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--kmeans", action="store_true", help="cfg5 only: also time the k-means centroid mode")
    ap.add_argument("--cpu-steps", type=int, default=None, help="decode steps of the CPU oracle sample (0 = skip)")
    ap.add_argument("--dcu", action="store_true",
                    help="every timed step is followed by the dynamic centroid update (Algorithm 2 line 12)")
    ap.add_argument("--window", default="", help="N_INIT,N_LOCAL: build and decode with a resident window (Algorithm 2 lines 10-11)")
    ap.add_argument("--sweep", default="", choices=["", "cprime", "c"],
                    help="step time against the number of probed centroids C' or of centroids C, around the paper's own "
                         "operating point (32K, C = 2048, C' = 4, rho = 2.5 rho' = 2560), as in its appendix tables of "
                         "throughput against C and against C'")
    ap.add_argument("--skip-128k", action="store_true", help="cfg2 only: do not append the other workloads' figures")
    ap.add_argument("--repeats", type=int, default=7, help="timed repeats of the K steps (median and p95 are reported)")
    ap.add_argument("--path", default="", choices=["", "auto", "staged", "fused"], help="how a decode step is launched")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if args.calibrate_copy:
        # 1 GiB read + 1 GiB written per launch of torch's copy kernel, 8 launches (the first is a warm-up)
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 8
        print(json.dumps({"calibrate_copy": True, "bytes_read_per_launch": src.numel() * 4,
                          "bytes_written_per_launch": src.numel() * 4, "launches": 8,
                          "GBps_read_plus_write": 2 * src.numel() * 4 / dt / 1e9}))
        return
    import paper_2512_15550_amd as ck
    from ctkvr_inputs import workload

    ck.load_library()
    torch.cuda.set_device(0)
    if args.sweep:
        import dataclasses
        base = workload("paper_llama")
        values = [1, 2, 4, 8, 16, 32] if args.sweep == "cprime" else [256, 512, 1024, 2048, 4096]
        points = []
        for v in values:
            wl = dataclasses.replace(base, n_probe=v) if args.sweep == "cprime" else dataclasses.replace(base, n_centroids=v)
            r = bench_decode(args, wl, args.steps if args.steps is not None else 64, 0)
            points.append({"C": wl.n_centroids, "n_probe": wl.n_probe, "us_per_step": r["value"], "L_recall_mean": r["L_recall_mean"],
                           "alpha": r["alpha"], "achieved_GBps": r["achieved_GBps"], "stage_us": r["stage_us"]})
        print(json.dumps({"metric": "decode retrieval+sparse-attn us/step against " + ("C'" if args.sweep == "cprime" else "C"),
                          "unit": "us/step", "n_gpus": 1, "data": "synthetic", "higher_is_better": False,
                          "config": {"workload": "paper_llama", "ctx_len": 32768, "list_len": base.list_len, "top_k": base.top_k},
                          "points": points}))
        return
    wl = workload(args.workload)
    if wl.n_decode == 0:
        return bench_build(args, wl)
    rec = bench_decode(args, wl, args.steps, args.cpu_steps)
    if wl.name == "cfg2" and not args.skip_128k:
        # the metric is quoted at 32K and at 128K; the ragged batch and the index build ride along in the same line
        keep = ("value", "us_per_step_p95", "unit", "steps", "repeats", "config", "tokens_per_s", "achieved_GBps", "hbm_frac",
                "algorithmic_bytes_per_step", "L_recall_mean", "alpha", "index_build_ms", "decode_path", "stage_us",
                "phase_us_first_block", "roofline")
        r3 = bench_decode(args, workload("cfg3"), args.steps, 0)
        rec["at_128k"] = {k: r3[k] for k in keep}
        r4 = bench_decode(args, workload("cfg4"), args.steps, 0)
        rec["at_cfg4"] = {k: r4[k] for k in keep}
        import copy
        a5 = copy.copy(args)
        a5.steps, a5.kmeans = 3, True
        rec["build_cfg5"] = bench_build(a5, workload("cfg5"), emit=False)
        # the rows next on the path, as plain step times: the resident window, the dynamic centroid update, and the
        # paper's own operating point on both head shapes and at its 4 % budget
        rec["variants"] = {}
        for name, wname, window, dcu in (("cfg2_window_128_512", "cfg2", "128,512", False), ("cfg2_centroid_update", "cfg2", "", True),
                                         ("cfg3_window_128_512", "cfg3", "128,512", False), ("cfg3_centroid_update", "cfg3", "", True),
                                         ("paper_llama", "paper_llama", "", False), ("paper_yi", "paper_yi", "", False),
                                         ("paper_budget4", "paper_budget4", "", False)):
            av = copy.copy(args)
            av.window, av.dcu, av.repeats = window, dcu, 5
            rv = bench_decode(av, workload(wname), 64, 0)
            rec["variants"][name] = {k: rv[k] for k in ("value", "us_per_step_p95", "unit", "steps", "repeats", "config")}
    print(json.dumps(rec))


def bench_decode(args, wl, steps, cpu_steps):
    """K timed decode steps of one workload; returns the record (not printed)."""
    import torch
    import paper_2512_15550_amd as ck
    from ctkvr_inputs import gen_batch
    from ctkvr_inputs import device as H   # device upload helpers; the CPU checker is imported in the cpu_baseline leg only

    K = steps if steps is not None else max(1, wl.n_decode)
    W = args.warmup
    n_q = max(1, min(wl.n_decode, K))
    t0 = time.time()
    bt = gen_batch(wl, n_decode=n_q)
    db = H.device_batch(bt)
    B, h, g, d = wl.batch, wl.h, wl.g, wl.d
    e = 2 if wl.dtype == "bf16" else 4
    q_all = H.to_dev(np.stack([np.stack([sq.q_decode[i] for sq in bt.seqs]) for i in range(n_q)]), wl)  # [n_q][B][h][d]
    t_gen = time.time() - t0

    torch.cuda.synchronize()
    t0 = time.time()
    n_init, n_local = (int(x) for x in args.window.split(",")) if args.window else (0, 0)
    idx = ck.ctkvr_build_index(H.params_of(wl, n_init=n_init, n_local=n_local), db.q_prefill, db.cu_seqlens, True,
                               db.k_pages, db.block_table, db.ctx_lens)
    torch.cuda.synchronize()
    build_ms = (time.time() - t0) * 1e3
    if args.path:
        ck.ctkvr_index_set_decode_path(idx, {"auto": ck.PATH_AUTO, "staged": ck.PATH_STAGED, "fused": ck.PATH_FUSED}[args.path])

    out = torch.empty((B, h, d), dtype=torch.float32, device="cuda")
    ncand = torch.zeros((K, B, g), dtype=torch.int32, device="cuda")

    def run_steps(n, first=0, record=True):
        for i in range(n):
            ck.ctkvr_decode_step(idx, q_all[(first + i) % n_q], db.k_pages, db.v_pages, db.block_table, out,
                                 out_ncand=ncand[i] if record else None)
            if args.dcu:
                ck.ctkvr_centroid_update(idx, q_all[(first + i) % n_q])

    # ---- warm-up -----------------------------------------------------------------
    run_steps(W, record=False)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps -------------------------------------------
    mode = args.mode
    graph = None
    if mode == "graph":
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    run_steps(K)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph.replay()            # untimed: first replay uploads the graph
            torch.cuda.synchronize()
        except Exception as exc:      # capture not possible: time plain launches instead
            print(f"bench.py: graph capture failed ({exc}); timing eager launches", file=sys.stderr)
            graph, mode = None, "eager"
    # R repeats of the same K steps, each bracketed by a synchronize on both sides (wall clock) and by a pair of
    # HIP events on the launch stream; value = the median repeat
    R = max(1, args.repeats)
    wall, evt = [], []
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(R):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        if graph is not None:
            graph.replay()
        else:
            run_steps(K)
        ev1.record()
        torch.cuda.synchronize()
        wall.append((time.perf_counter() - t0) / K * 1e6)
        evt.append(ev0.elapsed_time(ev1) / K * 1e3)
    ck.ctkvr_index_check(idx)
    us_per_step = float(np.median(wall))
    dt = us_per_step * K * 1e-6
    ev_us = float(np.median(evt))
    out_timed = out.clone()
    L = ncand.cpu().numpy().astype(np.int64)          # [K][B][g]

    # the last step's output must equal an eager run of the same query (graph replays are checked, not trusted)
    # (not with --dcu: the index has moved on since that step)
    ck.ctkvr_decode_step(idx, q_all[(K - 1) % n_q], db.k_pages, db.v_pages, db.block_table, out)
    torch.cuda.synchronize()
    if not args.dcu and not torch.equal(out, out_timed):
        raise SystemExit("bench.py: timed-region output differs from an eager re-run of the same step")

    # ---- per-kernel durations with HIP events on the launch stream, same K steps ----
    fused = ck.ctkvr_index_decode_path(idx) == ck.PATH_FUSED
    ck.ctkvr_profile_enable(idx, K)
    run_steps(K, record=False)
    stage_ms = ck.ctkvr_profile_collect(idx, K)
    ck.ctkvr_profile_enable(idx, 0)
    stage_us = {n: float(stage_ms[:, i].mean() * 1e3) for i, n in enumerate(ck.STAGE_NAMES)}
    floor_us = ck.ctkvr_measure_dispatch_floor(200)     # an empty kernel behind another one, in a graph, this run

    # ---- bytes --------------------------------------------------------------------
    L_step = L.sum(axis=2)                             # [K][B] recalled keys per sequence (all KV heads)
    bytes_step = np.array([sum(step_bytes(wl, wl.centroids_of(s), int(L_step[k, b]), e)
                               for b, s in enumerate(wl.ctx_lens)) for k in range(K)], dtype=np.float64)
    achieved = float(bytes_step.mean() / (dt / K)) / 1e9
    phases = None
    if fused:
        # ONE launch per step: the dominant kernel is the step.  Its average duration is the event-bracketed time
        # of the K back-to-back launches of the timed region divided by K, i.e. duration plus the dispatch gap
        # (floor_us bounds the gap from above), so the rate below is on the low side.
        kernel, kbytes, k_us, k_between = "decode_fused_kernel", float(bytes_step.mean()), ev_us, ev_us
        stage_us = {"fused_step": stage_us["centroid_cos"], "null": stage_us["null"]}
        ck.ctkvr_profile_phases(idx, True)
        run_steps(min(K, 8), record=False)
        t = ck.ctkvr_profile_phases(idx, False).astype(np.float64)
        names = ["cos", "probe+gather+score", "ranks+denominators", "keys+histogram", "classify+attend"]
        phases = {n: float((t[i + 1] - t[i]) / 100.0) for i, n in enumerate(names)}   # 100 MHz ticks -> us
        phases["select+merge"] = float((t[7] - t[5]) / 100.0)
        phases["own_work_before_each_barrier"] = [float((t[8 + i] - t[i]) / 100.0) for i in range(5)]
        phases["detail_us_since_entry"] = {str(i): float((t[i] - t[0]) / 100.0) for i in range(64) if t[i] > 0}
    else:
        # a pair of events around a kernel that does nothing reads stage_us["null"]; that kernel itself lasts about
        # floor_us; the rest is the bracketing's own cost
        kernel = "recall_score_kernel"
        kbytes = float(L.sum(axis=(1, 2)).mean()) * (d * e + 4)   # key row + its physical row index
        event_overhead = max(0.0, stage_us["null"] - floor_us)
        k_between = stage_us["score"]
        k_us = max(k_between - event_overhead, 1e-3)
    k_gbps = kbytes / (k_us * 1e-6) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{kernel}_{wl.name}.json")
    if os.path.exists(tpath):
        with open(tpath) as fh:
            traffic = json.load(fh)

    # ---- CPU oracle on a bounded sample (reported baseline) -------------------------
    cpu = None
    n_cpu = cpu_steps if cpu_steps is not None else {"cfg1": 4, "cfg2": 64, "cfg3": 2, "cfg4": 2}.get(wl.name, 4)
    if n_cpu > 0:
        import oracle
        nb = B if wl.name in ("cfg1", "cfg2") else 1   # long configs: first sequence only, scaled to the batch
        t0 = time.time()
        Qc = [oracle.centroids_last_c(sq.q_tail, wl.centroids_of(sq.s)) for sq in bt.seqs[:nb]]
        if wl.name in ("cfg1", "cfg2"):
            lists = [oracle.build_lists(sq.K, q, wl.list_len) for sq, q in zip(bt.seqs[:nb], Qc)]
        else:   # building the full oracle index would take minutes: only the probed lists are built, untimed
            lists = None
        t_obuild = time.time() - t0
        n_cpu = min(n_cpu, n_q)
        t_dec = 0.0
        for i in range(n_cpu):
            for b in range(nb):
                sq = bt.seqs[b]
                qv = sq.q_decode[i]
                if lists is not None:
                    t1 = time.perf_counter()
                    oracle.decode_step(qv, sq.K, sq.V, Qc[b], lists[b], wl.n_probe, wl.top_k)
                    t_dec += time.perf_counter() - t1
                else:
                    t1 = time.perf_counter()
                    cosv, probe = oracle.recall(qv, Qc[b], g, wl.n_probe)
                    t_dec += time.perf_counter() - t1
                    pairs = np.array([[kv, j] for kv in range(g) for j in probe[kv]], np.int32)
                    lst = np.zeros((g, Qc[b].shape[1], wl.list_len), np.int32)
                    built = oracle.build_lists(sq.K, Qc[b], wl.list_len, pairs=pairs)
                    for (kv, j), row in zip(pairs, built):
                        lst[kv, j] = row
                    t1 = time.perf_counter()
                    oracle.rerank_attend(qv, sq.K, sq.V, lst, probe, wl.top_k)
                    t_dec += time.perf_counter() - t1
        cpu_us = t_dec / n_cpu * 1e6 * (B / nb)
        # the same oracle on ONE thread, first step only
        one = None
        if lists is not None:
            nthr = oracle.num_threads()
            oracle.set_threads(1)
            t1 = time.perf_counter()
            for b in range(nb):
                sq = bt.seqs[b]
                oracle.decode_step(sq.q_decode[0], sq.K, sq.V, Qc[b], lists[b], wl.n_probe, wl.top_k)
            one = (time.perf_counter() - t1) * 1e6 * (B / nb)
            oracle.set_threads(nthr)
        cpu = {"value": cpu_us, "unit": "us/step", "cores": oracle.num_threads(), "kind": "oracle",
               "one_thread_us_per_step": one, "cpu_model": cpu_model(),
               "sample": f"{n_cpu} decode steps of {wl.name} on {nb} of {B} sequences"
                         + ("" if nb == B else f", scaled x{B // nb}") + f"; oracle index build {t_obuild:.1f} s not included"
                         + ("; one-thread figure from the first step" if one is not None else "")}

    rec = {
        "metric": "decode retrieval+sparse-attn us/step (and achieved HBM GB/s)",
        "value": us_per_step, "unit": "us/step", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": us_per_step / 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "storage_dtype": wl.dtype, "batch": B, "q_heads": h, "kv_heads": g,
                   "ctx_lens": wl.ctx_lens if B <= 4 else [min(wl.ctx_lens), max(wl.ctx_lens)],
                   "centroids": wl.n_centroids or f"ctx/{wl.centroid_div}", "n_probe": wl.n_probe,
                   "list_len": wl.list_len, "top_k": wl.top_k, "launch": mode, "centroid_update": bool(args.dcu),
                   "window": [n_init, n_local]},
        "us_per_step_p95": float(np.percentile(wall, 95)), "us_per_step_min": float(np.min(wall)), "repeats": R,
        "us_per_step_repeats": [float(x) for x in wall], "us_per_step_between_events": ev_us,
        "tokens_per_s": B / (dt / K), "tokens_per_s_32_layers": B / (dt / K) / 32,
        "achieved_GBps": achieved, "hbm_frac": achieved / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_step": float(bytes_step.mean()),
        "L_recall_mean": float(L.mean()), "alpha": float(L.mean()) / (wl.n_probe * wl.list_len),
        "index_build_ms": build_ms, "decode_path": "fused" if fused else "staged", "stage_us": stage_us,
        "phase_us_first_block": phases, "dispatch_floor_us": floor_us,
        "roofline": {"kernel": kernel, "bound": "hbm", "achieved": k_gbps, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": k_gbps / HBM_PEAK_GBPS,
                     "traffic": traffic.get("traffic_bytes_per_launch") if traffic else None,
                     "traffic_from_profile": traffic, "bytes_per_launch": kbytes, "avg_us": k_us,
                     "avg_us_between_events": k_between},
        "cpu_baseline": cpu,
        "input_gen_s": t_gen,
    }
    ck.ctkvr_free(idx)
    del db, q_all, out, ncand, idx
    torch.cuda.empty_cache()
    return rec


if __name__ == "__main__":
    main()
