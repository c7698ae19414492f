#!/usr/bin/env python3
"""Benchmark of the W4A8-FP linear-layer path on one MI355X.

A step is one pass of the hot path over one batch: fq_quantize_act (bf16 -> E4M3 + row scales)
followed by fq_w4a8_gemm on weights packed once beforehand (packing is offline, once per weight).
All inputs are synthetic (seeded) and resident in HBM before the timed region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

Prints one JSON line: whole-step throughput (`value`: median over REPS timed regions of K steps
each), the roofline figure of the GEMM call measured with HIP events around replays of a graph
that holds only the GEMM calls (REPS repetitions of at least MIN_LAUNCHES launches after a
warm-up of WARM_MS of replays; `frac` from the median, the best beside it), the small-M figures
for M = 1, 4, 16, 64 with a plain streaming read of the same weights beside them, and the CPU
oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP8_TFLOPS = 5033.0      # 256 CU x 2.4 GHz x 8192 flop/clk/CU, dense FP8 MFMA
PEAK_HBM_GBPS = 8000.0
DEFAULT_WORKLOAD = "c2_l2_7b_gateup"
DECODE_COPIES = 12            # rotating weight copies so that small-M launches read HBM, not cache
MID_COPIES = 6                # rotating weight copies for 64 < M <= 512
LARGE_GRAPH_STEPS = 10        # steps per captured graph at large M (one copy of the weights: they do not fit a cache)
REPS = 5                      # timed repetitions; median and best are reported
MIN_LAUNCHES = 50             # GEMM launches per repetition of the kernel timing (500 at small M), whatever --steps says
MIN_LAUNCHES_SMALL = 500
WARM_MS = 100.0               # warm-up: this many milliseconds of graph replays before every timed series


def _traffic_from_profiles(workload: str):
    """HBM bytes per GEMM launch measured with rocprofv3 --pmc, if a summary records them."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt")) +
                       glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        for line in open(path):
            m = re.match(r"\s*TRAFFIC_BYTES_PER_LAUNCH\s+(\S+)\s+([0-9.eE+]+)", line)
            if m and m.group(1) == workload:
                return float(m.group(2))
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true", help="skip the extra small-M (HBM-bound) figure")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the brief timing of the other large-M configurations (c3, c4a, c4b, fused gate/up)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="only run a plain device-to-device copy of BYTES bytes three times (reference "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the W4A8-FP GEMM of one linear layer on one "
              "MI355X); --gpus %d is not supported." % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2505_20839_amd import binding as fq, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.empty(args.copy_calibration, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": args.copy_calibration, "copies": 3}))
        return 0
    fq.lib()

    def upload(name):
        w = workloads.WORKLOADS[name]
        d = workloads.draw_workload(name)
        X = torch.from_numpy(d["X_bf16"].view(np.int16)).cuda().view(torch.bfloat16)
        packed = fq.fq_pack_weights(torch.from_numpy(d["q"]).cuda())
        gs = torch.from_numpy(d["gscale"]).cuda()
        return w, d, X, packed, gs

    def timed_series(side, graph, replays):
        """WARM_MS of replays, then REPS timed regions of `replays` replays each, every region bracketed by a
        stream synchronisation; returns (wall seconds per region, HIP-event seconds per region) as lists."""
        t_end = time.perf_counter() + WARM_MS * 1e-3
        while time.perf_counter() < t_end:
            for _ in range(4):
                graph.replay()
            side.synchronize()
        walls, evs = [], []
        for _ in range(REPS):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            side.synchronize()
            t0 = time.perf_counter()
            e0.record(side)
            for _ in range(replays):
                graph.replay()
            e1.record(side)
            side.synchronize()
            walls.append(time.perf_counter() - t0)
            evs.append(e0.elapsed_time(e1) * 1e-3)
        return walls, evs

    def run(name, steps, warmup, copies, graph_steps, with_read_floor=False):
        """Times `steps` steps, REPS times over; returns the workload, its inputs, and per-repetition
        seconds per step / per GEMM call / per quantiser call (lists of REPS values).

        A step is two or three short kernels, faster than Python can launch them one by one, so
        `graph_steps` steps are captured into a HIP graph and the graph is replayed (small M: each step
        of a graph on its own copy of the weights, `copies` in all, so that the weights come from HBM).
        The GEMM's mean duration comes from a second graph that holds only the GEMM calls, the
        quantiser's from a third."""
        w, d, X, packed, gs = upload(name)
        packs = [packed] + [packed.clone() for _ in range(copies - 1)]
        gss = [gs] + [gs.clone() for _ in range(copies - 1)]
        swiglu = w.epilogue == "swiglu"
        Y = torch.empty((w.M, w.N // 2 if swiglu else w.N), dtype=torch.bfloat16, device="cuda")
        gemm_fn = fq.fq_w4a8_gemm_swiglu if swiglu else fq.fq_w4a8_gemm
        if w.epilogue == "add":
            # the residual stream is updated in place, step after step (its values grow; timing only)
            R = torch.from_numpy(workloads.draw_residual(w.M, w.N, scale=workloads.RESIDUAL_SCALE, seed=w.seed)
                                 .view(np.int16)).cuda().view(torch.bfloat16)
            Y = R
            gemm_fn = lambda *a, **k: fq.fq_w4a8_gemm_add(*a, R, **k)   # noqa: E731
        need = fq.fq_w4a8_gemm_workspace_bytes(w.M, w.N, w.K)
        ws = torch.empty((max(need, 16),), dtype=torch.uint8, device="cuda")

        def gemm(A, s, i):
            gemm_fn(A, s, packs[i % copies], gss[i % copies], d["w_tscale"], w.N, out=Y, workspace=ws,
                    workspace_prepared=need > 0)

        # M <= 6, K <= 4096: quantiser and GEMM are one kernel (fq_w4a8_linear_ws, no workspace)
        fused = w.epilogue == "none" and fq.fq_w4a8_linear_workspace_bytes(w.M, w.N, w.K) == 0

        def step(i):
            if fused:
                fq.fq_w4a8_linear(X, packs[i % copies], gss[i % copies], d["w_tscale"], w.N, out=Y)
                return
            # large M: the quantiser also prepares the GEMM's workspace (fq_quantize_act_ws)
            A, s = fq.fq_quantize_act(X, workspace=ws if need > 0 else None)
            gemm(A, s, i)

        A_last, s_last = fq.fq_quantize_act(X, workspace=ws if need > 0 else None)   # operands of the GEMM-only graph
        for i in range(max(warmup, 1)):
            step(i)
        torch.cuda.synchronize()

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            g_steps = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_steps, stream=side):
                for i in range(graph_steps):
                    step(i)
            g_gemm = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_gemm, stream=side):
                for i in range(graph_steps):
                    gemm(A_last, s_last, i)
            g_quant = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_quant, stream=side):
                for i in range(graph_steps):
                    fq.fq_quantize_act(X, workspace=ws if need > 0 else None)
            reps = max(1, (steps + graph_steps - 1) // graph_steps)
            min_launches = MIN_LAUNCHES_SMALL if w.M <= 64 else MIN_LAUNCHES
            kreps = max(reps, (min_launches + graph_steps - 1) // graph_steps)

            wall, _ = timed_series(side, g_steps, reps)
            _, gemm_all = timed_series(side, g_gemm, kreps)
            _, quant_all = timed_series(side, g_quant, kreps)
            read_all = None
            if with_read_floor:                            # a kernel that only reads the same weights, same rotation
                sink = fq.fq_diag_stream_read(packs[0])
                g_read = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g_read, stream=side):
                    for i in range(graph_steps):
                        fq.fq_diag_stream_read(packs[i % copies], sink)   # (98.5 % of the bytes: the scale bytes are left out)
                _, read_all = timed_series(side, g_read, kreps)
        torch.cuda.current_stream().wait_stream(side)
        n, nk = reps * graph_steps, kreps * graph_steps
        per = lambda series, cnt: None if series is None else [t / cnt for t in series]   # noqa: E731
        return {"w": w, "d": d, "steps": n, "step_s": per(wall, n), "gemm_s": per(gemm_all, nk),
                "quant_s": per(quant_all, nk), "read_s": per(read_all, nk), "kernel_launches": nk}

    def table_mode(wl):
        """The paper's table mode (fq_w4a8_gemm_lut: weights rounded to E4M3(q * sigma), no per-group scaling) on
        workload `wl`: GEMM-call duration measured like the exact mode's, and how far its result lies from the
        exact mode's on the same operands (relative Frobenius distance of the two bf16 outputs)."""
        w, d, X, packed, gs = upload(wl)
        A, a_s = fq.fq_quantize_act(X)
        Yl = fq.fq_w4a8_gemm_lut(A, a_s, packed, gs, d["w_tscale"], w.N)
        Ye = fq.fq_w4a8_gemm(A, a_s, packed, gs, d["w_tscale"], w.N)
        torch.cuda.synchronize()
        rel = float((Yl.float() - Ye.float()).norm() / Ye.float().norm())
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for _ in range(LARGE_GRAPH_STEPS):
                    fq.fq_w4a8_gemm_lut(A, a_s, packed, gs, d["w_tscale"], w.N, out=Yl)
            _, ev = timed_series(side, g, MIN_LAUNCHES // LARGE_GRAPH_STEPS)
        torch.cuda.current_stream().wait_stream(side)
        per = sorted(t / MIN_LAUNCHES for t in ev)
        flop = 2.0 * w.M * w.N * w.K
        return {"workload": wl, "kernel": "fq_gemm_large_lut_kernel", "kernel_us": per[len(per) // 2] * 1e6,
                "kernel_us_best": per[0] * 1e6, "gemm_TFLOPs": flop / per[len(per) // 2] / 1e12,
                "frac_mfma_peak": flop / per[len(per) // 2] / 1e12 / PEAK_FP8_TFLOPS,
                "rel_frobenius_distance_from_exact_mode": rel}

    def ffn_chain(wl="ffn_l2_7b_gateup_swiglu"):
        """The gate/up layer with its fused epilogue followed by the quantisation of its output for the down
        projection: the separate quantiser (fq_w4a8_gemm_swiglu_ws + fq_quantize_act_ws, which searches each row for
        its largest magnitude) against fq_w4a8_gemm_swiglu_quant_ws (row maxima raised by the GEMM's epilogue, then an
        element-wise kernel); both leave the same codes, scales and prepared workspace."""
        w, d, X, packed, gs = upload(wl)
        NH = w.N // 2
        need = fq.fq_w4a8_gemm_workspace_bytes(w.M, w.N, w.K)
        ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
        A, a_s = fq.fq_quantize_act(X, workspace=ws)
        ws_next = torch.empty((fq.fq_w4a8_gemm_workspace_bytes(w.M, 4096, NH),), dtype=torch.uint8, device="cuda")
        H = torch.empty((w.M, NH), dtype=torch.bfloat16, device="cuda")

        def separate():
            fq.fq_w4a8_gemm_swiglu(A, a_s, packed, gs, d["w_tscale"], w.N, out=H, workspace=ws, workspace_prepared=True)
            fq.fq_quantize_act(H, workspace=ws_next)

        def fused():
            fq.fq_w4a8_gemm_swiglu_quant(A, a_s, packed, gs, d["w_tscale"], w.N, out=H, workspace=ws,
                                         workspace_prepared=True, next_workspace=ws_next)

        res = {"workload": wl, "M": w.M, "N": w.N, "K": w.K}
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for key, fn in (("separate_quantiser_us", separate), ("fused_row_maximum_us", fused)):
                fn()
                side.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    for _ in range(LARGE_GRAPH_STEPS):
                        fn()
                _, ev = timed_series(side, g, MIN_LAUNCHES // LARGE_GRAPH_STEPS)
                per = sorted(t / MIN_LAUNCHES for t in ev)
                res[key] = per[len(per) // 2] * 1e6
                res[key + "_best"] = per[0] * 1e6
                del g
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.empty_cache()
        return res

    def attention_operands(H=128, R=4, T=4096):
        """Decode attention operands on an INT4 key/value cache (fq_kv4_scores, fq_kv4_output): Llama3-8B, a batch of
        16 sequences x 8 key/value heads, 4 query heads each, 4096 cached tokens; HBM rate of the algorithmic bytes
        (packed cache + scales + FP8 operand + bf16 result), 6 rotating copies of the caches."""
        d = workloads.draw_kv_cache(H, R, T, seed=12)
        to_bf16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)   # noqa: E731
        Qc, qs = fq.fq_quantize_act(to_bf16(d["Q_bf16"].reshape(H * R, 128)))
        Pc, ps = fq.fq_quantize_act(to_bf16(d["P_bf16"].reshape(H * R, T)))
        Qc, qs, Pc, ps = Qc.view(H, R, 128), qs.view(H, R), Pc.view(H, R, T), ps.view(H, R)
        copies = 6
        kps = [fq.fq_kv4_pack(torch.from_numpy(d["Kq"]).cuda(), False) for _ in range(copies)]
        vps = [fq.fq_kv4_pack(torch.from_numpy(d["Vq"]).cuda(), True) for _ in range(copies)]
        ks, vs = torch.from_numpy(d["k_scale"]).cuda(), torch.from_numpy(d["v_scale"]).cuda()
        res = {"H": H, "R": R, "T": T}
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for key, fn, nbytes in (
                    ("fq_kv4_scores", lambda i: fq.fq_kv4_scores(Qc, qs, kps[i % copies], ks, 128 ** -0.5),
                     H * T * 64 + H * T + H * R * 128 + 2 * H * R * T),
                    ("fq_kv4_output", lambda i: fq.fq_kv4_output(Pc, ps, vps[i % copies], vs),
                     H * T * 64 + H * T + H * R * T + 2 * H * R * 128)):
                fn(0)
                side.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    for i in range(copies):
                        fn(i)
                _, ev = timed_series(side, g, 10)
                per = sorted(t / (10 * copies) for t in ev)
                us = per[len(per) // 2] * 1e6
                res[key] = {"us": us, "us_best": per[0] * 1e6, "algorithmic_bytes": nbytes, "GBps": nbytes / us / 1e3,
                            "frac_hbm": nbytes / us / 1e3 / PEAK_HBM_GBPS}
                del g
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.empty_cache()
        return res

    def offline_quantiser(N, K, reps=20):
        """Mean duration of the three offline stages on a synthetic N x K bf16 matrix (graph replays of
        `reps` calls each) and the HBM rate of their algorithmic bytes."""
        W = torch.from_numpy(workloads.draw_weights(N, K, seed=5).view(np.int16)).cuda().view(torch.bfloat16)
        lam = fq.fq_cas_scales(W, 0.02)
        n_pts = int(fq.fq_pts_exponent(W, lam)[0])
        stages = {"fq_cas_scales": (lambda: fq.fq_cas_scales(W, 0.02), 2 * N * K + 4 * K),
                  "fq_pts_exponent": (lambda: fq.fq_pts_exponent(W, lam), 2 * N * K + 4 * K),
                  "fq_quantize_weights": (lambda: fq.fq_quantize_weights(W, lam, n_pts), 3 * N * K + N * K // 128 + 4 * K)}
        out = {"N": N, "K": K, "n_pts": n_pts}
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for key, (fn, nbytes) in stages.items():
                fn()
                side.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    for _ in range(reps):
                        fn()
                g.replay()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                side.synchronize()
                e0.record(side)
                g.replay()
                e1.record(side)
                side.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / reps
                out[key] = {"us": us, "algorithmic_bytes": nbytes, "GBps": nbytes / us / 1e3,
                            "frac_hbm": nbytes / us / 1e3 / PEAK_HBM_GBPS}
                del g
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.empty_cache()
        return out

    import statistics

    def med(xs):
        return statistics.median(xs)

    name = args.workload
    w0 = workloads.WORKLOADS[name]
    decode_like = w0.M <= 64
    steps = args.steps if args.steps is not None else (2000 if decode_like else 200)
    warmup = args.warmup if args.warmup is not None else (50 if decode_like else 20)
    mid = 64 < w0.M <= 512                                # weights dominate the traffic: rotate copies here as well
    r = run(name, steps, warmup, DECODE_COPIES if decode_like else MID_COPIES if mid else 1,
            DECODE_COPIES if decode_like else MID_COPIES if mid else LARGE_GRAPH_STEPS, with_read_floor=decode_like)
    w, d, steps = r["w"], r["d"], r["steps"]
    step_s, gemm_s, quant_s = med(r["step_s"]), med(r["gemm_s"]), med(r["quant_s"])

    flop = 2.0 * w.M * w.N * w.K
    G = w.K // 128
    wbytes = w.N * w.K / 2 + w.N * G                      # packed INT4 + group scales
    swiglu = w.epilogue == "swiglu"
    gemm_bytes = wbytes + w.M * w.K + 4 * w.M + 2 * w.M * (w.N // 2 if swiglu else w.N) \
        + (2 * w.M * w.N if w.epilogue == "add" else 0)
    if decode_like:
        metric, unit = "W4A8 GEMM packed-weight GB/s at small M", "GB/s"
        value = wbytes / step_s / 1e9
        value_best = wbytes / min(r["step_s"]) / 1e9
        roof = {"bound": "hbm", "achieved": wbytes / gemm_s / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                "achieved_best": wbytes / min(r["gemm_s"]) / 1e9}
    else:
        metric = ("W4A8 GEMM TFLOPS (% FP8 MFMA peak) at M=2048; GB/s (% HBM) at M=16" if name == DEFAULT_WORKLOAD
                  else ("W4A8 gate/up GEMM with fused SiLU(gate)*up, TFLOPS at M=%d" if swiglu
                        else "W4A8 GEMM with the residual added in the epilogue, TFLOPS at M=%d" if w.epilogue == "add"
                        else "W4A8 GEMM TFLOPS at M=%d") % w.M)
        unit = "TFLOP/s"
        value = flop / step_s / 1e12
        value_best = flop / min(r["step_s"]) / 1e12
        roof = {"bound": "mfma", "achieved": flop / gemm_s / 1e12, "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s",
                "achieved_best": flop / min(r["gemm_s"]) / 1e12}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["frac_best"] = roof["achieved_best"] / roof["peak"]
    roof["traffic"] = _traffic_from_profiles(name)
    # what one fq_w4a8_gemm call launches: kernel_us is the median duration of the whole call over REPS
    # repetitions of `kernel_launches` launches each
    roof["kernel"] = ("fq_gemm_small16_kernel" if w.M <= 16 else "fq_gemm_smallm_kernel") if decode_like \
        else ("fq_gemm_ksplit_kernel" if fq.fq_w4a8_gemm_plan(w.M, w.N, w.K)["kernel"].startswith("ksplit") else "fq_gemm_large_kernel")
    roof["kernel_us"] = gemm_s * 1e6
    roof["kernel_us_best"] = min(r["gemm_s"]) * 1e6
    roof["kernel_us_all"] = [round(t * 1e6, 3) for t in r["gemm_s"]]
    roof["kernel_launches_per_repetition"] = r["kernel_launches"]
    roof["repetitions"] = REPS
    roof["quantize_us"] = quant_s * 1e6
    roof["algorithmic_bytes"] = gemm_bytes
    if r["read_s"] is not None:
        read_s = med(r["read_s"])
        roof["stream_read_us"] = read_s * 1e6
        roof["frac_of_measured_read"] = read_s / gemm_s

    out = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": step_s * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp8_e4m3 x int4 -> f32", "data": "synthetic",
        "value_best": value_best, "value_all": [(wbytes / t / 1e9) if decode_like else (flop / t / 1e12) for t in r["step_s"]],
        "protocol": "%.0f ms of graph replays as warm-up, then %d timed regions (each bracketed by a stream synchronisation) "
                    "of %d steps; value = median region" % (WARM_MS, REPS, steps),
        "config": {"workload": name, "M": w.M, "N": w.N, "K": w.K, "group": 128,
                   "step": (("fq_w4a8_linear_ws (quantiser and GEMM in one kernel)" if fq.fq_w4a8_linear_workspace_bytes(w.M, w.N, w.K) == 0
                             else "fq_quantize_act + fq_w4a8_gemm") if decode_like else
                            "fq_quantize_act_ws + fq_w4a8_gemm%s_ws (workspace prepared by the quantiser)"
                            % ("_swiglu" if swiglu else "_add" if w.epilogue == "add" else "")) +
                           " (weights packed once, offline)"},
        "roofline": roof,
    }

    def decode_entry(wl):
        """Packed-weight GB/s of the GEMM call at small M over rotating weight copies, and the same bytes read by
        a kernel that does nothing else (the ceiling one launch per GEMM can show at this size)."""
        rd = run(wl, 600, 50, DECODE_COPIES, DECODE_COPIES, with_read_floor=True)
        wd = rd["w"]
        wb = wd.N * wd.K / 2 + wd.N * (wd.K // 128)
        g, g_best, rs = med(rd["gemm_s"]), min(rd["gemm_s"]), med(rd["read_s"])
        torch.cuda.empty_cache()
        return {"workload": wl, "M": wd.M, "kernel": fq.fq_w4a8_gemm_plan(wd.M, wd.N, wd.K)["kernel"],
                "kernel_us": g * 1e6, "kernel_us_best": g_best * 1e6,
                "step_us": med(rd["step_s"]) * 1e6, "weight_GBps": wb / g / 1e9, "frac_hbm": wb / g / 1e9 / PEAK_HBM_GBPS,
                "frac_hbm_best": wb / g_best / 1e9 / PEAK_HBM_GBPS, "stream_read_us": rs * 1e6,
                "stream_read_GBps": wb / rs / 1e9, "frac_of_measured_read": rs / g,
                "launches_per_repetition": rd["kernel_launches"], "repetitions": REPS,
                "weight_copies_rotated": DECODE_COPIES}

    if not decode_like and not args.no_decode:
        # second half of the metric: packed-weight GB/s at M = 16 against the HBM roofline (and M = 1, 4, 64 beside it)
        out["decode_m16"] = decode_entry("c5_decode_m16")
        if not args.no_other_configs:
            out["decode_sweep"] = {wl: decode_entry(wl) for wl in ("c5_decode_m1", "c5_decode_m4", "c5_decode_m64")}

    def mid_entry(wl):
        """The GEMM call between decode and prefill (64 < M <= 512), over rotating weight copies: duration, which
        kernel served it, and both roofline fractions of its algorithmic bytes and operations."""
        rm = run(wl, 120, 12, MID_COPIES, MID_COPIES)
        wm = rm["w"]
        g, g_best = med(rm["gemm_s"]), min(rm["gemm_s"])
        nbytes = wm.N * wm.K / 2 + wm.N * (wm.K // 128) + wm.M * wm.K + 4 * wm.M + 2 * wm.M * wm.N
        fl = 2.0 * wm.M * wm.N * wm.K
        plan = fq.fq_w4a8_gemm_plan(wm.M, wm.N, wm.K)
        torch.cuda.empty_cache()
        return {"M": wm.M, "N": wm.N, "K": wm.K, "kernel": plan["kernel"], "k_slices": plan["ksplit_slices"],
                "kernel_us": g * 1e6, "kernel_us_best": g_best * 1e6, "quantize_us": med(rm["quant_s"]) * 1e6,
                "step_us": med(rm["step_s"]) * 1e6, "algorithmic_GBps": nbytes / g / 1e9,
                "frac_hbm": nbytes / g / 1e9 / PEAK_HBM_GBPS, "gemm_TFLOPs": fl / g / 1e12,
                "frac_mfma_peak": fl / g / 1e12 / PEAK_FP8_TFLOPS, "weight_copies_rotated": MID_COPIES}

    if not args.no_other_configs and not decode_like and name == DEFAULT_WORKLOAD:
        out["mid_m"] = {wl: mid_entry(wl) for wl in ("mid_l3_8b_up_m128", "mid_l3_8b_up_m256", "mid_l3_8b_up_m512",
                                                     "mid_l2_7b_down_m128", "mid_l2_7b_down_m256", "mid_l2_7b_down_m512")}
        others = {}
        for other in ("c3_l2_7b_down", "c4a_l3_8b_qkv", "c4b_l3_8b_up", "ffn_l2_7b_gateup_swiglu",
                      "ffn_l2_7b_down_residual"):
            if other == name:
                continue
            ro = run(other, 50, 5, 1, LARGE_GRAPH_STEPS)
            wo = ro["w"]
            fo = 2.0 * wo.M * wo.N * wo.K
            go = med(ro["gemm_s"])
            others[other] = {"M": wo.M, "N": wo.N, "K": wo.K, "kernel_us": go * 1e6, "kernel_us_best": min(ro["gemm_s"]) * 1e6,
                             "quantize_us": med(ro["quant_s"]) * 1e6, "step_us": med(ro["step_s"]) * 1e6,
                             "gemm_TFLOPs": fo / go / 1e12, "frac_mfma_peak": fo / go / 1e12 / PEAK_FP8_TFLOPS}
            torch.cuda.empty_cache()
        out["other_configs"] = others
        out["table_mode"] = table_mode(name)
        out["ffn_chain"] = ffn_chain()
        out["attention_operands"] = attention_operands()
        # the offline step that produces the weight operands, on the gate/up matrix of the same model
        out["offline_quantiser"] = offline_quantiser(11008, 4096)

    if not args.no_cpu_baseline:
        import oracle
        rows = min(w.M, 2048)
        Xs = d["X_bf16"][:rows]
        c0 = time.perf_counter()
        A_ref, s_ref = oracle.quantize_act(Xs)
        oracle.w4a8_gemm(A_ref, s_ref, d["q"], d["gscale"], d["w_tscale"])
        c1 = time.perf_counter()
        if decode_like:
            cv, cu = wbytes / (c1 - c0) / 1e9, "GB/s"
        else:
            cv, cu = 2.0 * rows * w.N * w.K / (c1 - c0) / 1e12, "TFLOP/s"
        out["cpu_baseline"] = {"value": cv, "unit": cu, "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "first %d of %d rows of %s, all %d columns; FP64 C oracle (quantiser + GEMM), %.1f s"
                                         % (rows, w.M, name, w.N, c1 - c0)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
