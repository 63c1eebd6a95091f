#!/usr/bin/env python3
"""Benchmark of the training hot path on one MI355X.

A step = dnn_forward + dnn_backward_update (fused SGD update) on one 256-frame minibatch of the
440-6x2048-8000 sigmoid/softmax DNN, fp32, synthetic speech-shaped inputs already resident in HBM.
Prints ONE JSON line: whole-job train frames/s, the roofline record of the dominant kernel of the step (the
grouped weight-gradient + SGD-update launch, timed live with HIP events on the launch stream), and the CPU oracle
timed beside it on a bounded sample.  `extras` carries every GEMM of the step timed by itself, per-step statistics,
the cold (no clock warm-up) figure and the side measurements: replica averaging, CD-1, the RBM stack, the averaging
sweep, the paper's own shape, NG-SGD (one replica, and 8 replicas averaged every 5 minibatches), and the tile plan
between the tuned minibatch sizes.

    python bench.py [--gpus 1] [--steps 200] [--warmup 10] [--no-cpu] [--no-extras] [--extras a,b,...]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3     # 256 CU x 4 SIMD x 64 FLOP/cycle x 2.4 GHz
PEAK_HBM_GBPS = 8000.0
ALL_EXTRAS = ("kernels", "stats", "averaging", "cd1", "stack", "sweep", "paper", "ngsgd", "ngsgd8", "plan")
# rocprofv3 counter summary of the roofline kernel: bench.py takes `traffic` from the record this file carries
ROOFLINE_PROFILE = os.path.join(ROOT, "profiles", "weight_update_grouped_mb256_hbm_counters.md")
ROOFLINE_KERNEL = "gemm_dma_grouped_kernel"


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def traffic_from_profile(kernel: str, minibatch: int):
    """HBM bytes per launch of `kernel` as the committed counter summary states them (FETCH_SIZE + WRITE_SIZE,
    scaled against a plain copy), or None when there is no summary for this kernel and minibatch."""
    try:
        m = re.search(r"<!--\s*bench:\s*(\{.*?\})\s*-->", open(ROOFLINE_PROFILE).read(), re.S)
        rec = json.loads(m.group(1))
    except Exception:
        return None
    if rec.get("kernel") != kernel or rec.get("minibatch") != minibatch:
        return None
    return float(rec["fetch_bytes"]) + float(rec["write_bytes"])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--minibatch", type=int, default=256)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle legs")
    ap.add_argument("--no-extras", action="store_true", help="skip every side measurement")
    ap.add_argument("--extras", default="all", help="comma list of side measurements: " + ", ".join(ALL_EXTRAS) + " (default all)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="bound on the oracle's training leg")
    ap.add_argument("--no-warm", action="store_true",
                    help="skip the clock warm-up bursts and the cold leg (for hardware-counter runs, where every launch is serialised)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (a kernel of known traffic, to scale HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no inter-GPU collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import gen
    from paper_1507_01239_amd import binding as B       # raises if the HIP library is not built

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    dims, n, lr, seed = gen.CONFIG_FULL_DIMS, args.minibatch, 0.008, 1234
    L = len(dims) - 1
    steps, warmup = args.steps, args.warmup
    shape = B.Shape(dims)
    P = B.mavg_param_count(shape)
    flop_per_frame = 2 * (3 * sum(dims[l] * dims[l - 1] for l in range(1, len(dims))) - dims[1] * dims[0])

    def want(name):
        return not args.no_extras and (args.extras == "all" or name in args.extras.split(","))

    def frac(tflops):
        return round(tflops / PEAK_FP32_MFMA_TFLOPS, 4)

    # ---- inputs resident in HBM before the timed region ------------------------------------------
    total = steps + warmup
    distinct = min(max(total, 16), 64)            # up to 64 distinct minibatches cycled; all resident
    log(f"generating {distinct} minibatches of {n} frames ...")
    xs = torch.stack([torch.from_numpy(gen.features_speech_like(n, dims[0], seed, 0, t)) for t in range(distinct)]).cuda()
    ys = torch.stack([torch.from_numpy(gen.labels_zipf(n, dims[-1], seed, 0, t)) for t in range(distinct)]).cuda()
    theta0 = gen.init_theta(dims, seed, 0.05)
    theta = torch.from_numpy(theta0).cuda()
    acts = torch.empty(B.mavg_act_count(shape, n), device="cuda")
    ws = torch.empty(B.mavg_workspace_bytes(shape, n, 1, B.MEAN_GRAD) + 256, dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, device="cuda")

    def step(t):
        x, y = xs[t % distinct], ys[t % distinct]
        B.dnn_forward(shape, 1, theta, P, x, 0, n, acts, 0, ws)
        B.dnn_backward_update(shape, 1, theta, P, x, 0, y, 0, n, acts, 0, lr, B.MEAN_GRAD, loss, ws)

    def timed_steps(first, count):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(first, first + count):
            step(t)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # The GPU raises its clocks only after some tens of milliseconds of continuous work (the same GEMM runs
    # 15-20 % slower right after an idle gap such as input generation or a host synchronisation).  A training
    # job is never idle, so every timed region below starts from that steady state: a burst of GEMM launches
    # on scratch buffers, which touches none of the training state and is not counted as warmup steps.  The
    # figure WITHOUT the burst (straight after input generation) is reported once as extras.cold_ms_per_step.
    wa = torch.randn(n, dims[-2], device="cuda")
    ww = torch.randn(dims[-1], dims[-2], device="cuda") * 0.05
    wc = torch.empty(n, dims[-1], device="cuda")
    wws = torch.empty(B.mavg_gemm_workspace_bytes(n, dims[-1], dims[-2], -1, 0) + 256, dtype=torch.uint8, device="cuda")

    def warm_clocks(seconds=0.3):
        if args.no_warm:
            return
        t_end = time.perf_counter() + seconds
        while time.perf_counter() < t_end:
            for _ in range(200):
                B.mavg_gemm(wa, dims[-2], 1, ww, dims[-2], 1, wc, dims[-1], n, dims[-1], dims[-2], 0, None, None, 0, 1.0, 0.0, -1, 0, wws)
            torch.cuda.synchronize()

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def event_ms(fn, reps, warm=3, burst=0.2):
        """Average milliseconds per call of fn over `reps` calls, HIP events on the launch stream (torch's current one)."""
        warm_clocks(burst)
        for _ in range(warm):
            fn()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    cold_ms = None
    if not args.no_warm:
        time.sleep(0.5)                                   # an idle gap, as after loading data
        for t in range(warmup):
            step(t)
        cold_ms = timed_steps(warmup, steps) / steps * 1e3
        theta.copy_(torch.from_numpy(theta0))             # the measured run starts from the initial parameters again
        log(f"cold (no clock warm-up burst): {cold_ms:.3f} ms/step")

    # ---- the measured run: W warmup steps, then exactly K steps between synchronisations --------------
    warm_clocks()
    for t in range(warmup):
        step(t)
    elapsed = timed_steps(warmup, steps)
    ms_per_step = elapsed / steps * 1e3
    frames_per_s = n * steps / elapsed
    final_loss = float(loss.item()) / n
    log(f"train: {ms_per_step:.3f} ms/step, {frames_per_s:,.0f} frames/s, mean loss {final_loss:.4f}")

    extras = {"step_mfma_tflops": round(frames_per_s * flop_per_frame / 1e12, 3),
              "step_mfma_frac": frac(frames_per_s * flop_per_frame / 1e12),
              "flop_per_frame": flop_per_frame, "final_mean_loss": round(final_loss, 4)}
    if cold_ms is not None:
        extras["cold_ms_per_step"] = round(cold_ms, 4)

    if want("stats"):
        # per-step durations over 200 further steps, an event between consecutive steps
        ns = 200
        warm_clocks()
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(ns + 1)]
        for t in range(ns):
            evs[t].record()
            step(total + t)
        evs[ns].record()
        torch.cuda.synchronize()
        d = sorted(evs[t].elapsed_time(evs[t + 1]) for t in range(ns))
        extras["step_ms_stats"] = {"steps": ns, "mean": round(statistics.fmean(d), 4), "median": round(d[ns // 2], 4),
                                   "min": round(d[0], 4), "p95": round(d[int(ns * 0.95)], 4), "max": round(d[-1], 4)}
        log(f"per-step: {extras['step_ms_stats']}")

    # ---- every GEMM launch of the step by itself, on scratch operands of the step's shapes ---------------
    # A_l: activations (0..1), D_l: output errors with rows padded to a multiple of 4 floats, Wl: a scratch copy
    # of the parameters, so that the training state above is not touched.
    ld = [0] + [(dims[l] + 3) // 4 * 4 for l in range(1, L + 1)]
    A = [torch.randn(n, dims[0], device="cuda")] + [torch.rand(n, dims[l], device="cuda") for l in range(1, L + 1)]
    D = [None] + [torch.randn(n, ld[l], device="cuda") * 1e-3 for l in range(1, L + 1)]
    th_s = torch.from_numpy(theta0).cuda()
    w_off, b_off, off = [0], [0], 0
    for l in range(1, L + 1):
        w_off.append(off)
        off += dims[l] * dims[l - 1]
        b_off.append(off)
        off += dims[l]
    Wl = [None] + [th_s[w_off[l]:w_off[l] + dims[l] * dims[l - 1]] for l in range(1, L + 1)]
    bl = [None] + [th_s[b_off[l]:b_off[l] + dims[l]] for l in range(1, L + 1)]
    gws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")

    def fwd(l):     # A_l = act(A_{l-1} W_l^T + b_l)
        B.mavg_gemm(A[l - 1], dims[l - 1], 1, Wl[l], dims[l - 1], 1, A[l], dims[l], n, dims[l], dims[l - 1],
                    2 if l < L else 1, bl[l], None, 0, 1.0, 0.0, -1, 0, gws)

    def bwd(l):     # D_{l-1} = (D_l W_l) * A_{l-1} (1 - A_{l-1})
        B.mavg_gemm(D[l], ld[l], 1, Wl[l], dims[l - 1], 0, D[l - 1], ld[l - 1], n, dims[l - 1], dims[l], 3, None,
                    A[l - 1], dims[l - 1], 1.0, 0.0, -1, 0, gws)

    update = [B.gemm_problem(D[l], ld[l], A[l - 1], dims[l - 1], Wl[l], dims[l - 1], dims[l], dims[l - 1], n, epi=4,
                             alpha=-1e-6, beta=1.0, rowsum_dst=bl[l], rowsum_alpha=-1e-6, rowsum_beta=1.0, a_pad4=True)
              for l in range(1, L + 1)]

    def dw():       # W_l <- W_l - lr D_l^T A_{l-1}, b_l <- b_l - lr colsum(D_l), all layers in one launch
        B.mavg_gemm_grouped(update, 0, 0)

    # ---- roofline of the dominant kernel of the step: the grouped weight update -------------------------
    dw_flop = 2.0 * n * sum(dims[l] * dims[l - 1] for l in range(1, L + 1))
    dw_ms = event_ms(dw, 100, warm=5, burst=0.3)
    dw_tflops = dw_flop / (dw_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma",
                "kernel": f"{ROOFLINE_KERNEL}<1,1,3,false,false> fp32: weight gradients + SGD update + bias row sums of all {L} layers "
                          f"in one launch (contraction = minibatch {n})",
                "achieved": round(dw_tflops, 3), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": frac(dw_tflops),
                "traffic": traffic_from_profile(ROOFLINE_KERNEL, n), "avg_launch_us": round(dw_ms * 1e3, 2),
                "flop_per_launch": dw_flop}
    log(f"roofline: {roofline}")

    if want("kernels"):
        rows = []

        def row(name, fn, flop, per_step, reps=100):
            ms = event_ms(fn, reps)
            tf = flop / (ms * 1e-3) / 1e12
            rows.append({"launch": name, "us": round(ms * 1e3, 2), "per_step": per_step, "TFLOP/s": round(tf, 2), "mfma_frac": frac(tf)})
        row(f"forward layer 1: {n}x{dims[1]}x{dims[0]}", lambda: fwd(1), 2.0 * n * dims[1] * dims[0], 1)
        row(f"forward hidden: {n}x{dims[2]}x{dims[1]}", lambda: fwd(2), 2.0 * n * dims[2] * dims[1], L - 2)
        row(f"forward output: {n}x{dims[L]}x{dims[L - 1]}", lambda: fwd(L), 2.0 * n * dims[L] * dims[L - 1], 1)
        row(f"back-propagation output: {n}x{dims[L - 1]}x{dims[L]} (with its reducer)", lambda: bwd(L), 2.0 * n * dims[L] * dims[L - 1], 1)
        row(f"back-propagation hidden: {n}x{dims[1]}x{dims[2]}", lambda: bwd(2), 2.0 * n * dims[2] * dims[1], L - 2)
        rows.append({"launch": "weight update, all layers", "us": roofline["avg_launch_us"], "per_step": 1,
                     "TFLOP/s": roofline["achieved"], "mfma_frac": roofline["frac"]})
        gemm_us = sum(r["us"] * r["per_step"] for r in rows)
        extras["step_gemm_launches"] = {"rows": rows, "sum_us_per_step": round(gemm_us, 1),
                                        "step_us": round(ms_per_step * 1e3, 1)}
        log(f"kernels: {extras['step_gemm_launches']}")

    if args.calibrate_copy:
        src = torch.empty(64 * 1024 * 1024, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    del A, D, th_s, Wl, bl, gws

    if want("averaging"):
        # replica averaging: 8 replicas of the same network resident in HBM (2*K*P*4 bytes per call)
        Kr = 8
        reps_t = torch.randn(Kr, P, device="cuda") * 0.05
        avg_ms = event_ms(lambda: B.replicas_average(reps_t, P, P, Kr), 20)
        gbps = 2.0 * Kr * P * 4 / (avg_ms * 1e-3) / 1e9
        extras["averaging"] = {"replicas": Kr, "params": P, "ms": round(avg_ms, 4), "GB/s": round(gbps, 1),
                               "frac_of_hbm_peak": round(gbps / PEAK_HBM_GBPS, 4)}
        log(f"averaging: {extras['averaging']}")
        del reps_t

    def cd1_leg(V, H, vis, flags, lr_r, v0, reps=20):
        w_, a_, c_ = [torch.from_numpy(t).cuda() for t in gen.rbm_params(V, H, seed, 0)]
        mw, ma, mc = torch.zeros_like(w_), torch.zeros_like(a_), torch.zeros_like(c_)
        rws = torch.empty(B.rbm_workspace_bytes(V, H, n) + 256, dtype=torch.uint8, device="cuda")
        err = torch.zeros(1, device="cuda")
        st = [0]

        def one():
            B.rbm_cd1_step(V, H, vis, w_, a_, c_, mw, ma, mc, v0, n, lr_r, 0.9, seed, st[0], 0, flags, err, rws)
            st[0] += 1
        ms = event_ms(one, reps)
        tf = 10.0 * n * V * H / (ms * 1e-3) / 1e12
        return {"ms": round(ms, 4), "frames/s": round(n / ms * 1e3, 1), "TFLOP/s": round(tf, 2), "frac_of_mfma_peak": frac(tf)}

    if want("cd1"):
        # RBM CD-1 steps (10*n*V*H FLOP each): Gaussian 440 -> 2048, then Bernoulli 2048 -> 2048 with sampled visibles;
        # rates 0.01 / 0.4 scaled by (1 - momentum), without which the recursion diverges on these inputs
        extras["cd1_gaussian_440x2048"] = cd1_leg(440, 2048, B.VIS_GAUSSIAN, 0, 0.001, xs[0])
        extras["cd1_bernoulli_2048x2048"] = cd1_leg(2048, 2048, B.VIS_BERNOULLI, B.SAMPLE_V1, 0.04, torch.rand(n, 2048, device="cuda"))
        log(f"cd1: {extras['cd1_gaussian_440x2048']} {extras['cd1_bernoulli_2048x2048']}")

    if want("stack"):
        # Sec. 5.1: the greedy stack of 6 RBMs (440 -> 2048, then five of 2048 -> 2048) trained for a bounded number
        # of minibatches each, then copied into the hidden layers of the DNN
        from paper_1507_01239_amd import pretrain as PT
        widths = list(dims[:-1])
        per_rbm = 50
        mbs = [xs[t] for t in range(min(distinct, 16))]
        init = [tuple(torch.from_numpy(t).cuda() for t in gen.rbm_params(widths[l - 1], widths[l], seed, l)) for l in range(1, len(widths))]
        warm_clocks(0.2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        times = PT.pretrain_stack(widths, mbs, init, per_rbm, 0.001, 0.04, 0.9, seed, timings=True)[1]
        th_stack = torch.from_numpy(theta0).cuda()
        PT.init_dnn_from_stack(shape, 1, th_stack, P, init)
        torch.cuda.synchronize()
        total_s = time.perf_counter() - t0
        extras["rbm_stack_6_rbms"] = {"minibatches_per_rbm": per_rbm, "minibatch": n,
                                      "frames/s_per_rbm": [round(n * per_rbm / s, 1) for s in times],
                                      "end_to_end_ms": round(total_s * 1e3, 2)}
        log(f"stack: {extras['rbm_stack_6_rbms']}")
        del init, th_stack

    def replicas_leg(rdims, Kr, nb, n_avgs, steps_of, use_ng=False, rank=30):
        """Kr replicas resident in HBM, one grouped launch per GEMM for all replicas, parameters averaged every
        n_avg minibatches; returns {n_avg: ms per minibatch of all replicas}."""
        rshape = B.Shape(rdims)
        PP = B.mavg_param_count(rshape)
        pstride = (PP + 63) // 64 * 64
        th = torch.zeros(Kr, pstride, device="cuda")
        th[:, :PP] = torch.from_numpy(gen.init_theta(rdims, seed, 0.05)).cuda()
        xb = torch.stack([torch.from_numpy(gen.features_speech_like(nb, rdims[0], seed, r, 0)) for r in range(Kr)]).cuda()
        yb = torch.stack([torch.from_numpy(gen.labels_zipf(nb, rdims[-1], seed, r, 0)) for r in range(Kr)]).cuda()
        astride = (B.mavg_act_count(rshape, nb) + 63) // 64 * 64
        ac = torch.empty(Kr, astride, device="cuda")
        fl = B.MEAN_GRAD | (B.USE_NGSGD if use_ng else 0)
        wk = torch.empty(B.mavg_workspace_bytes(rshape, nb, Kr, fl, rank) + 256, dtype=torch.uint8, device="cuda")
        kw = {}
        if use_ng:
            RL = len(rdims) - 1
            sb = B.ngsgd_state_bytes(max(rdims) + 1, rank)
            st_ = torch.zeros(Kr * 2 * RL, sb, dtype=torch.uint8, device="cuda")
            for r in range(Kr):
                for l in range(1, RL + 1):
                    B.ngsgd_state_init(st_[r * 2 * RL + 2 * (l - 1)], rdims[l - 1] + 1, rank)
                    B.ngsgd_state_init(st_[r * 2 * RL + 2 * (l - 1) + 1], rdims[l], rank)
            kw = dict(ng_state=st_, ng_state_stride=sb, ng_rank=rank, ng_alpha=4.0, ng_eta=1.0 - float(np.exp(-nb / 2000.0)))
        first = [use_ng]
        out = {}
        for n_avg in n_avgs:
            def run(count):
                for t in range(count):
                    B.dnn_forward(rshape, Kr, th, pstride, xb, nb * rdims[0], nb, ac, astride, wk)
                    B.dnn_backward_update(rshape, Kr, th, pstride, xb, nb * rdims[0], yb, nb, nb, ac, astride, lr,
                                          fl | (B.NG_FIRST if first[0] else 0), None, wk, **kw)
                    first[0] = False
                    if (t + 1) % n_avg == 0:
                        B.replicas_average(th, pstride, PP, Kr)
            run(1)
            warm_clocks(0.2)
            run(2)
            cnt = steps_of(n_avg)
            e0.record()
            run(cnt)
            e1.record()
            torch.cuda.synchronize()
            out[n_avg] = e0.elapsed_time(e1) / cnt
        return out

    def cell(ms, Kr, nb, fpf):
        tf = Kr * nb / ms * 1e3 * fpf / 1e12
        return {"ms_per_minibatch_of_all_replicas": round(ms, 3), "frames/s": round(Kr * nb / ms * 1e3, 1), "mfma_frac": frac(tf)}

    if want("sweep"):
        # model-averaging sweep (config 3): 8 replicas, minibatch 128..1024, averaged every 1, 2, 5, 10 minibatches
        out = {}
        for nb in (128, 256, 512, 1024):
            for n_avg, ms in replicas_leg(dims, 8, nb, (1, 2, 5, 10), lambda a: 20).items():
                out[f"mb{nb}_n{n_avg}"] = cell(ms, 8, nb, flop_per_frame)
        extras["averaging_sweep_8_replicas"] = out
        log(f"sweep: {out}")

    if want("paper"):
        # the paper's own shape (Sec. 5.1, 5.5): 440-6x2048-8806, minibatch 1024, m = 8, 16, 32 replicas on the one
        # GPU, averaged every 10 or 20 minibatches
        pd = gen.CONFIG_PAPER_DIMS
        pflop = 2 * (3 * sum(pd[l] * pd[l - 1] for l in range(1, len(pd))) - pd[1] * pd[0])
        out = {}
        for Kr in (8, 16, 32):
            for n_avg, ms in replicas_leg(pd, Kr, 1024, (10, 20), lambda a: a).items():
                out[f"m{Kr}_n{n_avg}"] = cell(ms, Kr, 1024, pflop)
        extras["paper_shape_440_6x2048_8806_mb1024"] = out
        log(f"paper shape: {out}")

    if want("ngsgd"):
        # NG-SGD step against the plain SGD step at minibatch 512, rank 30 (one replica)
        def train_ms(nb, use_ng, fold_every=1):
            xb = torch.from_numpy(gen.features_speech_like(nb, dims[0], seed, 1, 0)).cuda()
            yb = torch.from_numpy(gen.labels_zipf(nb, dims[-1], seed, 1, 0)).cuda()
            th = torch.from_numpy(theta0).cuda()
            ac = torch.empty(B.mavg_act_count(shape, nb), device="cuda")
            fl = B.MEAN_GRAD | (B.USE_NGSGD if use_ng else 0)
            w2 = torch.empty(B.mavg_workspace_bytes(shape, nb, 1, fl, 30) + 256, dtype=torch.uint8, device="cuda")
            kw, st_ = {}, None
            if use_ng:
                sb = B.ngsgd_state_bytes(max(dims) + 1, 30)
                st_ = torch.zeros(2 * L, sb, dtype=torch.uint8, device="cuda")
                for l in range(1, L + 1):
                    B.ngsgd_state_init(st_[2 * (l - 1)], dims[l - 1] + 1, 30)
                    B.ngsgd_state_init(st_[2 * (l - 1) + 1], dims[l], 30)
                kw = dict(ng_state=st_, ng_state_stride=sb, ng_rank=30, ng_alpha=4.0, ng_eta=1.0 - float(np.exp(-nb / 2000.0)))
            i = [0]

            def one(first=False):
                extra = 0
                if use_ng:
                    extra = B.NG_FIRST if first else (0 if i[0] % fold_every == 0 else B.NG_APPLY_ONLY)
                B.dnn_forward(shape, 1, th, P, xb, 0, nb, ac, 0, w2)
                B.dnn_backward_update(shape, 1, th, P, xb, 0, yb, 0, nb, ac, 0, lr, fl | extra, None, w2, **kw)
                i[0] += 1
            one(True)
            i[0] = 0
            ms = event_ms(one, 20)
            sweeps = None
            if use_ng:      # Jacobi sweeps of the last fold of each of the 14 states, and folds that ran out of sweeps
                raw = st_.cpu().numpy()
                info = []
                for j in range(2 * L):
                    dim = dims[j // 2] + 1 if j % 2 == 0 else dims[j // 2 + 1]
                    o = 30 * ((dim + 3) // 4 * 4) * 4 + 30 * 8 + 16
                    info.append(np.frombuffer(raw[j].tobytes(), np.int32, 2, o))
                sweeps = {"last_fold_sweeps_min_max": [int(min(v[0] for v in info)), int(max(v[0] for v in info))],
                          "folds_out_of_sweeps": int(sum(v[1] for v in info))}
            return ms, sweeps
        sgd_ms, _ = train_ms(512, False)
        ng_ms, sweeps = train_ms(512, True)
        ng4_ms, _ = train_ms(512, True, 4)
        extras["ngsgd_mb512_rank30"] = {"sgd_ms": round(sgd_ms, 4), "ngsgd_ms": round(ng_ms, 4),
                                        "overhead": round(ng_ms / sgd_ms - 1.0, 4),
                                        "ngsgd_frames/s": round(512 / ng_ms * 1e3, 1),
                                        "ngsgd_fold_every_4th_minibatch_ms": round(ng4_ms, 4),
                                        "overhead_fold_every_4th": round(ng4_ms / sgd_ms - 1.0, 4), "eigen_solver": sweeps}
        log(f"ngsgd: {extras['ngsgd_mb512_rank30']}")

    if want("ngsgd8"):
        # config 5 (Sec. 4 eq. 4 with Sec. 3 eq. 2; Sec. 5.7): 8 replicas, NG-SGD rank 30, minibatch 512, averaged every 5
        ms_ng = replicas_leg(dims, 8, 512, (5,), lambda a: 10, use_ng=True)[5]
        ms_sgd = replicas_leg(dims, 8, 512, (5,), lambda a: 10)[5]
        c = cell(ms_ng, 8, 512, flop_per_frame)
        c.update({"plain_sgd_ms": round(ms_sgd, 3), "overhead": round(ms_ng / ms_sgd - 1.0, 4)})
        extras["ngsgd_8_replicas_n5_mb512_rank30"] = c
        log(f"ngsgd, 8 replicas: {c}")

    if want("plan"):
        # the tile plan between the minibatch sizes it was tuned on: whole-step MFMA fraction, 1 / 3 / 8 replicas
        out = {}
        for nb in (64, 192, 320, 768):
            for Kr in (1, 3, 8):
                ms = replicas_leg(dims, Kr, nb, (1000000,), lambda a: 10)[1000000]
                out[f"mb{nb}_k{Kr}"] = cell(ms, Kr, nb, flop_per_frame)
        extras["plan_between_tuned_sizes"] = out
        log(f"plan: {out}")

    cpu_baseline = None
    if not args.no_cpu:
        # The oracle as it stands (float64 NumPy: its matrix products run in the BLAS NumPy is linked with, on that
        # library's threads), timed on this machine's host cores on bounded samples.
        from oracle import averaging as oavg
        from oracle import dnn as odnn
        from oracle import ngsgd as ong
        from oracle import rbm as orbm
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        kind = f"oracle (float64 NumPy, BLAS-backed matrix products, {int(cores)} threads)"
        th = theta0.astype(np.float64)
        xs_h, ys_h = xs.cpu().numpy(), ys.cpu().numpy()
        done, t0 = 0, time.perf_counter()
        while done < 50 and (time.perf_counter() - t0) < args.cpu_seconds:
            th, _, _ = odnn.sgd_step(th, dims, xs_h[done % distinct], ys_h[done % distinct], lr)
            done += 1
        cpu_el = time.perf_counter() - t0
        cpu_baseline = {"value": round(n * done / cpu_el, 1), "unit": "frames/s", "cores": int(cores), "kind": kind,
                        "sample": f"{done} minibatches of {n} frames of the same workload"}
        log(f"cpu_baseline: {cpu_baseline}")
        if not args.no_extras:
            other = {"kind": kind}
            # config 3, one cell: 8 replicas x 2 minibatches of 256, averaged after the second
            sh = [[(xs_h[(2 * k + t) % distinct], ys_h[(2 * k + t) % distinct]) for t in range(2)] for k in range(8)]
            t0 = time.perf_counter()
            oavg.train_with_averaging(theta0, dims, sh, lr, 2)
            other["config3_mb256_8_replicas_n2"] = {"frames/s": round(8 * 2 * n / (time.perf_counter() - t0), 1),
                                                    "sample": "8 replicas x 2 minibatches, one averaging"}
            # config 4: 20 CD-1 steps of each RBM
            for name, V, H, vis, lr_r, v0, sv in (("gaussian_440x2048", 440, 2048, orbm.GAUSSIAN, 0.001, xs_h[0], False),
                                                   ("bernoulli_2048x2048", 2048, 2048, orbm.BERNOULLI, 0.04,
                                                    np.random.default_rng(0).random((n, 2048)).astype(np.float32), True)):
                W_, a_, c_ = gen.rbm_params(V, H, seed, 0)
                MW, Ma, Mc = np.zeros_like(W_), np.zeros_like(a_), np.zeros_like(c_)
                t0 = time.perf_counter()
                for st in range(20):
                    W_, a_, c_, MW, Ma, Mc, _ = orbm.cd1_step(W_, a_, c_, MW, Ma, Mc, v0, vis, lr_r, 0.9, seed, st, 0, sample_v1=sv)
                other[f"config4_cd1_{name}"] = {"frames/s": round(20 * n / (time.perf_counter() - t0), 1), "sample": "20 CD-1 steps"}
            # config 5: NG-SGD rank 30 at minibatch 512, one replica: the first minibatch (three initial folds), then two more
            nb = 512
            s_in = [ong.init_state(dims[l - 1] + 1, 30) for l in range(1, len(dims))]
            s_out = [ong.init_state(dims[l], 30) for l in range(1, len(dims))]
            pre = ong.make_layer_preconditioner(s_in, s_out, 4.0, ong.default_eta(nb))
            th = theta0.astype(np.float64)
            ts = []
            for t in range(3):
                xb = gen.features_speech_like(nb, dims[0], seed, 1, t)
                yb = gen.labels_zipf(nb, dims[-1], seed, 1, t)
                t0 = time.perf_counter()
                th, _, _ = odnn.sgd_step(th, dims, xb, yb, lr, precondition=pre)
                ts.append(time.perf_counter() - t0)
            other["config5_ngsgd_mb512_rank30"] = {"frames/s": round(2 * nb / (ts[1] + ts[2]), 1), "first_minibatch_s": round(ts[0], 2),
                                                   "sample": "minibatches 2 and 3 of one replica; 8 replicas run one after the other on the "
                                                             "CPU, so the 8-replica rate is the same figure (extrapolated, not run)"}
            extras["cpu_oracle_other_configs"] = other
            log(f"cpu oracle, other configs: {other}")

    out = {"metric": "train frames/s, 6x2048 DNN mb256", "value": round(frames_per_s, 1), "unit": "frames/s",
           "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"440-6x2048-8000 sigmoid/softmax DNN, minibatch {n}, SGD lr 0.008, 1 replica "
                                  "(forward + cross-entropy backward + fused update)",
                      "minibatch": n, "params": P},
           "roofline": roofline, "cpu_baseline": cpu_baseline, "extras": extras}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
