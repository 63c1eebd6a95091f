#!/usr/bin/env python3
"""Benchmark of the training hot path on one MI355X.

A step = dnn_forward + dnn_backward_update (fused SGD update) on one 256-frame minibatch of the
440-6x2048-8000 sigmoid/softmax DNN, fp32, synthetic speech-shaped inputs already resident in HBM.
Prints ONE JSON line: whole-job train frames/s, the roofline record of the dominant kernel (timed live
with HIP events on the launch stream) and the CPU oracle timed beside it on a bounded sample.

    python bench.py [--gpus 1] [--steps 200] [--warmup 10] [--no-cpu] [--no-extras]
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

PEAK_FP32_MFMA_TFLOPS = 157.3     # 256 CU x 4 SIMD x 64 FLOP/cycle x 2.4 GHz
PEAK_HBM_GBPS = 8000.0
# HBM-side traffic of one launch of the roofline kernel (256 x 8000 x 2048 forward GEMM), from the two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, scaled by a plain copy of known size) summarised in
# profiles/gemm_output_layer_forward_hbm_counters.md: 99.1 MB fetched + 8.2 MB written.
ROOFLINE_TRAFFIC_BYTES = {256: 107.3e6}


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--minibatch", type=int, default=256)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-extras", action="store_true", help="skip the averaging / CD-1 side measurements")
    ap.add_argument("--extras", default="all",
                    help="comma list of the side measurements to run: averaging, cd1, sweep, paper, ngsgd (default all)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="bound on the oracle leg")
    ap.add_argument("--no-warm", action="store_true",
                    help="skip the clock warm-up bursts (for hardware-counter runs, where every launch is serialised)")
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
    steps, warmup = args.steps, args.warmup
    shape = B.Shape(dims)
    P = B.mavg_param_count(shape)
    flop_per_frame = 2 * (3 * sum(dims[l] * dims[l - 1] for l in range(1, len(dims))) - dims[1] * dims[0])

    # ---- inputs resident in HBM before the timed region ------------------------------------------
    total = steps + warmup
    distinct = min(total, 64)            # 64 distinct minibatches cycled; all resident
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

    # The GPU raises its clocks only after some tens of milliseconds of continuous work (the same GEMM runs
    # 15-20 % slower right after an idle gap such as input generation or a host synchronisation).  A training
    # job is never idle, so every timed region below starts from that steady state: a burst of GEMM launches
    # on scratch buffers, which touches none of the training state and is not counted as warmup steps.
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

    warm_clocks()
    for t in range(warmup):
        step(t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(warmup, total):
        step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / steps * 1e3
    frames_per_s = n * steps / elapsed
    final_loss = float(loss.item()) / n
    log(f"train: {ms_per_step:.3f} ms/step, {frames_per_s:,.0f} frames/s, mean loss {final_loss:.4f}")

    # ---- roofline of the dominant kernel: the output-layer GEMM (n x 8000 x 2048), forward form --
    # timed with HIP events on the stream the kernel is launched on (torch's current stream)
    M, N, K = n, dims[-1], dims[-2]
    a = torch.randn(M, K, device="cuda")
    w = torch.randn(N, K, device="cuda") * 0.05
    c = torch.empty(M, N, device="cuda")
    bias = torch.zeros(N, device="cuda")
    gws = torch.empty(B.mavg_gemm_workspace_bytes(M, N, K, -1, 0) + 256, dtype=torch.uint8, device="cuda")
    reps = 200
    warm_clocks()
    for _ in range(5):
        B.mavg_gemm(a, K, 1, w, K, 1, c, N, M, N, K, 1, bias, None, 0, 1.0, 0.0, -1, 0, gws)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        B.mavg_gemm(a, K, 1, w, K, 1, c, N, M, N, K, 1, bias, None, 0, 1.0, 0.0, -1, 0, gws)
    e1.record()
    torch.cuda.synchronize()
    gemm_ms = e0.elapsed_time(e1) / reps
    gemm_tflops = 2.0 * M * N * K / (gemm_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": f"gemm_dma_kernel fp32 {M}x{N}x{K} (output layer, forward)",
                "achieved": round(gemm_tflops, 3), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": round(gemm_tflops / PEAK_FP32_MFMA_TFLOPS, 4), "traffic": ROOFLINE_TRAFFIC_BYTES.get(n),
                "avg_launch_us": round(gemm_ms * 1e3, 2)}
    log(f"roofline: {roofline}")

    if args.calibrate_copy:
        src = torch.empty(64 * 1024 * 1024, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    extras = {"step_mfma_tflops": round(frames_per_s * flop_per_frame / 1e12, 3),
              "step_mfma_frac": round(frames_per_s * flop_per_frame / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4),
              "flop_per_frame": flop_per_frame, "final_mean_loss": round(final_loss, 4)}

    def want(name):
        return not args.no_extras and (args.extras == "all" or name in args.extras.split(","))

    if want("averaging"):
        # replica averaging: 8 replicas of the same network resident in HBM (2*K*P*4 bytes per call)
        Kr = 8
        reps_t = torch.randn(Kr, P, device="cuda") * 0.05
        warm_clocks(0.2)
        for _ in range(3):
            B.replicas_average(reps_t, P, P, Kr)
        e0.record()
        for _ in range(20):
            B.replicas_average(reps_t, P, P, Kr)
        e1.record()
        torch.cuda.synchronize()
        avg_ms = e0.elapsed_time(e1) / 20
        gbps = 2.0 * Kr * P * 4 / (avg_ms * 1e-3) / 1e9
        extras["averaging"] = {"replicas": Kr, "params": P, "ms": round(avg_ms, 4), "GB/s": round(gbps, 1),
                               "frac_of_hbm_peak": round(gbps / PEAK_HBM_GBPS, 4)}
        log(f"averaging: {extras['averaging']}")
        del reps_t

    if want("cd1"):
        # RBM CD-1 steps (10*n*V*H FLOP each): Gaussian 440 -> 2048, then Bernoulli 2048 -> 2048 with sampled visibles
        def cd1(V, H, vis, flags, lr_r, v0):
            w_, a_, c_ = [torch.from_numpy(t).cuda() for t in gen.rbm_params(V, H, seed, 0)]
            mw, ma, mc = torch.zeros_like(w_), torch.zeros_like(a_), torch.zeros_like(c_)
            rws = torch.empty(B.rbm_workspace_bytes(V, H, n) + 256, dtype=torch.uint8, device="cuda")
            err = torch.zeros(1, device="cuda")
            warm_clocks(0.2)
            for st in range(3):
                B.rbm_cd1_step(V, H, vis, w_, a_, c_, mw, ma, mc, v0, n, lr_r, 0.9, seed, st, 0, flags, err, rws)
            e0.record()
            for st in range(20):
                B.rbm_cd1_step(V, H, vis, w_, a_, c_, mw, ma, mc, v0, n, lr_r, 0.9, seed, 3 + st, 0, flags, err, rws)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 20
            return {"ms": round(ms, 4), "frames/s": round(n / ms * 1e3, 1),
                    "TFLOP/s": round(10.0 * n * V * H / (ms * 1e-3) / 1e12, 2),
                    "frac_of_mfma_peak": round(10.0 * n * V * H / (ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4)}
        extras["cd1_gaussian_440x2048"] = cd1(440, 2048, B.VIS_GAUSSIAN, 0, 0.01, xs[0])
        extras["cd1_bernoulli_2048x2048"] = cd1(2048, 2048, B.VIS_BERNOULLI, B.SAMPLE_V1, 0.4, torch.rand(n, 2048, device="cuda"))
        log(f"cd1: {extras['cd1_gaussian_440x2048']} {extras['cd1_bernoulli_2048x2048']}")

    if not args.no_extras:
        # NG-SGD step against the plain SGD step at minibatch 512, rank 30 (one replica)
        def train_ms(nb, use_ng, fold_every=1):
            xb = torch.from_numpy(gen.features_speech_like(nb, dims[0], seed, 1, 0)).cuda()
            yb = torch.from_numpy(gen.labels_zipf(nb, dims[-1], seed, 1, 0)).cuda()
            th = torch.from_numpy(theta0).cuda()
            ac = torch.empty(B.mavg_act_count(shape, nb), device="cuda")
            fl = B.MEAN_GRAD | (B.USE_NGSGD if use_ng else 0)
            w2 = torch.empty(B.mavg_workspace_bytes(shape, nb, 1, fl, 30) + 256, dtype=torch.uint8, device="cuda")
            kw = {}
            if use_ng:
                L = len(dims) - 1
                sb = B.ngsgd_state_bytes(max(dims) + 1, 30)
                st_ = torch.zeros(2 * L, sb, dtype=torch.uint8, device="cuda")
                for l in range(1, L + 1):
                    B.ngsgd_state_init(st_[2 * (l - 1)], dims[l - 1] + 1, 30)
                    B.ngsgd_state_init(st_[2 * (l - 1) + 1], dims[l], 30)
                kw = dict(ng_state=st_, ng_state_stride=sb, ng_rank=30, ng_alpha=4.0, ng_eta=1.0 - float(np.exp(-nb / 2000.0)))
            def one(first, i=0):
                extra = 0
                if use_ng:
                    extra = B.NG_FIRST if first else (0 if i % fold_every == 0 else B.NG_APPLY_ONLY)
                B.dnn_forward(shape, 1, th, P, xb, 0, nb, ac, 0, w2)
                B.dnn_backward_update(shape, 1, th, P, xb, 0, yb, 0, nb, ac, 0, lr, fl | extra, None, w2, **kw)
            one(True)
            warm_clocks(0.2)
            for i in range(3):
                one(False, i)
            e0.record()
            for i in range(20):
                one(False, i)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / 20
        # model-averaging sweep: 8 replicas resident in HBM, one grouped launch per GEMM for all replicas,
        # parameters averaged every n_avg minibatches
        def sweep():
            Kr, out = 8, {}
            th8 = torch.from_numpy(theta0).cuda().repeat(Kr, 1).contiguous()
            for nb in (128, 256, 512, 1024):
                xb = torch.stack([torch.from_numpy(gen.features_speech_like(nb, dims[0], seed, r, 0)) for r in range(Kr)]).cuda()
                yb = torch.stack([torch.from_numpy(gen.labels_zipf(nb, dims[-1], seed, r, 0)) for r in range(Kr)]).cuda()
                astride = (B.mavg_act_count(shape, nb) + 63) // 64 * 64
                ac = torch.empty(Kr, astride, device="cuda")
                w8 = torch.empty(B.mavg_workspace_bytes(shape, nb, Kr, B.MEAN_GRAD) + 256, dtype=torch.uint8, device="cuda")
                for n_avg in (1, 2, 5, 10):
                    def run(steps_):
                        for t in range(steps_):
                            B.dnn_forward(shape, Kr, th8, P, xb, nb * dims[0], nb, ac, astride, w8)
                            B.dnn_backward_update(shape, Kr, th8, P, xb, nb * dims[0], yb, nb, nb, ac, astride, lr, B.MEAN_GRAD, None, w8)
                            if (t + 1) % n_avg == 0:
                                B.replicas_average(th8, P, P, Kr)
                    warm_clocks(0.2)
                    run(n_avg if n_avg > 2 else 2)
                    e0.record()
                    run(20)
                    e1.record()
                    torch.cuda.synchronize()
                    ms = e0.elapsed_time(e1) / 20
                    out[f"mb{nb}_n{n_avg}"] = {"ms_per_minibatch_of_all_replicas": round(ms, 3),
                                               "frames/s": round(Kr * nb / ms * 1e3, 1),
                                               "mfma_frac": round(Kr * nb / ms * 1e3 * flop_per_frame / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4)}
                del xb, yb, ac, w8
            return out
        # the paper's own shape (Sec. 5.1, 5.5): 440-6x2048-8806, minibatch 1024, m replicas averaged every
        # 10 or 20 minibatches; m = 8, 16, 32 replicas all resident on the one GPU
        def paper_shape():
            pd = gen.CONFIG_PAPER_DIMS
            pshape = B.Shape(pd)
            PP = B.mavg_param_count(pshape)
            pstride = (PP + 63) // 64 * 64
            pflop = 2 * (3 * sum(pd[l] * pd[l - 1] for l in range(1, len(pd))) - pd[1] * pd[0])
            nb, out = 1024, {}
            th1 = torch.from_numpy(gen.init_theta(pd, seed, 0.05)).cuda()
            for Kr in (8, 16, 32):
                th = torch.zeros(Kr, pstride, device="cuda")
                th[:, :PP] = th1
                xb = torch.stack([torch.from_numpy(gen.features_speech_like(nb, pd[0], seed, r, 0)) for r in range(Kr)]).cuda()
                yb = torch.stack([torch.from_numpy(gen.labels_zipf(nb, pd[-1], seed, r, 0)) for r in range(Kr)]).cuda()
                astride = (B.mavg_act_count(pshape, nb) + 63) // 64 * 64
                ac = torch.empty(Kr, astride, device="cuda")
                wp = torch.empty(B.mavg_workspace_bytes(pshape, nb, Kr, B.MEAN_GRAD) + 256, dtype=torch.uint8, device="cuda")
                for n_avg in (10, 20):
                    def run(steps_):
                        for t in range(steps_):
                            B.dnn_forward(pshape, Kr, th, pstride, xb, nb * pd[0], nb, ac, astride, wp)
                            B.dnn_backward_update(pshape, Kr, th, pstride, xb, nb * pd[0], yb, nb, nb, ac, astride, lr, B.MEAN_GRAD, None, wp)
                            if (t + 1) % n_avg == 0:
                                B.replicas_average(th, pstride, PP, Kr)
                    warm_clocks(0.2)
                    run(2)
                    e0.record()
                    run(n_avg)
                    e1.record()
                    torch.cuda.synchronize()
                    ms = e0.elapsed_time(e1) / n_avg
                    out[f"m{Kr}_n{n_avg}"] = {"ms_per_minibatch_of_all_replicas": round(ms, 3),
                                              "frames/s": round(Kr * nb / ms * 1e3, 1),
                                              "mfma_frac": round(Kr * nb / ms * 1e3 * pflop / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4)}
                del th, xb, yb, ac, wp
            return out
        if want("sweep"):
            extras["averaging_sweep_8_replicas"] = sweep()
            log(f"sweep: {extras['averaging_sweep_8_replicas']}")
        if want("paper"):
            extras["paper_shape_440_6x2048_8806_mb1024"] = paper_shape()
            log(f"paper shape: {extras['paper_shape_440_6x2048_8806_mb1024']}")
        if want("ngsgd"):
            sgd_ms, ng_ms, ng4_ms = train_ms(512, False), train_ms(512, True), train_ms(512, True, 4)
            extras["ngsgd_mb512_rank30"] = {"sgd_ms": round(sgd_ms, 4), "ngsgd_ms": round(ng_ms, 4),
                                            "overhead": round(ng_ms / sgd_ms - 1.0, 4),
                                            "ngsgd_frames/s": round(512 / ng_ms * 1e3, 1),
                                            "ngsgd_fold_every_4th_minibatch_ms": round(ng4_ms, 4),
                                            "overhead_fold_every_4th": round(ng4_ms / sgd_ms - 1.0, 4)}
            log(f"ngsgd: {extras['ngsgd_mb512_rank30']}")

    cpu_baseline = None
    if not args.no_cpu:
        from oracle import dnn as odnn
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        th = theta0.astype(np.float64)
        xs_h, ys_h = xs.cpu().numpy(), ys.cpu().numpy()
        done, t0 = 0, time.perf_counter()
        while done < 50 and (time.perf_counter() - t0) < args.cpu_seconds:
            th, _, _ = odnn.sgd_step(th, dims, xs_h[done % distinct], ys_h[done % distinct], lr)
            done += 1
        cpu_el = time.perf_counter() - t0
        cpu_baseline = {"value": round(n * done / cpu_el, 1), "unit": "frames/s", "cores": int(cores), "kind": "oracle",
                        "sample": f"{done} minibatches of {n} frames of the same workload (fp64 NumPy oracle)"}
        log(f"cpu_baseline: {cpu_baseline}")

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
