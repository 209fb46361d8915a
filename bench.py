#!/usr/bin/env python3
"""Benchmark: forward convolution of the ResNet-50-shaped layer suite (fp32, batch 32) on one MI355X.

A step is one pass over the eight layers through polydl_conv2d_fwd (bias and ReLU fused), inputs
already resident in HBM.  Prints ONE JSON line: whole-suite TFLOP/s, the roofline of the
convolution kernel (nominal flops / kernel time measured with HIP events), per-layer and SGEMM
rows, and the CPU oracle timed on a bounded sample of the same layers.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--sweep] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

FP32_MFMA_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix peak
HBM_PEAK_GBS = 8000.0


def conv_flops(s, P, Q):
    return 2.0 * s.N * s.K * P * Q * s.C * s.R * s.S


def conv_bytes(s, P, Q):
    """Compulsory traffic: read input and filter once, write output once."""
    return 4.0 * (s.N * s.C * s.H * s.W + s.K * s.C * s.R * s.S + s.N * s.K * P * Q + s.K)


def time_calls(torch, fn, reps, batches=3):
    """Median over batches of the mean time (ms) of reps back-to-back calls between two events."""
    out = []
    for _ in range(batches):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        out.append(e0.elapsed_time(e1) / reps)
    out.sort()
    return out[len(out) // 2]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--sweep", action="store_true", help="also time every compiled variant per layer")
    ap.add_argument("--sweep-out", default="", help="with --sweep: write every candidate's time to this JSON file")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-sgemm", action="store_true")
    ap.add_argument("--layers", default="", help="comma list of suite layers to run (default: all eight); "
                    "a subset is for profiling one kernel and changes the workload the line reports")
    ap.add_argument("--tile", default="", help="force a variant bm,bn,bk,wm,wn[,split_k[,layout[,raster]]] (profiling)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU; --gpus %d is not supported "
                 "(the path has no multi-GPU part, see DESIGN.md)" % args.gpus)

    import numpy as np
    import torch
    import synth
    import paper_2006_02230_amd as P

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)

    suite = synth.RESNET50_SUITE(args.batch)
    chosen = [int(t) for t in args.layers.split(",") if t != ""] or list(range(len(suite)))
    forced = None
    if args.tile:
        t = [int(v) for v in args.tile.split(",")]
        t += [1, 0, 0][len(t) - 5:]
        forced = P.TileCfg(*t)
    layers = []
    for i, s in enumerate(suite):
        if i not in chosen:
            continue
        x, w, b = synth.conv_inputs(s, seed=100 + i, dist="normal", bias=True)
        Pq, Qq = synth.out_hw(s)
        layers.append(dict(shape=s, P=Pq, Q=Qq, x=torch.from_numpy(x).cuda(), w=torch.from_numpy(w).cuda(),
                           b=torch.from_numpy(b).cuda(),
                           out=torch.empty((s.N, s.K, Pq, Qq), dtype=torch.float32, device="cuda"),
                           index=i, flops=conv_flops(s, Pq, Qq), bytes=conv_bytes(s, Pq, Qq), host=(x, w, b)))

    def run_layer(L):
        s = L["shape"]
        P.conv2d_fwd(L["x"], L["w"], L["b"], out=L["out"], stride=s.stride, pad=s.pad, act="relu")

    def step():
        for L in layers:
            run_layer(L)

    P.set_tile_override(forced)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    total_flops = sum(L["flops"] for L in layers)
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    # per-layer kernel time: back-to-back launches of one layer between two events on the launch stream
    rows = []
    sweep_dump = []
    kern_ms_sum = 0.0
    for L in layers:
        i = L["index"]
        reps = 30
        ms = time_calls(torch, lambda L=L: run_layer(L), reps)
        tile = P.get_last_tile().as_dict()
        tf = L["flops"] / (ms * 1e-3) / 1e12
        ai = L["flops"] / L["bytes"]
        ceiling = min(FP32_MFMA_PEAK_TFLOPS, ai * HBM_PEAK_GBS / 1e3)
        rows.append(dict(layer=i, shape=[L["shape"].C, L["shape"].K, L["shape"].H, L["shape"].R, L["shape"].stride],
                         us=round(ms * 1e3, 2), tflops=round(tf, 2), frac_mfma=round(tf / FP32_MFMA_PEAK_TFLOPS, 4),
                         frac_roofline=round(tf / ceiling, 4), gbs=round(L["bytes"] / (ms * 1e-3) / 1e9, 1),
                         tile=tile))
        kern_ms_sum += ms
        if args.sweep:
            # every candidate the picker ranks, timed; the model's prediction beside it
            shape = tuple(L["shape"])[1:]
            cands = []
            t_sweep = time.perf_counter()
            for v in P.conv_candidates(shape):
                try:
                    P.set_tile_override(v)
                    run_layer(L)
                    vms = time_calls(torch, lambda L=L: run_layer(L), 8, batches=2)
                except P.PolydlError:
                    continue
                pred = P.model_conv2d(shape, v).predicted_us
                cands.append(dict(us=round(vms * 1e3, 2), pred_us=round(pred, 2), cfg=v.as_dict()))
            t_sweep = time.perf_counter() - t_sweep
            P.set_tile_override(forced)
            cands.sort(key=lambda c: c["us"])
            best = cands[0]
            t_pick = time.perf_counter()
            pcfg, prep = P.pick_conv2d(shape)
            t_pick = time.perf_counter() - t_pick
            rows[-1].update(sweep_best_us=best["us"], sweep_best_tile=best["cfg"],
                            pick_over_best=round(best["us"] / (ms * 1e3), 4), candidates=len(cands),
                            predicted_us=round(prep.predicted_us, 2), pick_seconds=round(t_pick, 5),
                            sweep_seconds=round(t_sweep, 3))
            sweep_dump.append(dict(layer=i, shape=list(shape), picked=pcfg.as_dict(), picked_us=round(ms * 1e3, 2),
                                   candidates=cands))
    achieved = total_flops / (kern_ms_sum * 1e-3) / 1e12

    sg = []
    if not args.no_sgemm:
        for n in synth.SGEMM_SIZES:
            A, B, C0 = synth.sgemm_inputs(n, n, n, seed=n)
            dA, dB, dC = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), torch.from_numpy(C0).cuda()
            P.sgemm(dA, dB, dC)
            ms = time_calls(torch, lambda: P.sgemm(dA, dB, dC), 20 if n >= 2048 else 100)
            tf = 2.0 * n ** 3 / (ms * 1e-3) / 1e12
            sg.append(dict(n=n, us=round(ms * 1e3, 2), tflops=round(tf, 2),
                           frac_mfma=round(tf / FP32_MFMA_PEAK_TFLOPS, 4), tile=P.get_last_tile().as_dict()))
            del dA, dB, dC

    cpu = None
    if not args.no_cpu:
        import oracle
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        done_flops, t_cpu, desc = 0.0, 0.0, []
        for i, L in enumerate(layers):
            s = L["shape"]
            x, w, b = L["host"]
            nsub = max(1, min(s.N, int(round(s.N * 2.0e9 / L["flops"]))))  # about 2 GFLOP per layer
            t = time.perf_counter()
            oracle.conv2d_fwd(x[:nsub], w, bias=b, stride=s.stride, pad=s.pad, act="relu")
            t_cpu += time.perf_counter() - t
            done_flops += L["flops"] * nsub / s.N
            desc.append("%d" % nsub)
        cpu = dict(value=round(done_flops / t_cpu / 1e12, 6), unit="TFLOP/s", cores=threads, kind="oracle",
                   sample="full oracle conv+bias+ReLU on the first n images of each layer, n = [%s] of %d "
                          "(%.1f GFLOP, %.1f s)" % (",".join(desc), args.batch, done_flops / 1e9, t_cpu))

    result = {
        "metric": "conv fwd TFLOP/s, ResNet-50-shaped 8-layer suite (fp32, bias+ReLU fused), 1 GPU",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "configs[2]: ResNet-50-shaped conv suite, fp32 NCHW, N=%d, layers %s, "
                               "in N(0,1), wt N(0,2/(CRS)), bias U[-0.1,0.1), ReLU"
                               % (args.batch, "0-7 (all eight)" if len(chosen) == 8 else str(chosen)),
                   "frac_of_fp32_mfma_peak": round(value / FP32_MFMA_PEAK_TFLOPS, 4)},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 3), "peak": FP32_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / FP32_MFMA_PEAK_TFLOPS, 4), "traffic": None,
                     "kernel": "polydl::conv_kernel (all 8 layers, nominal 2*N*K*P*Q*C*R*S flops / sum of "
                               "per-layer mean launch durations)"},
        "cpu_baseline": cpu,
        "layers": rows,
        "sgemm": sg,
        "event_ms_per_step": round(e0.elapsed_time(e1) / args.steps, 4),
    }
    if args.sweep and args.sweep_out:
        with open(args.sweep_out, "w") as f:
            json.dump(sweep_dump, f)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
