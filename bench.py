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
BF16_MFMA_PEAK_TFLOPS = 2500.0  # dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0

# HBM-side bytes of one pass over the suite (all kernels of the eight layers, batch 32), from the L2
# fetch and write-back counters of two rocprofv3 --pmc runs, each scaled by what the same counter
# reads for a plain 256 MiB elementwise copy.  Valid only for the kernel sources they were taken
# with: their digest is kept beside them and the bench line reports null when it no longer matches.
HBM_TRAFFIC = {"csrc_sha256": "ca308b75c528b96f8d363a677445d90f14efc25b0ef3d95c21e6ee9a9820a0e3", "batch": 32, "filters": "tap", "fetch_bytes": 431151611, "write_bytes": 349757488}


# L2 fetch + write-back bytes of config 4 from two rocprofv3 --pmc runs of `bench.py --copy-probe --counter-pass
# fusion` (same scaling as above): the fused launch, and the convolution + bias + activation launches it replaces.
FUSION_TRAFFIC = {"csrc_sha256": "ca308b75c528b96f8d363a677445d90f14efc25b0ef3d95c21e6ee9a9820a0e3", "fused_bytes": 109952017, "separate_bytes": 135724285}

COLD_ROTATION_BYTES = 640 * 1000 * 1000


def csrc_digest():
    import hashlib
    d = os.path.join(ROOT, "paper_2006_02230_amd", "csrc")
    h = hashlib.sha256()
    for f in sorted(os.listdir(d)):
        if f.endswith((".hip", ".hpp", ".cpp", ".h")):
            h.update(f.encode())
            h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()


def conv_flops(s, P, Q):
    return 2.0 * s.N * s.K * P * Q * s.C * s.R * s.S


def conv_bytes(s, P, Q):
    """Compulsory traffic: read input and filter once, write output once."""
    return 4.0 * (s.N * s.C * s.H * s.W + s.K * s.C * s.R * s.S + s.N * s.K * P * Q + s.K)


def time_calls(torch, fn, reps, batches=3):
    """Median over batches of the mean time (ms) of reps back-to-back calls between two events."""
    out = []
    # clocks and caches as in steady state: keep the GPU busy with the same call for about 30 ms
    t_warm = time.perf_counter()
    while time.perf_counter() - t_warm < 0.03:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
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


def vendor_rows(torch, P, synth, layers):
    """The same layers and GEMMs through the ROCm libraries PyTorch calls (MIOpen, rocBLAS/hipBLASLt), timed
    like the per-layer rows.  Context only: nothing here enters value or roofline."""
    F = torch.nn.functional
    torch.backends.cudnn.benchmark = True        # let MIOpen search its kernels for each shape
    torch.backends.cudnn.allow_tf32 = False
    torch.backends.cuda.matmul.allow_tf32 = False
    fp32 = []
    for L in layers:
        s = L["shape"]
        ref = F.relu(F.conv2d(L["x"], L["w"], L["b"], stride=s.stride, padding=s.pad))   # first call: the search
        run = lambda: P.conv2d_fwd(L["x"], L["w"], L["b"], out=L["out"], stride=s.stride, pad=s.pad, act="relu",
                                   w_tap=L["wt"])
        run()
        diff = float((L["out"] - ref).abs().max())
        del ref
        conv_ms = time_calls(torch, lambda: F.conv2d(L["x"], L["w"], None, stride=s.stride, padding=s.pad), 30)
        full_ms = time_calls(torch, lambda: F.relu_(F.conv2d(L["x"], L["w"], L["b"], stride=s.stride, padding=s.pad)), 30)
        ours_ms = time_calls(torch, run, 30)
        fp32.append(dict(layer=L["index"], vendor_conv_us=round(conv_ms * 1e3, 1),
                         vendor_conv_bias_relu_us=round(full_ms * 1e3, 1), polydl_us=round(ours_ms * 1e3, 1),
                         max_abs_diff=diff))
    bf16 = []
    for i, s in enumerate(synth.RESNET50_SUITE(64)):
        x = torch.randn(s.N, s.C, s.H, s.W, device="cuda").bfloat16()
        w = (torch.randn(s.K, s.C, s.R, s.S, device="cuda") * (2.0 / (s.C * s.R * s.S)) ** 0.5).bfloat16()
        b = torch.zeros(s.K, device="cuda").bfloat16()
        row = dict(layer=i)
        for name, fmt in (("nchw", torch.contiguous_format), ("nhwc", torch.channels_last)):
            xc, wc = x.contiguous(memory_format=fmt), w.contiguous(memory_format=fmt)
            F.conv2d(xc, wc, b, stride=s.stride, padding=s.pad)
            ms = time_calls(torch, lambda: F.relu_(F.conv2d(xc, wc, b, stride=s.stride, padding=s.pad)), 30)
            row["vendor_%s_us" % name] = round(ms * 1e3, 1)
        bf16.append(row)
    sg = []
    for n in synth.SGEMM_SIZES:
        A = torch.randn(n, n, device="cuda"); B = torch.randn(n, n, device="cuda"); C = torch.zeros(n, n, device="cuda")
        reps = 20 if n >= 4096 else 50
        v_ms = time_calls(torch, lambda: torch.matmul(A, B, out=C), reps)
        o_ms = time_calls(torch, lambda: P.sgemm(A, B, C, beta=0.0), reps)
        sg.append(dict(n=n, vendor_us=round(v_ms * 1e3, 1), vendor_tflops=round(2.0 * n ** 3 / v_ms / 1e9, 1),
                       polydl_us=round(o_ms * 1e3, 1), polydl_tflops=round(2.0 * n ** 3 / o_ms / 1e9, 1)))
    return dict(note="ROCm libraries as PyTorch %s calls them (MIOpen %s with its kernel search on; torch.matmul), "
                     "same box, same process; bf16 rows: bf16 output, batch 64, to set beside the bf16 block "
                     "(which writes fp32)" % (torch.__version__, torch.backends.cudnn.version()),
                fp32_layers=fp32,
                fp32_sum_us=dict(vendor_conv=round(sum(r["vendor_conv_us"] for r in fp32), 1),
                                 vendor_conv_bias_relu=round(sum(r["vendor_conv_bias_relu_us"] for r in fp32), 1),
                                 polydl=round(sum(r["polydl_us"] for r in fp32), 1)),
                bf16_layers_n64=bf16,
                bf16_sum_us=dict(vendor_nchw=round(sum(r["vendor_nchw_us"] for r in bf16), 1),
                                 vendor_nhwc=round(sum(r["vendor_nhwc_us"] for r in bf16), 1)),
                sgemm=sg)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps first; about 50 ms of them bring the clocks to their steady state")
    ap.add_argument("--clock-warm-ms", type=float, default=150.0,
                    help="untimed load before the warm-up steps that brings the clocks to their steady state")
    ap.add_argument("--counter-pass", default="", choices=["", "fusion", "bf16"],
                    help="run only a few launches of one row, for a rocprofv3 --pmc pass: 'fusion' = the "
                         "fused call and the three separate kernels of config 4, 'bf16' = the bf16 suite")
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--sweep", action="store_true", help="also time every compiled variant per layer")
    ap.add_argument("--filters", default="tap", choices=["tap", "kcrs"],
                    help="'tap': every layer's filter is also given as its [K][R][S][C] copy, made once before "
                         "the timed region (polydl_conv2d_fwd_tap); 'kcrs': KCRS only (polydl_conv2d_fwd_act)")
    ap.add_argument("--suite", default="resnet", choices=["resnet", "heldout", "heldout2", "heldout3"],
                    help="'heldout', 'heldout2', 'heldout3': three sets of fourteen other CNN layer shapes (pick quality off the "
                         "fitting set; not the headline workload)")
    ap.add_argument("--sweep-out", default="", help="with --sweep: write every candidate's time to this JSON file")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-sgemm", action="store_true")
    ap.add_argument("--no-bf16", action="store_true", help="skip the bfloat16 rows (same suite at batch 64)")
    ap.add_argument("--no-fusion", action="store_true", help="skip the fused-versus-separate epilogue row")
    ap.add_argument("--copy-probe", action="store_true", help="first run three plain 256 MiB device copies "
                    "(an elementwise kernel of known traffic that calibrates the HBM byte counters)")
    ap.add_argument("--no-layer-rows", action="store_true", help="skip the per-layer timing loops (counter runs)")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold-cache per-layer timings")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--vendor", action="store_true",
                    help="also time the ROCm libraries on the same operands, as context beside the CPU baseline: "
                         "MIOpen through torch.nn.functional.conv2d (+ in-place ReLU) per layer, fp32 at --batch "
                         "and bf16 at batch 64, and torch.matmul for the square SGEMM sizes")
    ap.add_argument("--layers", default="", help="comma list of suite layers to run (default: all eight); "
                    "a subset is for profiling one kernel and changes the workload the line reports")
    ap.add_argument("--tile", default="", help="force a variant bm,bn,bk,wm,wn[,split_k[,layout[,raster]]] (profiling)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU; --gpus %d is not supported "
                 "(the path has no multi-GPU part: it would shard over the batch with no exchange step)" % args.gpus)

    import numpy as np
    import torch
    import synth
    import paper_2006_02230_amd as P

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)

    if args.copy_probe:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    if args.counter_pass == "fusion":
        # dispatch order per repetition: fused convolution; then convolution, bias_add, activation
        s = synth.CONFIG4
        x, w, b = synth.conv_inputs(s, seed=300, dist="normal", bias=True)
        Pq, Qq = synth.out_hw(s)
        dx, dw, db = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda()
        out = torch.empty((s.N, s.K, Pq, Qq), dtype=torch.float32, device="cuda")
        for _ in range(4):
            P.conv2d_fwd(dx, dw, db, out=out, stride=s.stride, pad=s.pad, act="relu")
            torch.cuda.synchronize()
            P.conv2d_fwd(dx, dw, None, out=out, stride=s.stride, pad=s.pad, act=None)
            P.bias_add(out, db)
            P.activation(out, "relu")
            torch.cuda.synchronize()
        print(json.dumps({"counter_pass": "fusion", "tile": P.get_last_tile().as_dict()}))
        return
    if args.counter_pass == "bf16":
        for i, s in enumerate(synth.RESNET50_SUITE(64)):
            x, w, b = synth.conv_inputs(s, seed=200 + i, dist="normal", bias=True)
            xb = torch.from_numpy(synth.to_bf16_bits(x).view(np.int16)).cuda()
            wb = torch.from_numpy(synth.to_bf16_bits(w).view(np.int16)).cuda()
            x8, w8 = P.nchw_to_nchwc_bf16(xb, 8), P.kcrs_to_kcrsck_bf16(wb, 8, 1)
            db = torch.from_numpy(b).cuda()
            for _ in range(3):
                P.conv2d_fwd_bf16_blocked(x8, w8, s.C, db, stride=s.stride, pad=s.pad, act="relu")
            torch.cuda.synchronize()
        print(json.dumps({"counter_pass": "bf16"}))
        return

    suite = (synth.RESNET50_SUITE(args.batch) if args.suite == "resnet"
             else synth.HELDOUT_SUITE(args.batch, {"heldout": 1, "heldout2": 2, "heldout3": 3}[args.suite]))
    if args.suite != "resnet":
        args.no_bf16 = args.no_fusion = args.no_sgemm = True
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
        dw = torch.from_numpy(w).cuda()
        layers.append(dict(shape=s, P=Pq, Q=Qq, x=torch.from_numpy(x).cuda(), w=dw,
                           wt=P.filter_tap_copy(dw) if args.filters == "tap" else None,
                           b=torch.from_numpy(b).cuda(),
                           out=torch.empty((s.N, s.K, Pq, Qq), dtype=torch.float32, device="cuda"),
                           index=i, flops=conv_flops(s, Pq, Qq), bytes=conv_bytes(s, Pq, Qq), host=(x, w, b)))

    def run_layer(L, tap=True):
        s = L["shape"]
        P.conv2d_fwd(L["x"], L["w"], L["b"], out=L["out"], stride=s.stride, pad=s.pad, act="relu",
                     w_tap=L["wt"] if tap else None)

    def step(tap=True):
        for L in layers:
            run_layer(L, tap)

    P.set_tile_override(forced)
    # the GPU's clocks take tens of milliseconds of load to reach their steady state; a short --warmup
    # would otherwise put the ramp inside the timed steps.  Untimed, before the W warm-up steps.
    t_warm = time.perf_counter()
    while (time.perf_counter() - t_warm) * 1e3 < args.clock_warm_ms:
        for _ in range(5):
            step()
        torch.cuda.synchronize()
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

    # the same step recorded once into a HIP graph and replayed: what a caller that keeps the launch
    # sequence pays per step (no per-call argument marshalling, launches already formed)
    graph_ms = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            step()                      # scratch memory of this stream exists before the capture
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
            for _ in range(min(args.warmup, 20)):
                graph.replay()
            torch.cuda.synchronize()
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            tg = time.perf_counter()
            g0.record()
            for _ in range(args.steps):
                graph.replay()
            g1.record()
            torch.cuda.synchronize()
            graph_ms = (time.perf_counter() - tg) * 1e3 / args.steps
        del graph
    total_bytes = sum(L["bytes"] for L in layers)
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    # per-layer kernel time: back-to-back launches of one layer between two events on the launch stream
    rows = []
    sweep_dump = []
    kern_ms_sum = 0.0
    for L in ([] if args.no_layer_rows else layers):
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
        if not args.no_cold:
            # the same call over a rotation of distinct operand sets larger than the 256 MB last-level
            # cache taken twice, so that no call finds its operands or its output lines cached
            nsets = max(2, int(-(-COLD_ROTATION_BYTES // L["bytes"])))
            sets = [(L["x"].clone(), L["w"].clone(), L["b"].clone(), torch.empty_like(L["out"]),
                     None if L["wt"] is None else L["wt"].clone()) for _ in range(nsets)]
            turn = [0]

            def run_cold(L=L, sets=sets, turn=turn):
                x, w, b, o, wt = sets[turn[0] % len(sets)]
                turn[0] += 1
                P.conv2d_fwd(x, w, b, out=o, stride=L["shape"].stride, pad=L["shape"].pad, act="relu", w_tap=wt)

            cms = time_calls(torch, run_cold, max(reps, nsets))
            rows[-1].update(cold_us=round(cms * 1e3, 2), cold_sets=nsets,
                            cold_gbs=round(L["bytes"] / (cms * 1e-3) / 1e9, 1),
                            cold_frac_roofline=round(L["flops"] / (cms * 1e-3) / 1e12 / ceiling, 4))
            del sets
        if args.sweep:
            # every candidate the picker ranks, timed; the model's prediction beside it
            shape = tuple(L["shape"])[1:]
            cands = []
            t_sweep = time.perf_counter()
            for v in P.conv_candidates(shape, tap=L["wt"] is not None):
                try:
                    P.set_tile_override(v)
                    run_layer(L)
                    vms = time_calls(torch, lambda L=L: run_layer(L), 8, batches=3)
                except P.PolydlError:
                    continue
                rep = P.model_conv2d(shape, v)
                cands.append(dict(us=round(vms * 1e3, 2), pred_us=round(rep.predicted_us, 2),
                                  data_us=round(rep.mem_us, 3), mfma_us=round(rep.mfma_us, 3),
                                  eq1_cost=rep.eq1_cost, cfg=v.as_dict()))
            t_sweep = time.perf_counter() - t_sweep
            P.set_tile_override(forced)
            cands.sort(key=lambda c: c["us"])
            best = cands[0]
            t_pick = time.perf_counter()
            pcfg, prep = P.pick_conv2d(shape)
            t_pick = time.perf_counter() - t_pick
            prep = P.model_conv2d(shape, P.TileCfg(**tile))     # the prediction for the variant that ran
            # ablation: what each part of the model would have picked alone, on the same timings --
            # equation (1) over the placed working sets; the data term (equation (1) weighted by the
            # bytes that move); the matrix-core term
            alone = {}
            for key in ("eq1_cost", "data_us", "mfma_us"):
                c0 = min(cands, key=lambda c: (c[key], c["pred_us"]))
                alone[key + "_alone_over_best"] = round(best["us"] / c0["us"], 4)
            rows[-1].update(alone)
            rows[-1].update(sweep_best_us=best["us"], sweep_best_tile=best["cfg"],
                            pick_over_best=round(best["us"] / (ms * 1e3), 4), candidates=len(cands),
                            predicted_us=round(prep.predicted_us, 2), pick_seconds=round(t_pick, 5),
                            sweep_seconds=round(t_sweep, 3))
            # the learned ranking's choice among the same candidates (tournament of the pairwise network),
            # timed like the model's pick
            if os.path.exists(P.RANKER_PARAMS_PATH):
                P.ranker_load()
                t_learn = time.perf_counter()
                if L["wt"] is None:
                    lcfg, _, lwins, lgames = P.pick_conv2d_learned(shape)
                else:
                    # the same tournament over the candidates ranked with the filter copy
                    lc = P.conv_candidates(shape, tap=True)
                    w_l, order_l = P.ranker_tournament([P.ranker_stats_conv2d(shape, c) for c in lc])
                    lcfg, lwins, lgames = lc[order_l[0]], w_l[order_l[0]], 2 * (len(lc) - 1)
                t_learn = time.perf_counter() - t_learn
                P.set_tile_override(lcfg)
                run_layer(L)
                lms = time_calls(torch, lambda L=L: run_layer(L), reps)
                P.set_tile_override(forced)
                rows[-1].update(learned_tile=lcfg.as_dict(), learned_us=round(lms * 1e3, 2),
                                learned_over_best=round(best["us"] / (lms * 1e3), 4),
                                learned_wins=[lwins, lgames], learned_pick_seconds=round(t_learn, 4))
            sweep_dump.append(dict(layer=i, shape=list(shape), picked=tile, picked_us=round(ms * 1e3, 2),
                                   candidates=cands))
    if args.no_layer_rows:
        kern_ms_sum = e0.elapsed_time(e1) / args.steps
    achieved = total_flops / (kern_ms_sum * 1e-3) / 1e12

    # the same suite without the filter copies (polydl_conv2d_fwd_act on NCHW / KCRS alone): the step
    # timed the same way, and each layer's launch time
    kcrs_only = None
    if args.filters == "tap" and not args.no_layer_rows:
        for _ in range(min(args.warmup, 20)):
            step(tap=False)
        torch.cuda.synchronize()
        tk = time.perf_counter()
        for _ in range(args.steps):
            step(tap=False)
        torch.cuda.synchronize()
        k_ms = (time.perf_counter() - tk) * 1e3 / args.steps
        k_us = []
        for L in layers:
            k_us.append(round(time_calls(torch, lambda L=L: run_layer(L, tap=False), 30) * 1e3, 2))
        kcrs_only = dict(ms_per_step=round(k_ms, 4), value=round(total_flops / (k_ms * 1e-3) / 1e12, 3),
                         layers_us=k_us, achieved=round(total_flops / (sum(k_us) * 1e-6) / 1e12, 3),
                         frac=round(total_flops / (sum(k_us) * 1e-6) / 1e12 / FP32_MFMA_PEAK_TFLOPS, 4))

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
            if args.sweep:
                # every candidate the SGEMM picker ranks; candidates the model puts beyond 4x its best
                # prediction are not timed (they would take most of the sweep's time and none is near)
                pcfg, prep = P.pick_sgemm(n, n, n)
                cands = []
                t_sweep = time.perf_counter()
                for v in P.sgemm_candidates(n, n, n):
                    pred = P.model_sgemm(n, n, n, v).predicted_us
                    if pred > 4.0 * prep.predicted_us:
                        continue
                    try:
                        P.set_tile_override(v)
                        P.sgemm(dA, dB, dC)
                        vms = time_calls(torch, lambda: P.sgemm(dA, dB, dC), 4 if n >= 2048 else 10, batches=2)
                    except P.PolydlError:
                        continue
                    cands.append(dict(us=round(vms * 1e3, 2), pred_us=round(pred, 2), cfg=v.as_dict()))
                t_sweep = time.perf_counter() - t_sweep
                P.set_tile_override(forced)
                by_time = sorted(cands, key=lambda c: c["us"])
                by_pred = sorted(cands, key=lambda c: c["pred_us"])
                top = max(1, len(cands) // 20)   # the paper reports its GEMM picks among the top 5 % of the ranking
                best_in_top = min(c["us"] for c in by_pred[:top])
                sg[-1].update(sweep_best_us=by_time[0]["us"], sweep_best_tile=by_time[0]["cfg"],
                              pick_over_best=round(by_time[0]["us"] / (ms * 1e3), 4), candidates=len(cands),
                              predicted_us=round(prep.predicted_us, 2), sweep_seconds=round(t_sweep, 3),
                              top5pct_best_us=best_in_top,
                              top5pct_over_best=round(by_time[0]["us"] / best_in_top, 4))
            del dA, dB, dC
        # the (M, N, K) of the paper's GEMM-size table; values do not matter for the timing
        for (M, N, K) in synth.PAPER_GEMM_SIZES:
            dA = torch.rand((M, K), dtype=torch.float32, device="cuda") - 0.5
            dB = torch.rand((K, N), dtype=torch.float32, device="cuda") - 0.5
            dC = torch.zeros((M, N), dtype=torch.float32, device="cuda")
            P.sgemm(dA, dB, dC)
            ms = time_calls(torch, lambda: P.sgemm(dA, dB, dC), 10)
            tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
            sg.append(dict(mnk=[M, N, K], us=round(ms * 1e3, 2), tflops=round(tf, 2),
                           frac_mfma=round(tf / FP32_MFMA_PEAK_TFLOPS, 4), tile=P.get_last_tile().as_dict()))
            del dA, dB, dC

    # the same suite with bfloat16 inputs (fp32 accumulate and output) at batch 64: operands already in
    # the 8-channel blocked layouts, as a network that stays in that layout between layers holds them
    bf = None
    if not args.no_bf16 and len(chosen) == 8 and forced is None:
        bf_rows, bf_ms, bf_flops, tr_ms = [], 0.0, 0.0, 0.0
        for i, s in enumerate(synth.RESNET50_SUITE(64)):
            x, w, b = synth.conv_inputs(s, seed=200 + i, dist="normal", bias=True)
            Pq, Qq = synth.out_hw(s)
            xb = torch.from_numpy(synth.to_bf16_bits(x).view(np.int16)).cuda()
            wb = torch.from_numpy(synth.to_bf16_bits(w).view(np.int16)).cuda()
            db = torch.from_numpy(b).cuda()
            x8, w8 = P.nchw_to_nchwc_bf16(xb, 8), P.kcrs_to_kcrsck_bf16(wb, 8, 1)
            t_tr = time_calls(torch, lambda: (P.nchw_to_nchwc_bf16(xb, 8, out=x8),
                                              P.kcrs_to_kcrsck_bf16(wb, 8, 1, out=w8)), 10)
            out = torch.empty((s.N, s.K, Pq, Qq), dtype=torch.float32, device="cuda")
            fn = lambda: P.conv2d_fwd_bf16_blocked(x8, w8, s.C, db, out=out, stride=s.stride, pad=s.pad, act="relu")
            fn()
            ms = time_calls(torch, fn, 20)
            fl = conv_flops(s, Pq, Qq)
            # compulsory traffic with 2-byte operands (blocked tensors as they lie: channels padded to
            # eight) and the fp32 output; the layer's ceiling is the lower of the two rooflines
            by = 2.0 * (x8.numel() + w8.numel()) + 4.0 * (s.N * s.K * Pq * Qq + s.K)
            tfl = fl / (ms * 1e-3) / 1e12
            ceil_tf = min(BF16_MFMA_PEAK_TFLOPS, fl / by * HBM_PEAK_GBS / 1e3)
            bf_rows.append(dict(layer=i, us=round(ms * 1e3, 2), tflops=round(tfl, 2),
                                frac_mfma=round(tfl / BF16_MFMA_PEAK_TFLOPS, 4),
                                gbs=round(by / (ms * 1e-3) / 1e9, 1), ceiling_tflops=round(ceil_tf, 1),
                                bound="mfma" if ceil_tf >= BF16_MFMA_PEAK_TFLOPS else "hbm",
                                frac_roofline=round(tfl / ceil_tf, 4),
                                layout_us=round(t_tr * 1e3, 2), tile=P.get_last_tile().as_dict()))
            if args.sweep:
                shape = tuple(s)[1:]
                cands = []
                t_sweep = time.perf_counter()
                for v in P.conv_candidates_bf16(shape):
                    try:
                        P.set_tile_override(v)
                        fn()
                        vms = time_calls(torch, fn, 8, batches=3)
                        pred = P.model_conv2d_bf16(shape, v)
                    except P.PolydlError:
                        continue
                    cands.append(dict(us=round(vms * 1e3, 2), pred_us=round(pred, 2), cfg=v.as_dict()))
                t_sweep = time.perf_counter() - t_sweep
                P.set_tile_override(None)
                cands.sort(key=lambda c: c["us"])
                t_pick = time.perf_counter()
                pcfg, pus = P.pick_conv2d_bf16(shape)
                t_pick = time.perf_counter() - t_pick
                bf_rows[-1].update(sweep_best_us=cands[0]["us"], sweep_best_tile=cands[0]["cfg"],
                                   pick_over_best=round(cands[0]["us"] / (ms * 1e3), 4), candidates=len(cands),
                                   predicted_us=round(pus, 2), pick_seconds=round(t_pick, 5),
                                   sweep_seconds=round(t_sweep, 3))
            bf_ms += ms
            tr_ms += t_tr
            bf_flops += fl
            del xb, wb, x8, w8, out
        tf = bf_flops / (bf_ms * 1e-3) / 1e12
        ideal_ms = sum(conv_flops(s, *synth.out_hw(s)) / (r["ceiling_tflops"] * 1e12) * 1e3
                       for s, r in zip(synth.RESNET50_SUITE(64), bf_rows))
        bf = dict(roofline={"bound": "min(bf16 mfma, hbm) per layer", "achieved": round(tf, 2),
                            "peak": round(bf_flops / (ideal_ms * 1e-3) / 1e12, 1), "unit": "TFLOP/s",
                            "frac": round(ideal_ms / bf_ms, 4),
                            "note": "peak = suite flops / sum over layers of flops / min(2500 TFLOP/s, AI * 8 TB/s)"},
                  workload="configs[4]: the same eight layers, bf16 inputs in NCHW8c / KCRS8c, fp32 accumulate "
                           "and output, N=64, bias+ReLU fused",
                  tflops=round(tf, 2), frac_of_bf16_mfma_peak=round(tf / BF16_MFMA_PEAK_TFLOPS, 4),
                  us_per_pass=round(bf_ms * 1e3, 1), layout_transform_us_per_pass=round(tr_ms * 1e3, 1),
                  tflops_with_layout_transforms=round(bf_flops / ((bf_ms + tr_ms) * 1e-3) / 1e12, 2),
                  layers=bf_rows)

    # convolution + bias + ReLU as one kernel against the same three operators as three kernels
    fusion = None
    if not args.no_fusion and forced is None:
        s = synth.CONFIG4
        x, w, b = synth.conv_inputs(s, seed=300, dist="normal", bias=True)
        Pq, Qq = synth.out_hw(s)
        dx, dw, db = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda()
        out = torch.empty((s.N, s.K, Pq, Qq), dtype=torch.float32, device="cuda")
        fused = lambda: P.conv2d_fwd(dx, dw, db, out=out, stride=s.stride, pad=s.pad, act="relu")

        def separate():
            P.conv2d_fwd(dx, dw, None, out=out, stride=s.stride, pad=s.pad, act=None)
            P.bias_add(out, db)
            P.activation(out, "relu")
        conv_only = lambda: P.conv2d_fwd(dx, dw, None, out=out, stride=s.stride, pad=s.pad, act=None)
        fused(); separate(); conv_only()
        # the three are timed in turn, several times over, so that a drift of the clocks hits all alike
        samples = {"f": [], "s": [], "c": []}
        for _ in range(5):
            samples["f"].append(time_calls(torch, fused, 20, batches=1))
            samples["s"].append(time_calls(torch, separate, 20, batches=1))
            samples["c"].append(time_calls(torch, conv_only, 20, batches=1))
        t_f, t_s, t_c = (sorted(samples[k])[2] for k in ("f", "s", "c"))
        ob = 4.0 * s.N * s.K * Pq * Qq
        fusion = dict(workload="configs[3]: conv+bias+ReLU, N=%d C=K=%d %dx%d 3x3" % (s.N, s.C, s.H, s.W),
                      fused_us=round(t_f * 1e3, 2), separate_us=round(t_s * 1e3, 2), conv_only_us=round(t_c * 1e3, 2),
                      speedup=round(t_s / t_f, 3),
                      output_bytes=ob, algorithmic_bytes_saved=4 * ob,
                      measured_bytes_saved=(FUSION_TRAFFIC["separate_bytes"] - FUSION_TRAFFIC["fused_bytes"]
                                            if FUSION_TRAFFIC["csrc_sha256"] == csrc_digest() else None),
                      measured_bytes=({"fused": FUSION_TRAFFIC["fused_bytes"], "separate": FUSION_TRAFFIC["separate_bytes"],
                                       "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/config4_fusion_bytes.md"}
                                      if FUSION_TRAFFIC["csrc_sha256"] == csrc_digest() else None),
                      note="the two extra kernels each read and write the whole output once: four passes "
                           "over it that the fused epilogue never makes")
        # the element-wise operator BEFORE the convolution: fused into the operand staging against a
        # separate in-place pass over the input (ReLU is idempotent, so repeating it changes nothing)
        pre_fused = lambda: P.conv2d_fwd(dx, dw, db, out=out, stride=s.stride, pad=s.pad, act="relu", pre_act="relu")

        def pre_separate():
            P.activation(dx, "relu")
            P.conv2d_fwd(dx, dw, db, out=out, stride=s.stride, pad=s.pad, act="relu")
        pre_fused(); pre_separate()
        samples = {"f": [], "s": []}
        for _ in range(5):
            samples["f"].append(time_calls(torch, pre_fused, 20, batches=1))
            samples["s"].append(time_calls(torch, pre_separate, 20, batches=1))
        t_pf, t_ps = (sorted(samples[k])[2] for k in ("f", "s"))
        fusion["relu_before"] = dict(workload="ReLU + conv+bias+ReLU on the same layer", fused_us=round(t_pf * 1e3, 2),
                                     separate_us=round(t_ps * 1e3, 2), speedup=round(t_ps / t_pf, 3),
                                     input_bytes=4.0 * s.N * s.C * s.H * s.W,
                                     algorithmic_bytes_saved=8.0 * s.N * s.C * s.H * s.W)
        del dx, dw, out

    # batch normalisation + ReLU in one pass against the two operators as two kernels, on the
    # output tensors of the suite layers (memory bound: one read and one write per element)
    bn = None
    if not args.no_fusion and forced is None and len(chosen) == 8:
        bn_rows, t_fused, t_sep, nbytes = [], 0.0, 0.0, 0.0
        for L in layers:
            y = L["out"]
            K = y.shape[1]
            g, be = torch.rand(K, device="cuda") + 0.5, torch.rand(K, device="cuda") - 0.5
            mu, va = torch.rand(K, device="cuda") - 0.5, torch.rand(K, device="cuda") + 0.5
            dst = torch.empty_like(y)
            fused = lambda: P.bnorm_fwd(y, g, be, mu, va, 1e-5, out=dst, act="relu")

            def separate():
                P.bnorm_fwd(y, g, be, mu, va, 1e-5, out=dst, act=None)
                P.activation(dst, "relu")
            tf_, ts_ = [], []
            for _ in range(3):
                tf_.append(time_calls(torch, fused, 20, batches=1))
                ts_.append(time_calls(torch, separate, 20, batches=1))
            f_ms, s_ms = sorted(tf_)[1], sorted(ts_)[1]
            b = 8.0 * y.numel()
            bn_rows.append(dict(layer=L["index"], elements=y.numel(), fused_us=round(f_ms * 1e3, 2),
                                separate_us=round(s_ms * 1e3, 2), fused_gbs=round(b / (f_ms * 1e-3) / 1e9, 1),
                                frac_hbm=round(b / (f_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)))
            t_fused += f_ms
            t_sep += s_ms
            nbytes += b
            del dst
        bn = dict(workload="bnorm + ReLU on the eight NKPQ output tensors of the suite (N=%d), out of place" % args.batch,
                  fused_us=round(t_fused * 1e3, 1), separate_us=round(t_sep * 1e3, 1),
                  speedup=round(t_sep / t_fused, 3), fused_gbs=round(nbytes / (t_fused * 1e-3) / 1e9, 1),
                  # the kernel's rate is read on the largest tensor (the small ones show the launch cadence)
                  roofline={"bound": "hbm", "achieved": max(r["fused_gbs"] for r in bn_rows),
                            "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": round(max(r["fused_gbs"] for r in bn_rows) / HBM_PEAK_GBS, 4),
                            "kernel": "polydl::bnorm_act_kernel on the largest output tensor of the suite "
                                      "(%.0f MB read + written)" % (8.0 * max(r["elements"] for r in bn_rows) / 1e6)},
                  layers=bn_rows)

    # the blocked-layout transforms (pure permutations, memory bound): activations NCHW -> NCHW16c
    # and back, filters KCRS -> KCRS16c16k, on the tensors of the suite layers
    lay = None
    if not args.no_fusion and forced is None and len(chosen) == 8:
        lay_rows, t_all, b_all = [], 0.0, 0.0
        for L in layers:
            s = L["shape"]
            xb = P.nchw_to_nchwc(L["x"], 16)
            xr = torch.empty_like(L["x"])
            wb = P.kcrs_to_kcrsck(L["w"], 16, 16)
            t_fw = time_calls(torch, lambda: P.nchw_to_nchwc(L["x"], 16, out=xb), 20, batches=3)
            t_bw = time_calls(torch, lambda: P.nchwc_to_nchw(xb, s.C, out=xr), 20, batches=3)
            t_w = time_calls(torch, lambda: P.kcrs_to_kcrsck(L["w"], 16, 16, out=wb), 20, batches=3)
            # bytes moved: the source once and the (zero-padded) blocked tensor once
            b_act = 4.0 * (L["x"].numel() + xb.numel())
            lay_rows.append(dict(layer=L["index"], act_to_blocked_us=round(t_fw * 1e3, 2),
                                 act_to_blocked_gbs=round(b_act / (t_fw * 1e-3) / 1e9, 1),
                                 act_from_blocked_us=round(t_bw * 1e3, 2),
                                 act_from_blocked_gbs=round(b_act / (t_bw * 1e-3) / 1e9, 1),
                                 filter_pack_us=round(t_w * 1e3, 2)))
            t_all += t_fw
            b_all += b_act
            del xb, xr, wb
        # the suite's inputs are small (3 - 25 MB): their rows mostly show the launch cadence.  The
        # kernel's own rate is taken on an activation of the size the early layers produce.
        big = torch.randn((args.batch, 64, 112, 112), dtype=torch.float32, device="cuda")
        big_b = P.nchw_to_nchwc(big, 16)
        big_r = torch.empty_like(big)
        t_bf = time_calls(torch, lambda: P.nchw_to_nchwc(big, 16, out=big_b), 20, batches=3)
        t_bb = time_calls(torch, lambda: P.nchwc_to_nchw(big_b, 64, out=big_r), 20, batches=3)
        b_big = 8.0 * big.numel()
        lay = dict(workload="NCHW <-> NCHW16c on the suite inputs (N=%d) and on a %d x 64 x 112 x 112 activation, "
                            "KCRS -> KCRS16c16k on the suite filters; back-to-back launches into preallocated "
                            "tensors" % (args.batch, args.batch),
                   roofline={"bound": "hbm", "achieved": round(b_big / (t_bf * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": round(b_big / (t_bf * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                             "kernel": "polydl::nchwc_wide_kernel, NCHW -> NCHW16c of the large activation "
                                       "(%.0f MB read + written per launch)" % (b_big / 1e6)},
                   large=dict(to_blocked_us=round(t_bf * 1e3, 2), to_blocked_gbs=round(b_big / (t_bf * 1e-3) / 1e9, 1),
                              from_blocked_us=round(t_bb * 1e3, 2), from_blocked_gbs=round(b_big / (t_bb * 1e-3) / 1e9, 1)),
                   suite_gbs=round(b_all / (t_all * 1e-3) / 1e9, 1),
                   layers=lay_rows)
        del big, big_b, big_r

    # config 1: one small convolution (N = 1): a latency case (1.5 us of matrix-core work), with the oracle
    # beside it on one thread and on all of them
    cfg1 = None
    if not args.no_fusion and forced is None:
        s = synth.CONFIG1
        x, w, _ = synth.conv_inputs(s, seed=0, dist="uniform")
        Pq, Qq = synth.out_hw(s)
        dx, dw = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        out = torch.empty((s.N, s.K, Pq, Qq), dtype=torch.float32, device="cuda")
        fn = lambda: P.conv2d_fwd(dx, dw, None, out=out, stride=s.stride, pad=s.pad, act=None)
        fn()
        ms = time_calls(torch, fn, 200)
        fl = conv_flops(s, Pq, Qq)
        cfg1 = dict(workload="configs[0]: N=1 C=K=64 56x56 3x3 s1 p1, no bias, U[-1,1), seed 0",
                    us=round(ms * 1e3, 2), tflops=round(fl / (ms * 1e-3) / 1e12, 2),
                    frac_mfma=round(fl / (ms * 1e-3) / 1e12 / FP32_MFMA_PEAK_TFLOPS, 4),
                    mfma_time_at_peak_us=round(fl / (FP32_MFMA_PEAK_TFLOPS * 1e12) * 1e6, 2),
                    tile=P.get_last_tile().as_dict())
        if not args.no_cpu:
            import ctypes
            import oracle
            omp = ctypes.CDLL("libgomp.so.1")
            all_threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
            for label, nt in (("oracle_1_thread_ms", 1), ("oracle_all_threads_ms", all_threads)):
                omp.omp_set_num_threads(nt)
                oracle.conv2d_fwd(x, w, stride=s.stride, pad=s.pad)
                t = time.perf_counter()
                reps = 3 if nt == 1 else 20
                for _ in range(reps):
                    oracle.conv2d_fwd(x, w, stride=s.stride, pad=s.pad)
                cfg1[label] = round((time.perf_counter() - t) / reps * 1e3, 3)
            omp.omp_set_num_threads(all_threads)
            cfg1["oracle_threads"] = all_threads
        del dx, dw, out

    cpu = None
    if not args.no_cpu:
        import oracle
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        done_flops, t_cpu, passes = 0.0, 0.0, 0
        nsub = min(args.batch, 8)          # the first 8 images of every layer: a quarter of the batch
        while t_cpu < 12.0 and passes < 40:
            for L in layers:
                s = L["shape"]
                x, w, b = L["host"]
                t = time.perf_counter()
                oracle.conv2d_fwd(x[:nsub], w, bias=b, stride=s.stride, pad=s.pad, act="relu")
                t_cpu += time.perf_counter() - t
                done_flops += L["flops"] * nsub / s.N
            passes += 1
        cpu = dict(value=round(done_flops / t_cpu / 1e12, 6), unit="TFLOP/s", cores=threads, kind="oracle",
                   sample="fp64 oracle conv+bias+ReLU on the first %d of %d images of every layer, %d passes "
                          "(%.1f GFLOP in %.1f s)" % (nsub, args.batch, passes, done_flops / 1e9, t_cpu))

    vendor = None
    if args.vendor:
        vendor = vendor_rows(torch, P, synth, layers)

    traffic = None
    if (HBM_TRAFFIC["csrc_sha256"] == csrc_digest() and args.batch == HBM_TRAFFIC["batch"] and len(chosen) == 8
            and args.suite == "resnet" and args.filters == HBM_TRAFFIC.get("filters", "kcrs")
            and forced is None):
        traffic = HBM_TRAFFIC["fetch_bytes"] + HBM_TRAFFIC["write_bytes"]
    result = {
        "metric": "conv fwd TFLOP/s, ResNet-50-shaped 8-layer suite (fp32, bias+ReLU fused), 1 GPU",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": ("configs[2]: ResNet-50-shaped conv suite, fp32 NCHW, N=%d, layers %s, "
                                "in N(0,1), wt N(0,2/(CRS)), bias U[-0.1,0.1), ReLU"
                                % (args.batch, "0-7 (all eight)" if len(chosen) == 8 else str(chosen)))
                               if args.suite == "resnet" else
                               ("held-out CNN layer shapes (not the headline workload), fp32 NCHW, N=%d, layers %s"
                                % (args.batch, str(chosen))),
                   "filters": ("KCRS, and the same filter as [K][R][S][C] (KCRSck with bc = C, bk = 1) made once "
                               "before the timed region and passed with it (polydl_conv2d_fwd_tap); the row "
                               "kcrs_only times the suite without the copies") if args.filters == "tap"
                              else "KCRS only (polydl_conv2d_fwd_act)",
                   "frac_of_fp32_mfma_peak": round(value / FP32_MFMA_PEAK_TFLOPS, 4),
                   "clock_warm_ms": args.clock_warm_ms},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 3), "peak": FP32_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / FP32_MFMA_PEAK_TFLOPS, 4), "traffic": traffic,
                     "traffic_unit": "bytes per suite pass (L2 fetch + write-back); algorithmic: %d" % total_bytes,
                     "traffic_source": "not measured in this run: counters of an earlier rocprofv3 --pmc run of the "
                                       "same kernel sources (digest checked), null when the sources have changed",
                     "kernel": "polydl::conv_kernel / polydl::conv_patch_kernel as picked per layer (all 8 "
                               "layers, nominal 2*N*K*P*Q*C*R*S flops / sum of per-layer mean launch durations)"},
        "cpu_baseline": cpu,
        "layers": rows,
        "kcrs_only": kcrs_only,
        "sgemm": sg,
        "bf16": bf,
        "fusion": fusion,
        "config1": cfg1,
        "bnorm_relu": bn,
        "layouts": lay,
        "vendor": vendor,
        "event_ms_per_step": round(e0.elapsed_time(e1) / args.steps, 4),
        "graph_ms_per_step": None if graph_ms is None else round(graph_ms, 4),
        "value_graph": None if graph_ms is None else round(total_flops / (graph_ms * 1e-3) / 1e12, 3),
    }
    if args.sweep and args.sweep_out:
        with open(args.sweep_out, "w") as f:
            json.dump(sweep_dump, f)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
