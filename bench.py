#!/usr/bin/env python3
"""Throughput of the binary-network forward pass on one MI355X.

A step is one bnn_forward over one batch: Config 3 of the benchmark set (440 -> 6 x 2048 -> 3400, binary
weights and binary activations, 4096 synthetic frames, 32-bit packed words), all seven layers, inputs and
the packed model already resident in HBM.  The K timed steps are issued round-robin to --streams HIP streams (default 4:
four batches in flight, as a server with queued batches runs them); "single_stream" in the line is the same K steps one
after the other.  Prints ONE JSON line with frames/s, binary TOPS, the roofline
of the dominant kernel (timed live with HIP events on the launch stream) and the CPU oracle timed on the
host cores on a bounded sample of the same workload.

The line also carries "configs": a short run of the other benchmark configurations (C1, C2, C4 and two corners of the
C5 product sweep) beside C3's own figures; --no-configs leaves them out.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-configs] [--arm mfma|mfma_i8|valu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Published MI355X peaks used as roofline denominators.
PEAK_MFMA_FP4_TFLOPS = 10100.0          # dense fp4/fp6 MFMA
PEAK_MFMA_INT8_TOPS = 5000.0            # dense int8 MFMA
PEAK_VALU_LANE_OPS = 256 * 4 * 16 * 2.4e9   # 256 CUs x 4 SIMD16 x 2.4 GHz = 39.3 T lane-ops/s
PEAK_FP32_VALU_TFLOPS = 2 * PEAK_VALU_LANE_OPS / 1e12      # one v_fma_f32 per lane-op, unpacked: 78.6 TFLOP/s
PEAK_XOR_POPC_TOPS = 2 * 32 * PEAK_VALU_LANE_OPS / 2 / 1e12  # xor + bcnt per 32 binary MACs: 1258 binary TOP/s


def gemm_sweep(args, bnn, workloads, G, torch) -> int:
    """Isolated binary x binary GEMM (Config 5): int32 = K - 2 popcount(XOR), one JSON line per shape and arm."""
    for kv in args.opt:
        key, val = kv.split("=")
        bnn.bnn_set_option(getattr(bnn, "BNN_OPT_" + key), int(val))
    for shape in workloads.GEMM_SWEEP:
        for arm_name, arm in (("mfma", bnn.BNN_ARM_MFMA), ("mfma_i8", bnn.BNN_ARM_MFMA_I8), ("valu", bnn.BNN_ARM_VALU_XOR)):
            reps = 10 if shape.M * shape.K * shape.N < 1e12 else 3
            line = time_gemm(shape, arm, reps, bnn, workloads, G, torch)
            line["arm"] = arm_name
            print(json.dumps(line), flush=True)
    return 0


def time_config(cid, steps, workloads, G, torch) -> dict:
    """bnn_forward on one configuration: 3 warm-up steps, then `steps` timed ones (host clock around a synchronize)."""
    cfg = workloads.CONFIGS[cid]
    Ws, bs = workloads.make_net_params(cfg)
    model = G.GpuModel(Ws, bs, cfg.hidden_act, cfg.word_bits, real_weight_layers=cfg.real_weight_layers)
    X = G.to_dev(workloads.make_frames(cfg))
    out = torch.empty((cfg.M, model.N_out), dtype=torch.float32, device=G.DEV)
    for _ in range(3):
        model.forward(X, out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        model.forward(X, out)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    line = {"workload": cfg.name, "batch_frames": cfg.M, "steps": steps, "ms_per_step": round(ms, 4),
            "frames_per_s": round(cfg.M / (ms * 1e-3), 1),
            "tops_all_layers": round(2.0 * cfg.macs_per_frame() * cfg.M / (ms * 1e-3) / 1e12, 2),
            "binbin_share_of_macs": round(cfg.binbin_macs_per_frame() / cfg.macs_per_frame(), 3)}
    del model, X, out, Ws, bs
    torch.cuda.empty_cache()
    return line


def time_gemm(shape, arm, reps, bnn, workloads, G, torch) -> dict:
    """The isolated binary x binary product (Config 5) at one shape, int32 outputs."""
    M, K, N = shape.M, shape.K, shape.N
    A = G.to_dev(workloads.random_words(0, 500 + workloads.TENSOR_ABITS, M, K // 32))
    B = G.to_dev(workloads.random_words(0, 500 + workloads.TENSOR_BBITS, N, K // 32))
    Y = torch.empty((M, N), dtype=torch.int32, device=G.DEV)

    def call():
        bnn.bnn_layer_binw_binx_arm(A.data_ptr(), B.data_ptr(), 0, 0, M, K, N, bnn.BNN_ACT_RAW_I32, 32, Y.data_ptr(), arm,
                                    G.stream())
    for _ in range(2):
        call()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        call()
    b.record()
    torch.cuda.synchronize()
    us = a.elapsed_time(b) * 1e3 / reps
    del A, B, Y
    torch.cuda.empty_cache()
    return {"workload": f"C5 binary GEMM M={M} K={K} N={N} int32 out", "us": round(us, 1),
            "binary_tops": round(2.0 * M * K * N / us / 1e6, 1), "output_GBps": round(4.0 * M * N / 1e9 / (us * 1e-6), 1)}


def all_configs(args, bnn, workloads, G, torch) -> int:
    """bnn_forward on Configs 1-4 and 6-10 (Config 5 is --gemm-sweep): one JSON line each."""
    for kv in args.opt:
        key, val = kv.split("=")
        bnn.bnn_set_option(getattr(bnn, "BNN_OPT_" + key), int(val))
    only = [int(v) for v in args.only.split(",")] if args.only else None
    for cid in (1, 2, 3, 4, 6, 7, 8, 9, 10):
        if only and cid not in only:
            continue
        steps = 200 if cid == 1 else (10 if cid in (4, 9, 10) else 50)
        print(json.dumps(time_config(cid, steps, workloads, G, torch)), flush=True)
    return 0


def hidden_k_sweep(args, bnn, workloads, G, torch) -> int:
    """The Sign-layer kernel of the hidden layers (4096 frames, 2048 units) with the input width K swept: what a launch
    costs beyond its products shows as the time that does not shrink with K.  One JSON line per K."""
    M, N = 4096, 2048
    for K in (512, 1024, 2048, 4096, 8192):
        A = G.to_dev(workloads.random_words(0, 1, M, K // 32))
        B = G.to_dev(workloads.random_words(0, 2, N, K // 32))
        sc = torch.full((N,), 0.5, device=G.DEV)
        bi = torch.zeros(N, device=G.DEV)
        Y = G.word_tensor(M, N, 32)

        def call():
            bnn.bnn_layer_binw_binx(A.data_ptr(), B.data_ptr(), sc.data_ptr(), bi.data_ptr(), M, K, N, bnn.BNN_ACT_SIGN, 32,
                                    Y.data_ptr(), G.stream())
        for _ in range(5):
            call()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(200):
            call()
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / 200
        print(json.dumps({"workload": f"Sign layer M={M} K={K} N={N}, launched back to back", "us_per_launch": round(us, 2),
                          "tflops": round(2.0 * M * K * N / us / 1e6, 1),
                          "frac_of_fp4_mfma_peak": round(2.0 * M * K * N / us / 1e6 / PEAK_MFMA_FP4_TFLOPS, 3)}), flush=True)
    return 0


def streaming(args, bnn, workloads, G, torch) -> int:
    """Latency of one bnn_forward on a few frames at a time (the paper's on-device use): one JSON line per batch size."""
    for kv in args.opt:
        key, val = kv.split("=")
        bnn.bnn_set_option(getattr(bnn, "BNN_OPT_" + key), int(val))
    only = [int(v) for v in args.only.split(",")] if args.only else [3, 10]
    for cid in only:
        cfg = workloads.CONFIGS[cid]
        Ws, bs = workloads.make_net_params(cfg)
        model = G.GpuModel(Ws, bs, cfg.hidden_act, cfg.word_bits, real_weight_layers=cfg.real_weight_layers)
        for M in (1, 4, 16, 64):
            X = G.to_dev(workloads.make_frames(cfg, M))
            out = torch.empty((M, model.N_out), dtype=torch.float32, device=G.DEV)
            for _ in range(10):
                model.forward(X, out)
            torch.cuda.synchronize()
            steps = 500
            t0 = time.perf_counter()
            for _ in range(steps):
                model.forward(X, out)
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) * 1e6 / steps
            # the same pass waited for every time (what one caller sees from call to result), and as one captured graph
            # (its launches become one: the host's share of a pass drops from about 27 us to a few)
            t0 = time.perf_counter()
            for _ in range(200):
                model.forward(X, out)
                torch.cuda.synchronize()
            us_sync = (time.perf_counter() - t0) * 1e6 / 200
            us_graph = us_graph_sync = None
            try:
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    model.forward(X, out)
                torch.cuda.synchronize()
                eager = out.clone()
                out.fill_(float("nan"))
                for _ in range(10):
                    g.replay()
                torch.cuda.synchronize()
                assert torch.equal(out, eager), "a replayed pass gives the eager pass's result"
                t0 = time.perf_counter()
                for _ in range(steps):
                    g.replay()
                torch.cuda.synchronize()
                us_graph = (time.perf_counter() - t0) * 1e6 / steps
                t0 = time.perf_counter()
                for _ in range(200):
                    g.replay()
                    torch.cuda.synchronize()
                us_graph_sync = (time.perf_counter() - t0) * 1e6 / 200
                del g
            except Exception as e:
                print(f"bench.py: graph capture failed ({e})", file=sys.stderr)
                torch.cuda.synchronize()
            print(json.dumps({"workload": cfg.name.split(" M=")[0] + f" M={M} (streaming)", "batch_frames": M,
                              "latency_us": round(us, 1), "frames_per_s": round(M / (us * 1e-6), 1),
                              "latency_us_waited_for": round(us_sync, 1),
                              "latency_us_graph_replay": None if us_graph is None else round(us_graph, 1),
                              "latency_us_graph_replay_waited_for": None if us_graph_sync is None else round(us_graph_sync, 1),
                              "kernel_launches": model.n_layers + 1}), flush=True)
        del model, Ws, bs
        torch.cuda.empty_cache()
    return 0


def train_step(args, bnn, workloads, G, torch) -> int:
    """One minibatch of Alg. 1 + Alg. 2 (binary weights and activations, Config 3's layer sizes): forward with the
    pre-activations kept, backward, gradient-norm clipping, clipped update, re-binarisation.  One JSON line per
    minibatch size with the time of each phase."""
    import numpy as np
    for kv in args.opt:
        key, val = kv.split("=")
        bnn.bnn_set_option(getattr(bnn, "BNN_OPT_" + key), int(val))
    cfg = workloads.CONFIGS[3]
    Ws, rs = workloads.make_net_params(cfg)
    L, wb, st = len(Ws), 32, G.stream()
    dev = G.DEV
    f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device=dev)
    for M in (256, 4096):
        X = G.to_dev(workloads.make_frames(cfg, M))
        labels = G.to_dev(np.random.default_rng(0).integers(0, cfg.dims[-1], M).astype(np.int32))
        W = [G.to_dev(w) for w in Ws]
        r = [G.to_dev(b) for b in rs]
        Wp = [G.word_tensor(w.shape[0], w.shape[1], wb) for w in Ws]
        WpT = [G.word_tensor(w.shape[1], w.shape[0], wb) for w in Ws]
        hhat = [f32(M, w.shape[0]) for w in Ws]
        bits = [G.word_tensor(M, w.shape[0], wb) for w in Ws[:-1]]
        hbT = [None] + [G.word_tensor(w.shape[1], M, wb) for w in Ws[1:]]
        gbuf = [f32(M, w.shape[0]) for w in Ws]
        gin = [f32(M, w.shape[1]) for w in Ws]
        gt = [f32(w.shape[0], M) for w in Ws]
        ht = [f32(w.shape[1], M) for w in Ws]
        gw = [f32(*w.shape) for w in Ws]
        gr = [f32(w.shape[0]) for w in Ws]
        ws = torch.empty(4096, dtype=torch.uint8, device=dev)
        norm = f32(1)
        P = G.ptr

        def binarise():
            for l in range(L):
                N, K = Ws[l].shape
                bnn.bnn_pack_weights(P(W[l]), N, K, wb, P(Wp[l]), 0, st)
                bnn.bnn_pack_weights_transposed(P(W[l]), N, K, wb, P(WpT[l]), st)

        def forward():
            for l in range(L):
                N, K = Ws[l].shape
                src = X if l == 0 else bits[l - 1]
                fn = bnn.bnn_layer_binw_realx if l == 0 else bnn.bnn_layer_binw_binx
                act = bnn.BNN_ACT_LINEAR if l < L - 1 else bnn.BNN_ACT_LOGSOFTMAX
                fn(P(src), P(Wp[l]), 0, P(r[l]), M, K, N, act, wb, P(hhat[l]), st)
                if l < L - 1:
                    bnn.bnn_pack_activations(P(hhat[l]), M, N, wb, P(bits[l]), st)

        # the two backward products with binary operands, in the oracle's order (fp32, ascending index) or on the int8
        # matrix cores (bnn_layer_binw_realx_i8: closer to the exact sum, not the same bits)
        i8_bytes = max(max(bnn.bnn_layer_binw_realx_i8_workspace_bytes(w.shape[0], M, w.shape[1]),
                           bnn.bnn_layer_binw_realx_i8_workspace_bytes(M, w.shape[0], w.shape[1])) for w in Ws)
        i8_ws = torch.empty(i8_bytes, dtype=torch.uint8, device=dev)
        fast = [False]

        def weight_grad_binh(l, N, K):
            if fast[0]:
                bnn.bnn_layer_binw_realx_i8(P(gt[l]), P(hbT[l]), 0, 0, N, M, K, wb, P(gw[l]), P(i8_ws), i8_bytes, st)
            else:
                bnn.bnn_backward_weight_binh(P(gt[l]), P(hbT[l]), N, K, M, wb, P(gw[l]), st)

        def input_grad_binw(l, N, K):
            if fast[0]:
                bnn.bnn_layer_binw_realx_i8(P(gbuf[l]), P(WpT[l]), 0, 0, M, N, K, wb, P(gbuf[l - 1]), P(i8_ws), i8_bytes, st)
            else:
                bnn.bnn_backward_input_binw(P(gbuf[l]), P(WpT[l]), M, N, K, wb, P(gbuf[l - 1]), st)

        def backward():
            bnn.bnn_softmax_xent_grad(P(hhat[-1]), P(labels), M, cfg.dims[-1], P(gbuf[-1]), st)
            for l in range(L - 1, -1, -1):
                N, K = Ws[l].shape
                g = gbuf[l]
                if l < L - 1:
                    bnn.bnn_mask_grad(P(g), P(hhat[l]), M * N, 1.0, P(g), st)
                bnn.bnn_transpose_f32(P(g), M, N, P(gt[l]), st)
                if l == 0:          # real input frames
                    bnn.bnn_transpose_f32(P(X), M, K, P(ht[l]), st)
                    bnn.bnn_backward_weight(P(gt[l]), P(ht[l]), N, K, M, P(gw[l]), st)
                else:               # the input is Sign(hhat of the layer below): its transposed bits, add/subtract
                    bnn.bnn_pack_weights_transposed(P(hhat[l - 1]), M, K, wb, P(hbT[l]), st)
                    weight_grad_binh(l, N, K)
                bnn.bnn_bias_grad(P(g), M, N, P(gr[l]), st)
                if l > 0:
                    input_grad_binw(l, N, K)

        def update():
            for l in range(L):
                N, K = Ws[l].shape
                bnn.bnn_grad_norm_clip(P(gw[l]), N * K, 15.0, P(ws), P(norm), st)
                bnn.bnn_update_clip(P(W[l]), P(gw[l]), N * K, 1e-3, 1, st)
                bnn.bnn_update_clip(P(r[l]), P(gr[l]), N, 1e-3, 0, st)

        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / reps

        binarise()
        reps = 20 if M <= 256 else 5
        ms = {"binarise": timed(binarise, reps), "forward": timed(forward, reps), "backward": timed(backward, reps),
              "update": timed(update, reps)}
        fast[0] = True
        backward_i8 = timed(backward, reps)
        fast[0] = False
        total = sum(ms.values())
        flops = 3 * 2.0 * cfg.macs_per_frame() * M - 2.0 * cfg.dims[0] * cfg.dims[1] * M   # forward + two backward products
        print(json.dumps({"workload": f"training step, {cfg.name.split(' M=')[0]}, minibatch {M}", "batch_frames": M,
                          "ms_per_step": round(total, 3), "frames_per_s": round(M / (total * 1e-3), 1),
                          "phase_ms": {k: round(v, 3) for k, v in ms.items()},
                          "tflops_products": round(flops / (total * 1e-3) / 1e12, 1),
                          "backward_ms_int8_products": round(backward_i8, 3),
                          "ms_per_step_int8_products": round(total - ms["backward"] + backward_i8, 3)}), flush=True)
        del X, labels, W, r, Wp, WpT, hhat, bits, hbT, gbuf, gin, gt, ht, gw, gr, i8_ws
        torch.cuda.empty_cache()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--arm", choices=["mfma", "mfma_i8", "valu"], default="mfma",
                    help="arm of the binary product: 4-bit-float MFMA (default), int8 MFMA, or XOR/popcount on the vector ALU")
    ap.add_argument("--cpu-sample-frames", type=int, default=4096)
    ap.add_argument("--streams", type=int, default=4,
                    help="steps in flight: the K timed steps go round-robin to this many HIP streams, each with its own "
                         "batch, output and workspace (1 = one step after the other)")
    ap.add_argument("--no-graphs", action="store_true",
                    help="steps in flight: launch every kernel from the host instead of replaying one captured forward pass per stream")
    ap.add_argument("--no-cooperative", action="store_true",
                    help="leave BNN_OPT_COOPERATIVE off: the output layer then runs as product kernel + row kernel")
    ap.add_argument("--no-configs", action="store_true",
                    help="leave the short runs of the other configurations (the line's \"configs\" array) out")
    ap.add_argument("--copy-calibration", action="store_true", help="run 10 plain 256 MiB device copies (counter calibration)")
    ap.add_argument("--only", default="", help="with --all-configs: comma-separated configuration numbers to run")
    ap.add_argument("--train-step", action="store_true",
                    help="one minibatch of forward + backward + update (Alg. 1 and 2) at Config 3's sizes")
    ap.add_argument("--streaming", action="store_true",
                    help="latency of bnn_forward on 1, 4, 16 and 64 frames (Configs 3 and 10, or --only)")
    ap.add_argument("--all-configs", action="store_true",
                    help="time bnn_forward on Configs 1-4 instead (one JSON line each; the default run is Config 3 only)")
    ap.add_argument("--hidden-k-sweep", action="store_true",
                    help="time the hidden layers' Sign kernel at input widths 512 .. 8192 (fixed cost of a launch)")
    ap.add_argument("--gemm-sweep", action="store_true", help="time the isolated binary GEMM sweep (Config 5) instead")
    ap.add_argument("--opt", action="append", default=[], help="kernel option as KEY=VALUE with KEY a BNN_OPT_* name, e.g. MFMA_LDS=0")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (frames are independent; a multi-GPU run would just split "
              "the batch with no communication). Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_1706_09453_amd as bnn
    import workloads
    import harness as G

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.gemm_sweep:
        return gemm_sweep(args, bnn, workloads, G, torch)
    if args.hidden_k_sweep:
        return hidden_k_sweep(args, bnn, workloads, G, torch)
    if args.all_configs:
        return all_configs(args, bnn, workloads, G, torch)
    if args.streaming:
        return streaming(args, bnn, workloads, G, torch)
    if args.train_step:
        return train_step(args, bnn, workloads, G, torch)
    if args.copy_calibration:
        # A plain device-to-device copy of known size: the reference the FETCH_SIZE / WRITE_SIZE counters are scaled by.
        nbytes = 256 << 20
        src = torch.empty(nbytes, dtype=torch.uint8, device=G.DEV).fill_(7)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": nbytes, "copies": 10}))
        return 0
    cfg = workloads.CONFIGS[3]
    M = cfg.M
    Ws, bs = workloads.make_net_params(cfg)
    X_host = workloads.make_frames(cfg)
    model = G.GpuModel(Ws, bs, cfg.hidden_act, cfg.word_bits)
    X = G.to_dev(X_host)
    out = torch.empty((M, model.N_out), dtype=torch.float32, device=G.DEV)
    arm = {"mfma": bnn.BNN_ARM_MFMA, "mfma_i8": bnn.BNN_ARM_MFMA_I8, "valu": bnn.BNN_ARM_VALU_XOR}[args.arm]
    bnn.bnn_set_option(bnn.BNN_OPT_BINX_ARM, arm)
    # This process runs one stream and nothing else on the GPU, which is what BNN_OPT_COOPERATIVE asks of its caller: the
    # output layer then finishes its log-Softmax inside the product kernel.
    cooperative = not args.no_cooperative
    bnn.bnn_set_option(bnn.BNN_OPT_COOPERATIVE, 1 if cooperative else 0)
    for kv in args.opt:
        key, val = kv.split("=")
        bnn.bnn_set_option(getattr(bnn, "BNN_OPT_" + key), int(val))

    # ---- whole forward pass: W warm-up steps, then exactly K timed steps
    for _ in range(args.warmup):
        model.forward(X, out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        model.forward(X, out)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    dev_ms = e0.elapsed_time(e1)
    single_ms_per_step = wall_ms / args.steps
    ms_per_step = single_ms_per_step
    frames_per_s = M / (ms_per_step * 1e-3)

    # ---- the same K steps with several of them in flight: S streams, each with its own batch of 4096 frames, its own
    #      output and workspace (what a server with batches queued up does).  A hidden-layer launch gives every SIMD one
    #      wave; a second launch beside it fills the matrix cores' idle slots and the gaps between dependent launches.
    #      Kernels that wait for each other need the device to themselves, so BNN_OPT_COOPERATIVE is off here.
    S = max(1, args.streams)
    pipelined = None
    if S > 1:
        bnn.bnn_set_option(bnn.BNN_OPT_COOPERATIVE, 0)
        nbytes = bnn.bnn_forward_workspace_bytes(model.layers, model.n_layers, M)
        Xs = [X] + [X.clone() for _ in range(S - 1)]
        outs = [torch.empty_like(out) for _ in range(S)]
        wss = [torch.empty(max(nbytes, 256), dtype=torch.uint8, device=G.DEV) for _ in range(S)]
        torch.cuda.synchronize()
        streams = None

        def step(i):
            j = i % S
            bnn.bnn_forward(model.layers, model.n_layers, Xs[j].data_ptr(), M, outs[j].data_ptr(), wss[j].data_ptr(), nbytes,
                            streams[j].cuda_stream)
        # Streams share the process's few hardware queues, and which streams end up on one queue (and then run one
        # after the other) depends on the order the runtime created them in: as part of the warm-up, a few sets of S
        # streams out of 2 S + 1 candidates run 40 untimed steps each, and the fastest set takes the timed steps.
        pool = [torch.cuda.current_stream()] + [torch.cuda.Stream() for _ in range(2 * S)]
        best = None
        for first in range(0, S + 2):
            streams = pool[first:first + S]
            for i in range(2 * S):
                step(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(40):
                step(i)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            if best is None or dt < best[0]:
                best = (dt, first)
        streams = pool[best[1]:best[1] + S]
        # One captured forward pass per stream (its 8 launches become one graph launch): the host then needs 10 us per
        # step instead of 35, so all S streams have work a few tens of microseconds after the timed region starts.  In
        # the steady state the graph is no faster than the launches themselves; on K = 20 steps it is 5 % of the time.
        graphs = None
        if not args.no_graphs:
            try:
                graphs = []
                for j in range(S):
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=streams[j]):
                        step(j)
                    graphs.append(g)
                torch.cuda.synchronize()
            except Exception as e:   # capture refused: launch the kernels one by one, as before
                print(f"bench.py: graph capture failed ({e}); launching eagerly", file=sys.stderr)
                graphs = None
                torch.cuda.synchronize()

        def timed_step(i):
            if graphs is None:
                step(i)
            else:
                with torch.cuda.stream(streams[i % S]):
                    graphs[i % S].replay()
        for o in outs:
            o.fill_(float("nan"))   # what the checks below see is what the timed steps wrote
        for i in range(max(args.warmup, S)):
            timed_step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            timed_step(i)
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
        frames_per_s = M / (ms_per_step * 1e-3)
        scale_out = float(out.abs().max())
        pipelined = {"streams": S, "graph_replays": graphs is not None, "stream_set": f"candidates {best[1]}..{best[1] + S - 1} of {len(pool)} (fastest of {S + 2} sets in the warm-up)",
                     "ms_per_step": round(ms_per_step, 5), "frames_per_s": round(frames_per_s, 1),
                     "outputs_identical_across_streams": all(torch.equal(outs[0], o) for o in outs[1:]),
                     "max_abs_diff_to_single_stream": float((outs[0] - out).abs().max()), "output_scale": scale_out}
        del Xs, wss, graphs
        bnn.bnn_set_option(bnn.BNN_OPT_COOPERATIVE, 1 if cooperative else 0)

    macs_all = cfg.macs_per_frame() * M
    macs_bin = cfg.binbin_macs_per_frame() * M

    # ---- per-layer kernels, same launch configuration, timed one layer at a time with HIP events
    acts = [X]
    ws_bits = [torch.empty((M, bnn.bnn_packed_words(d["N"], cfg.word_bits)), dtype=torch.int32, device=G.DEV)
               for d in model.descs[:-1]]
    layer_us = []
    reps = 200   # (its own loops of back-to-back launches, whatever --steps is: 20 launches after an idle device read 10 % long)
    # layer 1 exactly as bnn_forward runs it: a one-layer network (real input -> Sign bits)
    first = bnn.make_layer_array(model.descs[:1])
    first_ws_bytes = bnn.bnn_forward_workspace_bytes(first, 1, M)
    first_ws = torch.empty(max(first_ws_bytes, 256), dtype=torch.uint8, device=G.DEV)
    for l, d in enumerate(model.descs):
        src = X if l == 0 else ws_bits[l - 1]
        dst = out if l == model.n_layers - 1 else ws_bits[l]
        fn = bnn.bnn_layer_binw_binx if d["x_is_binary"] else bnn.bnn_layer_binw_realx

        def call():
            if l == 0:
                bnn.bnn_forward(first, 1, src.data_ptr(), M, dst.data_ptr(), first_ws.data_ptr(), first_ws_bytes,
                                G.stream())
            else:
                fn(src.data_ptr(), d["Wp"], d["scale"], d["bias"], M, d["K"], d["N"], d["act"], d["word_bits"],
                   dst.data_ptr(), G.stream())
        for _ in range(3):
            call()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            call()
        b.record()
        torch.cuda.synchronize()
        layer_us.append(a.elapsed_time(b) * 1e3 / reps)

    # ---- the hidden layers' kernel with four launches in flight (four streams, own output each, same operands): what the
    #      kernel sustains when a second workgroup shares each CU, as in the pipelined steps above
    in_flight = None
    if S > 1 and model.n_layers > 2:
        d = model.descs[1]
        st4 = streams
        dst4 = [torch.empty_like(ws_bits[1]) for _ in range(S)]
        torch.cuda.synchronize()

        def call4(i):
            bnn.bnn_layer_binw_binx(ws_bits[0].data_ptr(), d["Wp"], d["scale"], d["bias"], M, d["K"], d["N"], d["act"],
                                    d["word_bits"], dst4[i % S].data_ptr(), st4[i % S].cuda_stream)
        for i in range(8 * S):
            call4(i)
        torch.cuda.synchronize()
        n4 = 100 * S
        t0 = time.perf_counter()
        for i in range(n4):
            call4(i)
        torch.cuda.synchronize()
        us4 = (time.perf_counter() - t0) * 1e6 / n4
        tf4 = 2.0 * M * d["K"] * d["N"] / (us4 * 1e-6) / 1e12
        in_flight = {"streams": S, "avg_launch_us": round(us4, 2), "achieved": round(tf4, 1),
                     "identical_outputs": all(torch.equal(dst4[0], o) for o in dst4[1:]) and torch.equal(dst4[0], ws_bits[1])}

    # kernel groups: layer 1 (real input), hidden binary layers (one kernel, launched 5x per step), output layer
    hidden_us = layer_us[1:-1]
    groups = {
        "realx layer 1 (quantize + int8 MFMA filter + exact resolution)": (layer_us[0], 1, 2.0 * M * cfg.dims[0] * cfg.dims[1]),
        "binx hidden kernel (2048x2048, sign+repack)": (sum(hidden_us), len(hidden_us),
                                                        2.0 * M * cfg.dims[1] * cfg.dims[2]),
        "binx output kernel + log-softmax": (layer_us[-1], 1, 2.0 * M * cfg.dims[-2] * cfg.dims[-1]),
    }
    dominant = max(groups, key=lambda k: groups[k][0])
    tot_us, launches, flops_per_launch = groups[dominant]
    avg_us = tot_us / launches
    achieved_tflops = flops_per_launch / (avg_us * 1e-6) / 1e12
    if dominant.startswith("realx"):
        bound, peak = "mfma", PEAK_MFMA_INT8_TOPS / 3.0   # three int8 digit products per fp32 multiply-add
    elif args.arm == "mfma":
        bound, peak = "mfma", PEAK_MFMA_FP4_TFLOPS
    elif args.arm == "mfma_i8":
        bound, peak = "mfma", PEAK_MFMA_INT8_TOPS
    else:
        bound, peak = "alu", PEAK_XOR_POPC_TOPS
    # HBM bytes per launch of each kernel group from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by a plain copy
    # (profiles/forward_c3_hbm_traffic.txt); measured for this workload with the matrix-core arm only
    measured_traffic = {"realx": (8.19 + 1.00) * 2 ** 20, "binx hidden": (5.35 + 1.00) * 2 ** 20,
                        "binx output": (8.09 + 26.81 + 27.27 + 53.13) * 2 ** 20}   # (output layer: the two-kernel path)
    traffic = None
    if args.arm == "mfma" and not args.opt:
        traffic = next(int(v) for k, v in measured_traffic.items() if dominant.startswith(k))
    bin_us = sum(layer_us[1:])
    binbin_tops = 2.0 * macs_bin / (bin_us * 1e-6) / 1e12
    roofline = {"bound": bound, "achieved": round(achieved_tflops, 3), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved_tflops / peak, 4), "traffic": traffic,
                "traffic_source": None if traffic is None else
                "stored, not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE per dispatch, scaled by a "
                "plain copy of known size (profiles/forward_c3_hbm_traffic.txt)",
                "kernel": dominant, "avg_launch_us": round(avg_us, 2), "launches_per_step": launches,
                # every binary x binary layer of the step (5 hidden + the output layer with its log-softmax), products
                # over the sum of their launch times, against the same matrix-core peak
                "frac_all_binbin": round(binbin_tops / peak, 4) if bound == "mfma" and not dominant.startswith("realx") else None}
    if in_flight and dominant.startswith("binx hidden") and bound == "mfma":
        # the same kernel, same shape, with launches in flight on several streams (host clock over 100 launches per stream)
        in_flight["frac"] = round(in_flight["achieved"] / peak, 4)
        roofline["launches_in_flight"] = in_flight

    result = {
        "metric": "frames/sec, 6x2048 binarized DNN (binary weights and activations), batch 4096, 1xMI355X",
        "value": round(frames_per_s, 1), "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"mfma": "b1 (+-1 as fp4-e2m1 MFMA operands, exact fp32 accumulate) + f32",
                  "mfma_i8": "b1 (+-1 as int8 MFMA operands, int32 accumulate) + f32",
                  "valu": "b1 (xor+popcount u32) + f32"}[args.arm],
        "data": "synthetic",
        "config": {"workload": cfg.name, "dims": list(cfg.dims), "batch_frames": M, "word_bits": cfg.word_bits,
                   "binx_arm": args.arm, "steps_in_flight": S,
                   "options": {"BNN_OPT_COOPERATIVE": 0 if S > 1 else int(cooperative)}},
        # one step after the other on one stream (with the cooperative output layer unless --no-cooperative)
        "single_stream": {"ms_per_step": round(single_ms_per_step, 5), "frames_per_s": round(M / (single_ms_per_step * 1e-3), 1),
                          "options": {"BNN_OPT_COOPERATIVE": int(cooperative)}},
        "device_ms_per_step_single_stream": round(dev_ms / args.steps, 5),
        "binary_tops_all_layers": round(2.0 * macs_all / (ms_per_step * 1e-3) / 1e12, 2),
        "binary_tops_binbin_kernels": round(binbin_tops, 2),
        "layer_us": [round(v, 2) for v in layer_us],
        "roofline": roofline,
    }

    # ---- the CPU oracle on the host cores, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        S = min(args.cpu_sample_frames, M)
        layers = orc.make_layers(Ws, bs, cfg.hidden_act, cfg.word_bits)
        orc.forward(layers, X_host[:8], form="xor")                       # warm-up (loads the library)
        t0 = time.perf_counter()
        ref = orc.forward(layers, X_host[:S], form="xor")
        dt = time.perf_counter() - t0
        import ctypes
        gomp = ctypes.CDLL("libgomp.so.1")                                # the OpenMP runtime the oracle's library uses
        cores = int(gomp.omp_get_max_threads())
        # the same oracle on ONE thread, on a sample sized for a few seconds
        S1 = max(32, min(S, S // max(cores, 1)))
        gomp.omp_set_num_threads(1)
        t1 = time.perf_counter()
        orc.forward(layers, X_host[:S1], form="xor")
        dt1 = time.perf_counter() - t1
        gomp.omp_set_num_threads(cores)
        got = out[:S].cpu().numpy()
        err = float(np.max(np.abs(got.astype(np.float64) - ref)))
        result["cpu_baseline"] = {"value": round(S / dt, 1), "unit": "frames/s", "cores": cores, "kind": "oracle",
                                  "sample": f"first {S} of the {M} frames, all 7 layers, XOR/popcount form, "
                                            f"{dt:.2f} s wall",
                                  "single_thread": {"value": round(S1 / dt1, 1), "unit": "frames/s", "cores": 1,
                                                    "sample": f"first {S1} frames, {dt1:.2f} s wall"},
                                  "gpu_vs_oracle_max_abs_err": err,
                                  "oracle_output_scale": float(np.max(np.abs(ref)))}
    # ---- the other configurations, a short run each (their parity is the tests' business; these are timings only)
    if not args.no_configs and args.arm == "mfma" and not args.opt:
        del model, X, out, ws_bits, first_ws
        torch.cuda.empty_cache()
        lines = [time_config(1, 100, workloads, G, torch), time_config(2, 20, workloads, G, torch),
                 {"workload": cfg.name, "batch_frames": M, "steps": args.steps, "ms_per_step": round(single_ms_per_step, 4),
                  "frames_per_s": round(M / (single_ms_per_step * 1e-3), 1),
                  "tops_all_layers": round(2.0 * macs_all / (single_ms_per_step * 1e-3) / 1e12, 2),
                  "binbin_share_of_macs": round(macs_bin / macs_all, 3)},
                 time_config(4, 10, workloads, G, torch)]
        corners = [workloads.GEMM_SWEEP[0], workloads.GEMM_SWEEP[-1]]
        lines += [time_gemm(sh, bnn.BNN_ARM_MFMA, 10 if sh.M * sh.K * sh.N < 1e12 else 3, bnn, workloads, G, torch)
                  for sh in corners]
        result["configs"] = lines          # every entry: one step after the other on one stream
    if pipelined:
        result["pipelined"] = pipelined
    if cooperative:
        result["cooperative_timeouts"] = bnn.bnn_cooperative_timeouts()
    print(json.dumps(result))
    if result.get("cooperative_timeouts"):
        print("bench.py: a cooperative kernel's bounded wait ran out", file=sys.stderr)
        return 1
    if pipelined and not (pipelined["outputs_identical_across_streams"] and
                          pipelined["max_abs_diff_to_single_stream"] <= 1e-4 * pipelined["output_scale"]):
        print("bench.py: the steps in flight on several streams disagree with each other or with the single-stream pass",
              file=sys.stderr)
        return 1
    cb = result.get("cpu_baseline")
    if cb and not cb["gpu_vs_oracle_max_abs_err"] <= 1e-4 * cb["oracle_output_scale"]:
        print("bench.py: the timed output disagrees with the oracle beyond 1e-4 of the output scale", file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
