#!/usr/bin/env python3
"""Benchmark of the W4A8 quantized linear hot path on one MI355X.

Workload (default): the Qwen2-7B-shaped configuration - 28 blocks of
q|k|v 3584->4608, o 3584->3584, gate|up 3584->37888, down 18944->3584 plus the
lm_head 3584->152064 - as one decode step (batch 1) and one prefill pass
(M = 1024 tokens, 28 blocks).  One "step" = activation quantization + linear
for every projection of the decode pass, then of the prefill pass.  Inputs are
synthetic and resident in HBM before the timed region; every block has its own
packed buffer (3.8 GB in total, far beyond the 256 MB Infinity Cache), so the
decode pass streams weights from HBM.

Prints ONE JSON line.  `value` is the decode GEMV rate in GB/s of algorithmic
bytes; the prefill rate in int8 TOPS is in `prefill_value`.
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

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published (5.0 POP/s)
G = 64
# HBM traffic per launch (bytes, mean over a pass) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this file, scaled by a copy kernel of known size; see profiles/ for the runs.  None = not measured
# for the current kernels.
PREFILL_TRAFFIC_BYTES = 171.1e6   # profiles/bench_qwen2-7b_hbm_traffic.txt
DECODE_TRAFFIC_BYTES = 33.9e6     # same file


GROUP_PARAM_BYTES = 5    # fp32 scale + 1-byte zero point; 8 with an fp32 group minimum (--weight-mode minfloat);
                         # 16 for int8 weights (two 4-bit planes, each with step and minimum)
CODE_BYTES_X2 = 1        # bytes of codes per two weights: 1 for int4, 2 for int8


def decode_bytes(N, K):
    """Algorithmic bytes of one decode GEMV: codes + per-group parameters, the int8
    activation row, and the fp32 output."""
    return CODE_BYTES_X2 * N * K // 2 + GROUP_PARAM_BYTES * N * (K // G) + K + 4 * N


def prefill_ops(M, N, K):
    return 2 * M * N * K


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--model", default="qwen2-7b", choices=["qwen2-1.5b", "qwen2-7b", "llama3-8b"])
    ap.add_argument("--phase", default="both", choices=["both", "decode", "prefill"])
    ap.add_argument("--lm-head-prefill", action="store_true",
                    help="also time the LM head through the prefill GEMM at the prefill batch (per_layer.prefill_lm_head)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 512 MiB device copy, as the known-size reference for rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--weight-mode", default="zp", choices=["zp", "minfloat", "int8"],
                    help="weight quantizer: int4 with an integer zero point (the benchmark configuration), int4 "
                         "as Eq. 1 is printed (float group minimum), or int8 weights (float group minimum)")
    ap.add_argument("--act16", action="store_true",
                    help="also time the fp16-activation entry points (W4A16 / W8A16) per layer: per_layer "
                         "gains decode16_* (GB/s of their algorithmic bytes) and prefill16_* (TFLOP/s)")
    ap.add_argument("--separate-projections", action="store_true",
                    help="run q, k, v and gate, up as launches of their own instead of concatenated along N")
    ap.add_argument("--warm", action="store_true",
                    help="also time the decode GEMV of each layer on ONE packed buffer over and over (weights stay "
                         "in the Infinity Cache): per_layer decode_*_warm, a cache-resident figure, not HBM")
    ap.add_argument("--peaks", action="store_true",
                    help="also measure what this GPU sustains (streaming read, matrix instructions with and "
                         "without the epilogue's vector work) and report it as `achievable`")
    ap.add_argument("--out16", action="store_true",
                    help="also time the prefill call with binary16 output per layer (per_layer prefill_o16_*)")
    ap.add_argument("--two-call-decode", action="store_true",
                    help="decode pass calls mnnq_quant_act + mnnq_linear_decode per layer instead of "
                         "mnnq_linear_decode_fused (fp32 row in, quantizer inside the call)")
    args = ap.parse_args()
    args.fused_decode = not args.two_call_decode
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; the path would shard by output rows "
              "but no multi-GPU figure is produced.  Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2506_10443_amd import binding as B, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B.lib()  # fail loudly if the HIP library is not built
    wmode = {"zp": B.MODE_W4_ZP_INT, "minfloat": B.MODE_W4_MIN_FLOAT, "int8": B.MODE_W8_MIN_FLOAT}[args.weight_mode]
    global GROUP_PARAM_BYTES, CODE_BYTES_X2
    GROUP_PARAM_BYTES = {"zp": 5, "minfloat": 8, "int8": 16}[args.weight_mode]
    CODE_BYTES_X2 = 2 if args.weight_mode == "int8" else 1

    spec = synth.MODELS[args.model]
    n_blocks = spec["blocks"]
    M_pre = spec["prefill_m"]
    layers = synth.block_layers(args.model, fused=not args.separate_projections)   # q|k|v and gate|up share their input

    # ---- weights: one block drawn on the host (seeded), packed into n_blocks distinct buffers
    t0 = time.time()
    packed = {name: [] for name, _, _ in layers}
    pack_bytes_in = 0
    pack_ms = 0.0
    for name, N, K in layers:
        parts = [synth.weights(*spec["layers"][p], synth.layer_seed(args.model, 0, p))
                 for p in synth.fused_parts(name)]
        W = torch.from_numpy(np.concatenate(parts) if len(parts) > 1 else parts[0]).to(dev)
        del parts
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n_blocks):
            packed[name].append(B.mnnq_pack_weights(W, mode=wmode))
        e1.record()
        torch.cuda.synchronize()
        pack_ms += e0.elapsed_time(e1)
        pack_bytes_in += n_blocks * N * K * 4
        del W
    lm = None
    if spec["lm_head"] is not None:
        N, K = spec["lm_head"]
        W = torch.from_numpy(synth.weights(N, K, synth.layer_seed(args.model, 0, "lm_head"))).to(dev)
        lm = (B.mnnq_pack_weights(W, mode=wmode), N, K)
        del W
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    # ---- activations (fp32, resident) and static outputs
    def act(M, K, seed):
        return torch.from_numpy(synth.activations(M, K, seed, outliers=True)).to(dev)

    io_dec, io_pre = {}, {}
    for i, (name, N, K) in enumerate(layers):
        for M, io in ((1, io_dec), (M_pre, io_pre)):
            x = act(M, K, 9000 + 10 * i + (0 if M == 1 else 1))
            xq = torch.empty((M, K), dtype=torch.int8, device=dev)
            sx = torch.empty((M,), dtype=torch.float32, device=dev)
            y = torch.empty((M, N), dtype=torch.float32, device=dev)
            io[name] = (x, xq, sx, y)
    if lm is not None:
        x = act(1, lm[2], 9990)
        io_dec["lm_head"] = (x, torch.empty((1, lm[2]), dtype=torch.int8, device=dev),
                             torch.empty((1,), dtype=torch.float32, device=dev),
                             torch.empty((1, lm[1]), dtype=torch.float32, device=dev))

    # scratch of the fused decode call (quantized row + scale), shared by all layers of the pass
    ws_dec = torch.empty(max(B.mnnq_workspace_size(1, N, K) for _, N, K in
                             layers + ([("lm_head", lm[1], lm[2])] if lm else [])),
                         dtype=torch.uint8, device=dev)

    def decode_layer(p, N, K, io, fused=None):
        x, xq, sx, y = io
        if args.fused_decode if fused is None else fused:
            B.mnnq_linear_decode_fused(p, N, K, x, out=y, workspace=ws_dec, mode=wmode)
        else:
            B.mnnq_quant_act(x, want_xsum=False, out=(xq, sx, None))
            B.mnnq_linear_decode(p, N, K, xq, sx, out=y, mode=wmode)

    def decode_pass(fused=None):
        for b in range(n_blocks):
            for name, N, K in layers:
                decode_layer(packed[name][b], N, K, io_dec[name], fused)
        if lm is not None:
            decode_layer(lm[0], lm[1], lm[2], io_dec["lm_head"], fused)

    def prefill_pass():
        for b in range(n_blocks):
            for name, N, K in layers:
                x, xq, sx, y = io_pre[name]
                B.mnnq_quant_act(x, want_xsum=False, out=(xq, sx, None))
                B.mnnq_linear_prefill(packed[name][b], N, K, xq, sx, out=y, mode=wmode)

    do_dec = args.phase in ("both", "decode")
    do_pre = args.phase in ("both", "prefill")

    # ---- HIP graphs of the two passes (no memset nodes are recorded: the library issues kernels only)
    graphs = {}
    if not args.no_graph:
        side = torch.cuda.Stream()
        for key, fn, on in (("decode", decode_pass, do_dec), ("prefill", prefill_pass, do_pre)):
            if not on:
                continue
            with torch.cuda.stream(side):
                fn()                       # eager run first (also warms the code objects)
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                fn()
            graphs[key] = g
    run_dec = graphs["decode"].replay if "decode" in graphs else decode_pass
    run_pre = graphs["prefill"].replay if "prefill" in graphs else prefill_pass

    def step(evs=None):
        if evs is not None:
            evs[0].record()
        if do_dec:
            run_dec()
        if evs is not None:
            evs[1].record()
        if do_pre:
            run_pre()
        if evs is not None:
            evs[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_start) * 1e3
    dec_ms = [e[0].elapsed_time(e[1]) for e in events]
    pre_ms = [e[1].elapsed_time(e[2]) for e in events]
    ms_per_step = wall_ms / args.steps

    # ---- algorithmic work of one pass
    dec_bytes = n_blocks * sum(decode_bytes(N, K) for _, N, K in layers)
    if lm is not None:
        dec_bytes += decode_bytes(lm[1], lm[2])
    pre_ops = n_blocks * sum(prefill_ops(M_pre, N, K) for _, N, K in layers)
    dec_mean = float(np.mean(dec_ms)) if do_dec else None
    pre_mean = float(np.mean(pre_ms)) if do_pre else None
    dec_gbs = dec_bytes / (dec_mean * 1e-3) / 1e9 if do_dec else None
    pre_tops = pre_ops / (pre_mean * 1e-3) / 1e12 if do_pre else None

    # ---- per-kernel timing: HIP events on the launch stream around a back-to-back run of
    #      launches of ONE kernel, cycling through the per-block buffers so that weights
    #      come from HBM.  The small gaps between launches are included (conservative).
    def time_launches(fn_list, reps):
        # replayed as a HIP graph so that the host's launch rate does not limit short kernels
        side2 = torch.cuda.Stream()
        with torch.cuda.stream(side2):
            for fn in fn_list[:4]:
                fn()
        side2.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side2):
            for fn in fn_list:
                fn()
        g.replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            g.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / (reps * len(fn_list))  # mean ms per launch

    roof_pre = roof_dec = None
    per_layer = {}
    if do_pre:
        fns, ops = [], 0
        for name, N, K in layers:
            x, xq, sx, y = io_pre[name]
            lay = [(lambda p=packed[name][b], N=N, K=K, xq=xq, sx=sx, y=y:
                    B.mnnq_linear_prefill(p, N, K, xq, sx, out=y, mode=wmode)) for b in range(n_blocks)]
            t = time_launches(lay, 2)
            per_layer["prefill_" + name] = {"us": round(t * 1e3, 2),
                                            "tops": round(prefill_ops(M_pre, N, K) / (t * 1e-3) / 1e12, 1)}
            fns += lay
            ops += n_blocks * prefill_ops(M_pre, N, K)
        t = time_launches(fns, 2)
        ach = ops / len(fns) / (t * 1e-3) / 1e12
        roof_pre = {"kernel": "prefill_kernel (W4A8 int8 MFMA GEMM), all %d launches of a pass" % len(fns),
                    "bound": "mfma", "achieved": round(ach, 1), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                    "frac": round(ach / INT8_PEAK_TOPS, 4), "traffic": PREFILL_TRAFFIC_BYTES if (args.model, args.weight_mode) == ("qwen2-7b", "zp") else None,
                    "algorithmic_ops_per_launch": ops // len(fns), "avg_launch_us": round(t * 1e3, 2)}
    if do_dec:
        fns, byt = [], 0
        for name, N, K in layers:
            x, xq, sx, y = io_dec[name]
            lay = [(lambda p=packed[name][b], N=N, K=K, xq=xq, sx=sx, y=y:
                    B.mnnq_linear_decode(p, N, K, xq, sx, out=y, mode=wmode)) for b in range(n_blocks)]
            t = time_launches(lay, 4)
            per_layer["decode_" + name] = {"us": round(t * 1e3, 2),
                                           "gbs": round(decode_bytes(N, K) / (t * 1e-3) / 1e9, 1)}
            fns += lay
            byt += n_blocks * decode_bytes(N, K)
            if args.warm:
                t = time_launches(lay[:1] * n_blocks, 4)
                per_layer["decode_" + name + "_warm"] = {"us": round(t * 1e3, 2), "cache_resident": True,
                                                         "gbs": round(decode_bytes(N, K) / (t * 1e-3) / 1e9, 1)}
        t = time_launches(fns, 4)
        ach = byt / len(fns) / (t * 1e-3) / 1e9
        roof_dec = {"kernel": "decode_kernel (W4A8 GEMV), all %d block launches of a pass" % len(fns),
                    "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": DECODE_TRAFFIC_BYTES if (args.model, args.weight_mode) == ("qwen2-7b", "zp") else None,
                    "algorithmic_bytes_per_launch": byt // len(fns), "avg_launch_us": round(t * 1e3, 2)}
        if lm is not None:
            x, xq, sx, y = io_dec["lm_head"]
            t = time_launches([lambda: B.mnnq_linear_decode(lm[0], lm[1], lm[2], xq, sx, out=y, mode=wmode)] * 4, 4)
            per_layer["decode_lm_head"] = {"us": round(t * 1e3, 2),
                                           "gbs": round(decode_bytes(lm[1], lm[2]) / (t * 1e-3) / 1e9, 1)}

    # ---- the LM head through the prefill GEMM (a shape stress: a real prefill needs only the last token's row;
    #      reported separately, not part of any pass)
    if args.lm_head_prefill and lm is not None and do_pre:
        xf = torch.from_numpy(synth.activations(M_pre, lm[2], 4242, outliers=True)).to(dev)
        xq_l, sx_l, _ = B.mnnq_quant_act(xf, want_xsum=False)
        y_l = torch.empty((M_pre, lm[1]), dtype=torch.float32, device=dev)
        t = time_launches([lambda: B.mnnq_linear_prefill(lm[0], lm[1], lm[2], xq_l, sx_l, out=y_l, mode=wmode)] * 2, 3)
        per_layer["prefill_lm_head"] = {"us": round(t * 1e3, 2),
                                        "tops": round(prefill_ops(M_pre, lm[1], lm[2]) / (t * 1e-3) / 1e12, 1)}
        del xf, xq_l, sx_l, y_l

    # ---- fp16 activations on the same packed weights (reported beside the target path, not part of `value`)
    if args.act16:
        for name, N, K in layers:
            if do_pre:
                x16 = io_pre[name][0].to(torch.float16)
                y = io_pre[name][3]
                lay = [(lambda p=packed[name][b], N=N, K=K, x16=x16, y=y:
                        B.mnnq_linear_prefill_f16(p, N, K, x16, out=y, mode=wmode)) for b in range(n_blocks)]
                t = time_launches(lay, 2)
                per_layer["prefill16_" + name] = {"us": round(t * 1e3, 2),
                                                  "tflops": round(prefill_ops(M_pre, N, K) / (t * 1e-3) / 1e12, 1)}
            if do_dec:
                x16 = io_dec[name][0].to(torch.float16)
                y = io_dec[name][3]
                lay = [(lambda p=packed[name][b], N=N, K=K, x16=x16, y=y:
                        B.mnnq_linear_decode_f16(p, N, K, x16[0], out=y[0], mode=wmode)) for b in range(n_blocks)]
                try:
                    t = time_launches(lay, 4)
                except B.MnnqError:      # the fp16 row of this layer does not fit the GEMV's LDS staging
                    per_layer["decode16_" + name] = None
                    continue
                per_layer["decode16_" + name] = {"us": round(t * 1e3, 2),
                                                 "gbs": round((decode_bytes(N, K) + K) / (t * 1e-3) / 1e9, 1)}

    if args.out16 and do_pre:
        for name, N, K in layers:
            x, xq, sx, y = io_pre[name]
            y16 = torch.empty((M_pre, N), dtype=torch.float16, device=dev)
            lay = [(lambda p=packed[name][b], N=N, K=K, xq=xq, sx=sx, y16=y16:
                    B.mnnq_linear_prefill_o16(p, N, K, xq, sx, out=y16, mode=wmode)) for b in range(n_blocks)]
            t = time_launches(lay, 2)
            per_layer["prefill_o16_" + name] = {"us": round(t * 1e3, 2),
                                                "tops": round(prefill_ops(M_pre, N, K) / (t * 1e-3) / 1e12, 1)}

    # ---- the same decode pass through the fused entry point (quantizer inside the GEMV), for comparison
    dec_other = None
    if do_dec and not args.no_graph:
        other_fused = not args.fused_decode
        side3 = torch.cuda.Stream()
        with torch.cuda.stream(side3):
            decode_pass(other_fused)
        side3.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side3):
            decode_pass(other_fused)
        g.replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            g.replay()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / 10
        dec_other = {"path": "fused" if other_fused else "two-call", "ms": round(ms, 4),
                     "gbs": round(dec_bytes / (ms * 1e-3) / 1e9, 1)}

    if args.calibrate_copy:
        src = torch.empty(128 * 1024 * 1024, dtype=torch.int32, device=dev).fill_(7)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- what the GPU sustains, measured with the library's register-only / streaming helper kernels
    achievable = None
    if args.peaks:
        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) * 1e-3 / reps
        sink = torch.zeros(4, dtype=torch.float32, device=dev)
        big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)       # 1 GiB: 4x the Infinity Cache
        t = timed(lambda: B.mnnq_peak_read(big, sink), 10)
        achievable = {"hbm_read_gbs": round(big.numel() / t / 1e9, 1)}
        del big
        cus = torch.cuda.get_device_properties(dev).multi_processor_count
        ops = {0: 2 * 16 * 16 * 64, 1: 2 * 16 * 16 * 32, 2: 2 * 16 * 16 * 128}
        for key, kind, epi in (("mfma_int8_tops", 0, 0), ("mfma_fp16_tflops", 1, 0), ("mfma_fp8_tflops", 2, 0),
                               ("mfma_int8_with_cvt_fma_tops", 0, 1), ("mfma_int8_with_cvt_fma_8int_tops", 0, 2)):
            best = 0.0
            for w in (2, 4):
                n = [0]
                t = timed(lambda: n.__setitem__(0, B.mnnq_peak_mfma(kind, epi, w, 2000, sink)), 3)
                best = max(best, cus * 4 * w * n[0] * ops[kind] / t / 1e12)
            achievable[key] = round(best, 1)

    # ---- CPU baseline: the oracle, as it stands, on the host cores, on a bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        cores = len(os.sched_getaffinity(0))
        oracle.set_threads(cores)
        name, N, K = max(layers, key=lambda l: l[1] * l[2])          # the largest projection of a block
        Nc = min(N, 4096)
        Wc = synth.weights(Nc, K, 4242)
        q, s, z = oracle.quant_weights(Wc)
        xs = synth.activations(16, K, 4243)
        xq_o, sx_o, _ = oracle.quant_act(xs)
        oracle.linear_w4a8(xq_o[:1], sx_o[:1], q, s, z, want_acc=False)   # warm
        t1 = time.perf_counter(); reps = 0
        while time.perf_counter() - t1 < 4.0:
            oracle.linear_w4a8(xq_o[:1], sx_o[:1], q, s, z, want_acc=False); reps += 1
        cpu_dec_s = (time.perf_counter() - t1) / reps
        t1 = time.perf_counter(); reps = 0
        while time.perf_counter() - t1 < 8.0:
            oracle.linear_w4a8(xq_o, sx_o, q, s, z, want_acc=False); reps += 1
        cpu_pre_s = (time.perf_counter() - t1) / reps
        cpu = {"value": round(decode_bytes(Nc, K) / cpu_dec_s / 1e9, 3), "unit": "GB/s", "cores": cores,
               "kind": "oracle",
               "prefill_value": round(prefill_ops(16, Nc, K) / cpu_pre_s / 1e12, 5), "prefill_unit": "TOP/s",
               "sample": "oracle O4 (scalar C, OpenMP over rows) on %d rows of a [%d x %d] layer: "
                         "decode M=1 for 4 s, prefill M=16 for 8 s" % (Nc, N, K)}

    out = {
        "metric": "decode GEMV HBM GB/s (% peak); prefill W4A8 GEMM int8 TOPS (% MFMA peak)",
        "value": round(dec_gbs, 1) if do_dec else round(pre_tops, 1),
        "unit": "GB/s" if do_dec else "TOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8",   # int8 x int4 -> int32 group sums, fp32 epilogue
        "data": "synthetic: N(0,0.02) weights of one block drawn on the host (seeded) and packed into "
                "%d distinct buffers, N(0,1) activations with 0.1%% outlier channels x20" % n_blocks,
        "config": {"workload": "%s-shaped W4A8 linears: decode batch 1 (%d blocks%s) + prefill M=%d (%d blocks), "
                               "q|k|v and gate|up concatenated along N" %
                               (args.model, n_blocks, " + lm_head" if lm else "", M_pre, n_blocks),
                   "arithmetic": "int8 x int4 -> int32, fp32 epilogue",
                   "group": 64, "graph": not args.no_graph, "phase": args.phase,
                   "fused_decode_quant": bool(args.fused_decode), "weight_mode": args.weight_mode,
                   "concatenated_projections": not args.separate_projections},
        "decode_ms": round(dec_mean, 4) if do_dec else None,
        "decode_gbs": round(dec_gbs, 1) if do_dec else None,
        "decode_frac_of_hbm_peak": round(dec_gbs / HBM_PEAK_GBS, 4) if do_dec else None,
        "decode_other_path": dec_other,
        "prefill_ms": round(pre_mean, 4) if do_pre else None,
        "prefill_value": round(pre_tops, 1) if do_pre else None, "prefill_unit": "TOP/s",
        "prefill_frac_of_int8_peak": round(pre_tops / INT8_PEAK_TOPS, 4) if do_pre else None,
        "roofline": roof_pre if roof_pre is not None else roof_dec,
        "roofline_decode": roof_dec,
        "per_layer": per_layer,
        "cpu_baseline": cpu,
        "achievable": achievable,
        "pack_gbs_fp32_in": round(pack_bytes_in / (pack_ms * 1e-3) / 1e9, 1),
        "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
