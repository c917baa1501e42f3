#!/usr/bin/env python3
"""Benchmark of the W4A8 quantized linear hot path on one MI355X.

Headline workload (benchmark configs[3], the configuration the targets are stated on): the
Qwen2-7B-shaped layers - 28 blocks of q|k|v 3584->4608, o 3584->3584, gate|up 3584->37888,
down 18944->3584 plus the lm_head 3584->152064 - as one decode step (batch 1, activation quantizer
fused into the GEMV) and one prefill pass (M = 1024 tokens, 28 blocks: activation quantizer, operand
rearrangement and GEMM per projection).  One "step" = the decode pass, then the prefill pass.
Inputs are synthetic and resident in HBM before the timed region; every block has its own packed
weights (far beyond the 256 MB Infinity Cache) and its own fp32 activations.

Prints ONE JSON line.  `value` is the decode rate in GB/s of algorithmic bytes; the prefill rate in
int8 TOP/s is `prefill_value`; `roofline` describes the dominant kernel (the prefill GEMM),
`roofline_decode` the fused decode kernels; `configs` holds the other BASELINE configurations;
`cpu_baseline` the oracle on the host cores.
"""
from __future__ import annotations

import argparse
import ctypes
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published (5.0 POP/s)
FP16_PEAK_TFLOPS = 2500.0    # MI355X dense fp16 MFMA, published
G = 64

# bytes of group parameters and of codes per two weights, by weight mode
GROUP_PARAM_BYTES = {"zp": 5, "minfloat": 8, "int8": 16, "int8n": 8}
CODE_BYTES_X2 = {"zp": 1, "minfloat": 1, "int8": 2, "int8n": 2}


def decode_bytes(N, K, wm="zp", act_bytes=1):
    """Algorithmic bytes of one decode GEMV: codes + per-group parameters, the activation row
    (int8 codes; 2 bytes with fp16 activations), and the fp32 output."""
    return CODE_BYTES_X2[wm] * N * K // 2 + GROUP_PARAM_BYTES[wm] * N * (K // G) + act_bytes * K + 4 * N


def prefill_ops(M, N, K):
    return 2 * M * N * K


def source_digest():
    """Digest of the kernel sources: measured HBM traffic stored under profiles/ is only reported
    while it still describes these kernels."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2506_10443_amd", "csrc")
    for f in sorted(os.listdir(d)):
        if f.startswith("mnnq_") and (f.endswith(".hip") or f.endswith(".h")):
            h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def stored_traffic(key):
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE runs, or None."""
    p = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        t = json.load(open(p))
    except (OSError, ValueError):
        return None
    if t.get("source_digest") != source_digest():
        return None
    return t.get(key)


class BenchLib:
    """libmnnq_bench.so: an empty kernel, a streaming read and register-only matrix loops."""

    def __init__(self):
        p = os.path.join(ROOT, "paper_2506_10443_amd", "lib", "libmnnq_bench.so")
        self.L = ctypes.CDLL(p)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        self.L.mnnqb_empty.argtypes = [vp]
        self.L.mnnqb_peak_read.argtypes = [vp, sz, vp, vp]
        self.L.mnnqb_peak_mfma.argtypes = [i32, i32, i32, i32, i32, vp, vp]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--model", default="qwen2-7b", choices=["qwen2-1.5b", "qwen2-7b", "llama3-8b"])
    ap.add_argument("--phase", default="both", choices=["both", "decode", "prefill"])
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the other BASELINE configurations (config 1, Qwen2-1.5B, Llama-3-8B W4A8 / W4A16)")
    ap.add_argument("--no-plane", action="store_true",
                    help="pack without the matrix-core plane: the prefill runs the int8 GEMM on the chunk layout")
    ap.add_argument("--weight-mode", default="zp", choices=["zp", "minfloat", "int8", "int8n"],
                    help="weight quantizer: int4 with an integer zero point (the benchmark configuration), int4 "
                         "as Eq. 1 is printed (float group minimum), int8 weights (float group minimum) as two 4-bit "
                         "planes, or int8 weights as bytes (int8n)")
    ap.add_argument("--act16", action="store_true", help="also time the fp16-activation entry points per layer")
    ap.add_argument("--separate-projections", action="store_true",
                    help="run q, k, v and gate, up as launches of their own instead of concatenated along N")
    ap.add_argument("--two-call-decode", action="store_true",
                    help="decode pass calls mnnq_quant_act + mnnq_linear_decode per layer instead of the fused call")
    ap.add_argument("--lm-head-prefill", action="store_true", help="also time the LM head through the prefill GEMM")
    ap.add_argument("--prefill-plan", type=int, default=None, choices=[0, 1, 2, 3, 4, 5],
                    help="force one tile plan of the fp6 GEMM for every layer (tuning; default: the library's choice)")
    ap.add_argument("--debug-set", action="append", default=[], metavar="KEY=VALUE",
                    help="a test / tuning switch of the library for the whole run (mnnq_debug_set), e.g. MNNQ_PREFILL_TILE=v1")
    ap.add_argument("--peaks", action="store_true", help="(default) measure what this GPU sustains (`achievable`)")
    ap.add_argument("--no-peaks", action="store_true", help="skip the measurement of what this GPU sustains")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 512 MiB device copy (reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
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
    def note(*a):
        # progress lines on stderr, flushed before each GPU step (stdout carries the one JSON line)
        print("[bench]", *a, file=sys.stderr, flush=True)

    note("initialising the GPU")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if not os.path.exists(B.LIB_PATH):   # fail loudly if the HIP library is not built: there is no other path
        raise RuntimeError("libmnnq.so is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    torch.zeros(16, device=dev).sum().item()     # first allocation and kernel before the library is loaded
    B.lib()
    if args.prefill_plan is not None:
        B.mnnq_debug_set("MNNQ_PREFILL6_PLAN", args.prefill_plan)
    for kv in args.debug_set:
        key, _, val = kv.partition("=")
        B.mnnq_debug_set(key, val)
    bench_lib = []

    def BL():
        # libmnnq_bench.so is loaded on first use (--peaks only)
        if not bench_lib:
            bench_lib.append(BenchLib())
        return bench_lib[0]
    use_graph = not args.no_graph

    def stream_ptr():
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    # ------------------------------------------------------------------ timing helpers
    def time_graph(fn_list, reps):
        """Mean ms per entry of fn_list, replayed back to back as one HIP graph (so that the host's
        launch rate does not limit short kernels); HIP events on the replay stream."""
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            for fn in fn_list[:4]:
                fn()
        side.synchronize()
        if use_graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for fn in fn_list:
                    fn()
            run = g.replay
        else:
            def run():
                for fn in fn_list:
                    fn()
        run()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            run()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / (reps * len(fn_list))

    def capture(fn):
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            fn()                       # eager run first (also warms the code objects)
        side.synchronize()
        if not use_graph:
            return fn
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            fn()
        return g.replay

    def time_run(run, reps):
        run()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            run()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    # ------------------------------------------------------------------ one model's buffers and passes
    class Model:
        def __init__(self, model, wm, plane, fused_proj=True, n_blocks=None):
            self.model, self.wm = model, wm
            spec = synth.MODELS[model]
            self.n_blocks = spec["blocks"] if n_blocks is None else n_blocks
            self.M = spec["prefill_m"]
            self.layers = synth.block_layers(model, fused=fused_proj)
            base = {"zp": B.MODE_W4_ZP_INT, "minfloat": B.MODE_W4_MIN_FLOAT, "int8": B.MODE_W8_MIN_FLOAT,
                    "int8n": B.MODE_W8_MIN_FLOAT | B.NATIVE_8BIT}[wm]
            self.mode = base | (B.WITH_MATRIX_PLANE if (plane and wm == "zp") else 0)
            self.plane = bool(self.mode & B.WITH_MATRIX_PLANE)
            t0 = time.time()
            self.packed = {}
            self.pack_ms, self.pack_bytes_in = 0.0, 0
            for name, N, K in self.layers:
                note("packing", model, name, N, K, "x", self.n_blocks, "mode", self.mode)
                parts = [synth.weights(*spec["layers"][p], synth.layer_seed(model, 0, p)) for p in synth.fused_parts(name)]
                W = torch.from_numpy(np.concatenate(parts) if len(parts) > 1 else parts[0]).to(dev)
                del parts
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                self.packed[name] = [B.mnnq_pack_weights(W, mode=self.mode) for _ in range(self.n_blocks)]
                e1.record()
                torch.cuda.synchronize()
                self.pack_ms += e0.elapsed_time(e1)
                self.pack_bytes_in += self.n_blocks * N * K * 4
                del W
            self.lm = None
            if spec["lm_head"] is not None:
                N, K = spec["lm_head"]
                note("packing", model, "lm_head", N, K)
                W = torch.from_numpy(synth.weights(N, K, synth.layer_seed(model, 0, "lm_head"))).to(dev)
                self.lm = (B.mnnq_pack_weights(W, mode=self.mode), N, K)
                del W
            torch.cuda.synchronize()
            self.setup_s = time.time() - t0
            self.io_dec, self.io_pre = {}, {}

        def all_layers(self):
            return self.layers + ([("lm_head", self.lm[1], self.lm[2])] if self.lm else [])

        def make_decode_io(self, outliers=True):
            for i, (name, N, K) in enumerate(self.all_layers()):
                x = torch.from_numpy(synth.activations(1, K, 9000 + 10 * i, outliers=outliers)).to(dev)
                self.io_dec[name] = (x, torch.empty((1, K), dtype=torch.int8, device=dev),
                                     torch.empty((1,), dtype=torch.float32, device=dev),
                                     torch.empty((1, N), dtype=torch.float32, device=dev))
            self.ws_dec = torch.empty(max(B.mnnq_workspace_size(1, N, K) for _, N, K in self.all_layers()),
                                      dtype=torch.uint8, device=dev)

        def make_prefill_io(self, outliers=True):
            """fp32 activations of every block in a buffer of their own (cold inputs); the int8 codes, the
            scales, the rearranged activations and the output are produced and consumed inside a block's
            calls and are shared by the blocks."""
            M = self.M
            for i, (name, N, K) in enumerate(self.layers):
                x0 = torch.from_numpy(synth.activations(M, K, 9001 + 10 * i, outliers=outliers)).to(dev)
                xs = [x0] + [x0.clone() for _ in range(self.n_blocks - 1)]
                ws = torch.empty(max(16, B.mnnq_workspace_size(M, N, K, 64, self.mode)), dtype=torch.uint8, device=dev)
                self.io_pre[name] = (xs, torch.empty((M, K), dtype=torch.int8, device=dev),
                                     torch.empty((M,), dtype=torch.float32, device=dev),
                                     torch.empty((M, N), dtype=torch.float32, device=dev), ws)

        # decode: one call per projection
        def decode_layer(self, p, N, K, io, fused):
            x, xq, sx, y = io
            if fused:
                B.mnnq_linear_decode_fused(p, N, K, x, out=y, workspace=self.ws_dec, mode=self.mode)
            else:
                B.mnnq_quant_act(x, want_xsum=False, out=(xq, sx, None))
                B.mnnq_linear_decode(p, N, K, xq, sx, out=y, mode=self.mode)

        def decode_pass(self, fused=True):
            for b in range(self.n_blocks):
                for name, N, K in self.layers:
                    self.decode_layer(self.packed[name][b], N, K, self.io_dec[name], fused)
            if self.lm is not None:
                self.decode_layer(self.lm[0], self.lm[1], self.lm[2], self.io_dec["lm_head"], fused)

        # prefill: quantizer + linear call (which rearranges the codes and runs the GEMM) per projection
        def prefill_pass(self):
            for b in range(self.n_blocks):
                for name, N, K in self.layers:
                    xs, xq, sx, y, ws = self.io_pre[name]
                    B.mnnq_quant_act(xs[b], want_xsum=False, out=(xq, sx, None))
                    B.mnnq_linear_prefill(self.packed[name][b], N, K, xq, sx, out=y, mode=self.mode, workspace=ws)

        def dec_bytes(self):
            return self.n_blocks * sum(decode_bytes(N, K, self.wm) for _, N, K in self.layers) + \
                (decode_bytes(self.lm[1], self.lm[2], self.wm) if self.lm else 0)

        def pre_ops(self):
            return self.n_blocks * sum(prefill_ops(self.M, N, K) for _, N, K in self.layers)

        # per-kernel timings of the prefill pass
        def prefill_kernels(self):
            """Per layer: the activation quantizer, the operand rearrangement and the GEMM, each timed as
            launches of its own; and all GEMM launches of a pass together."""
            per, gemm_fns = {}, []
            for name, N, K in self.layers:
                xs, xq, sx, y, ws = self.io_pre[name]
                nb = self.n_blocks
                # (every loop variable a launch uses is bound as a default argument: the launches are replayed again
                # after the loop, when the names point at the last layer)
                tq = time_graph([(lambda x=xs[b], xq=xq, sx=sx: B.mnnq_quant_act(x, want_xsum=False, out=(xq, sx, None)))
                                 for b in range(nb)], 2)
                entry = {"quant_us": round(tq * 1e3, 2)}
                if self.plane and B.mnnq_plan_debug(0, self.M, N, K, mode=self.mode)[7] == 6:   # the pass takes the fp6 GEMM here
                    planes = ws[:B.lib().mnnq_act_planes_size(self.M, K, 64)]
                    tp = time_graph([lambda xq=xq, planes=planes: B.mnnq_act_planes(xq, out=planes)] * nb, 2)
                    lay = [(lambda p=self.packed[name][b], N=N, K=K, planes=planes, sx=sx, y=y:
                            B.mnnq_linear_prefill_planes(p, self.M, N, K, planes, sx, out=y, mode=self.mode))
                           for b in range(nb)]
                    entry["planes_us"] = round(tp * 1e3, 2)
                else:
                    lay = [(lambda p=self.packed[name][b], N=N, K=K, xq=xq, sx=sx, y=y:
                            B.mnnq_linear_prefill(p, N, K, xq, sx, out=y, mode=self.mode))
                           for b in range(nb)]
                tg = time_graph(lay, 2)
                entry["gemm_us"] = round(tg * 1e3, 2)
                entry["gemm_tops"] = round(prefill_ops(self.M, N, K) / (tg * 1e-3) / 1e12, 1)
                entry["gemm_frac"] = round(entry["gemm_tops"] / INT8_PEAK_TOPS, 4)
                per["prefill_" + name] = entry
                gemm_fns += lay
            t = time_graph(gemm_fns, 2)
            return per, t, len(gemm_fns)

        def decode_kernels(self, fused=True):
            per, fns = {}, []
            for name, N, K in self.layers:
                io = self.io_dec[name]
                lay = [(lambda p=self.packed[name][b], N=N, K=K, io=io: self.decode_layer(p, N, K, io, fused))
                       for b in range(self.n_blocks)]
                t = time_graph(lay, 4)
                per["decode_" + name] = {"us": round(t * 1e3, 2), "gbs": round(decode_bytes(N, K, self.wm) / (t * 1e-3) / 1e9, 1)}
                if fused:   # the GEMV alone, on a row quantized beforehand
                    x, xq, sx, y = io
                    B.mnnq_quant_act(x, want_xsum=False, out=(xq, sx, None))
                    t2 = time_graph([(lambda p=self.packed[name][b], N=N, K=K, xq=xq, sx=sx, y=y:
                                      B.mnnq_linear_decode(p, N, K, xq, sx, out=y, mode=self.mode))
                                     for b in range(self.n_blocks)], 4)
                    per["decode_" + name]["gemv_alone_us"] = round(t2 * 1e3, 2)
                # the same launch on one packed buffer over and over: every weight byte already in the Infinity
                # Cache - what is left is the kernel's latency chain, not HBM time
                tw = time_graph([lay[0]] * self.n_blocks, 4)
                per["decode_" + name]["cache_resident_us"] = round(tw * 1e3, 2)
                fns += lay
            t = time_graph(fns, 4)
            if self.lm is not None:
                io = self.io_dec["lm_head"]
                tl = time_graph([lambda: self.decode_layer(self.lm[0], self.lm[1], self.lm[2], io, fused)] * 4, 4)
                kern = 2 if (fused and self.lm[0].numel() > (96 << 20)) else 1
                per["decode_lm_head"] = {"us": round(tl * 1e3, 2), "kernels": kern,
                                         "gbs": round(decode_bytes(self.lm[1], self.lm[2], self.wm) / (tl * 1e-3) / 1e9, 1)}
            return per, t, len(fns)

    def launch_floor_us(n):
        """Mean time per kernel of a graph of n kernels that do next to nothing, on one stream (dependent,
        like a pass): the activation quantizer on one row of 64 values."""
        x0 = torch.zeros((1, 64), dtype=torch.float32, device=dev)
        o0 = (torch.empty((1, 64), dtype=torch.int8, device=dev), torch.empty((1,), dtype=torch.float32, device=dev), None)
        t = time_graph([lambda: B.mnnq_quant_act(x0, want_xsum=False, out=o0)] * n, 4)
        return t * 1e3

    # ================================================================== headline model
    do_dec = args.phase in ("both", "decode")
    do_pre = args.phase in ("both", "prefill")
    fused_dec = not args.two_call_decode
    mdl = Model(args.model, args.weight_mode, not args.no_plane, fused_proj=not args.separate_projections)
    if do_dec:
        mdl.make_decode_io()
    if do_pre:
        mdl.make_prefill_io()
    note("decode pass: eager run and graph capture")
    run_dec = capture(lambda: mdl.decode_pass(fused_dec)) if do_dec else None
    torch.cuda.synchronize()
    note("prefill pass: eager run and graph capture")
    run_pre = capture(mdl.prefill_pass) if do_pre else None
    torch.cuda.synchronize()
    note("timed steps")

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

    dec_bytes, pre_ops = mdl.dec_bytes(), mdl.pre_ops()
    dec_mean = float(np.mean(dec_ms)) if do_dec else None
    pre_mean = float(np.mean(pre_ms)) if do_pre else None
    dec_gbs = dec_bytes / (dec_mean * 1e-3) / 1e9 if do_dec else None
    pre_tops = pre_ops / (pre_mean * 1e-3) / 1e12 if do_pre else None

    # ------------------------------------------------------------------ per-kernel figures and rooflines
    per_layer, roof_pre, roof_dec, dec_decomp, pre_decomp = {}, None, None, None, None
    headline_cfg = (args.model, args.weight_mode) == ("qwen2-7b", "zp") and not args.separate_projections
    if do_pre:
        note("per-kernel timings: prefill")
        per, t, n = mdl.prefill_kernels()
        per_layer.update(per)
        ach = pre_ops / n / (t * 1e-3) / 1e12
        kern = "prefill6_kernel (fp6 matrix instructions on int8 x int4 operands)" if mdl.plane else "prefill_kernel (int8 MFMA)"
        roof_pre = {"kernel": "%s, all %d GEMM launches of a pass" % (kern, n),
                    "bound": "mfma", "achieved": round(ach, 1), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                    "frac": round(ach / INT8_PEAK_TOPS, 4),
                    "traffic": stored_traffic("prefill_gemm_bytes_per_launch") if (headline_cfg and mdl.plane) else None,
                    "algorithmic_ops_per_launch": pre_ops // n, "avg_launch_us": round(t * 1e3, 2)}
        parts = {k: sum(v.get(k, 0.0) for v in per.values()) * mdl.n_blocks * 1e-3 for k in ("quant_us", "planes_us", "gemm_us")}
        pre_decomp = {"pass_ms": round(pre_mean, 4), "sum_of_kernels_ms": round(sum(parts.values()), 4),
                      "quant_act_ms": round(parts["quant_us"], 4), "act_planes_ms": round(parts["planes_us"], 4),
                      "gemm_ms": round(parts["gemm_us"], 4), "kernels_per_pass": (3 if mdl.plane else 2) * n}
    if do_dec:
        note("per-kernel timings: decode")
        per, t, n = mdl.decode_kernels(fused_dec)
        per_layer.update(per)
        byt = mdl.n_blocks * sum(decode_bytes(N, K, mdl.wm) for _, N, K in mdl.layers)
        ach = byt / n / (t * 1e-3) / 1e9
        what = "decode_kernel, fused form (activation quantizer inside the GEMV)" if fused_dec else \
            "quant_act_kernel + decode_kernel per layer"
        roof_dec = {"kernel": "%s: the %d block launches the timed pass makes" % (what, n),
                    "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4),
                    "traffic": stored_traffic("decode_fused_bytes_per_launch") if (headline_cfg and fused_dec) else None,
                    "algorithmic_bytes_per_launch": byt // n, "avg_launch_us": round(t * 1e3, 2)}
        n_kern = n * (1 if fused_dec else 2) + (per.get("decode_lm_head", {}).get("kernels", 0) if fused_dec else (2 if mdl.lm else 0))
        floor = launch_floor_us(n_kern)
        ksum = sum(per["decode_" + name]["us"] for name, _, _ in mdl.layers) * mdl.n_blocks + \
            (per["decode_lm_head"]["us"] if mdl.lm else 0.0)
        dec_decomp = {"pass_us": round(dec_mean * 1e3, 1), "sum_of_kernels_us": round(ksum, 1), "kernels_per_pass": n_kern,
                      "launch_floor_us": round(floor, 2),
                      "launch_floor_total_us": round(floor * n_kern, 1),
                      "fused_kernel_frac": round(ach / HBM_PEAK_GBS, 4),
                      "note": "per-kernel times are means over back-to-back graph replays of that kernel alone and "
                              "include the gap to the next launch; launch_floor_us is the same measurement for a "
                              "kernel with next to no work (the quantizer on 64 values)"}
        # the other decode path, for comparison
        if use_graph:
            other = capture(lambda: mdl.decode_pass(not fused_dec))
            ms = time_run(other, 10)
            dec_decomp["other_path"] = {"path": "two-call" if fused_dec else "fused", "ms": round(ms, 4),
                                        "gbs": round(dec_bytes / (ms * 1e-3) / 1e9, 1)}

    if args.lm_head_prefill and mdl.lm is not None and do_pre:
        p, N, K = mdl.lm
        xf = torch.from_numpy(synth.activations(mdl.M, K, 4242, outliers=True)).to(dev)
        xq_l, sx_l, _ = B.mnnq_quant_act(xf, want_xsum=False)
        y_l = torch.empty((mdl.M, N), dtype=torch.float32, device=dev)
        ws_l = torch.empty(max(16, B.mnnq_workspace_size(mdl.M, N, K, 64, mdl.mode)), dtype=torch.uint8, device=dev)
        t = time_graph([lambda: B.mnnq_linear_prefill(p, N, K, xq_l, sx_l, out=y_l, mode=mdl.mode, workspace=ws_l)] * 2, 3)
        per_layer["prefill_lm_head"] = {"us": round(t * 1e3, 2), "tops": round(prefill_ops(mdl.M, N, K) / (t * 1e-3) / 1e12, 1)}
        del xf, xq_l, sx_l, y_l, ws_l

    if args.act16:
        for name, N, K in mdl.layers:
            if do_pre:
                x16 = mdl.io_pre[name][0][0].to(torch.float16)
                y = mdl.io_pre[name][3]
                t = time_graph([(lambda p=mdl.packed[name][b], N=N, K=K, x16=x16, y=y:
                                 B.mnnq_linear_prefill_f16(p, N, K, x16, out=y, mode=mdl.mode))
                                for b in range(mdl.n_blocks)], 2)
                per_layer["prefill16_" + name] = {"us": round(t * 1e3, 2),
                                                  "tflops": round(prefill_ops(mdl.M, N, K) / (t * 1e-3) / 1e12, 1)}
            if do_dec:
                x16 = mdl.io_dec[name][0].to(torch.float16)
                y = mdl.io_dec[name][3]
                try:
                    t = time_graph([(lambda p=mdl.packed[name][b], N=N, K=K, x16=x16, y=y:
                                     B.mnnq_linear_decode_f16(p, N, K, x16[0], out=y[0], mode=mdl.mode))
                                    for b in range(mdl.n_blocks)], 4)
                except B.MnnqError:      # the fp16 row of this layer does not fit the GEMV's LDS staging
                    per_layer["decode16_" + name] = None
                    continue
                per_layer["decode16_" + name] = {"us": round(t * 1e3, 2),
                                                 "gbs": round(decode_bytes(N, K, mdl.wm, 2) / (t * 1e-3) / 1e9, 1)}

    if args.calibrate_copy:
        src = torch.empty(128 * 1024 * 1024, dtype=torch.int32, device=dev).fill_(7)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    achievable = None
    if not args.no_peaks:
        note("what the GPU sustains (streaming read, matrix loops)")
        sink = torch.zeros(4, dtype=torch.float32, device=dev)
        big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)       # 1 GiB: 4x the Infinity Cache
        t = time_run(lambda: BL().L.mnnqb_peak_read(big.data_ptr(), big.numel(), sink.data_ptr(), stream_ptr()), 10) * 1e-3
        achievable = {"hbm_read_gbs": round(big.numel() / t / 1e9, 1)}
        del big
        cus = torch.cuda.get_device_properties(dev).multi_processor_count
        # operations per matrix instruction; kinds 3 / 4 count the GEMM's int8-equivalent operations (half of
        # what the instruction does: an int8 activation takes two fp6 operands)
        ops = {0: 2 * 16 * 16 * 64, 1: 2 * 16 * 16 * 32, 2: 2 * 16 * 16 * 128, 3: 32 * 32 * 64, 4: 32 * 32 * 64}
        for key, kind, epi, waves in (("mfma_int8_tops", 0, 0, (2, 4)), ("mfma_fp16_tflops", 1, 0, (2, 4)),
                                      ("mfma_fp8_tflops", 2, 0, (2, 4)),
                                      ("mfma_int8_with_cvt_fma_tops", 0, 1, (2, 4)),
                                      ("mfma_int8_with_cvt_fma_8int_tops", 0, 2, (2, 4)),
                                      ("mfma_fp6_pairs_int8_equivalent_tops", 3, 0, (1, 2)),
                                      ("mfma_fp6_pairs_with_fma_int8_equivalent_tops", 4, 0, (1, 2))):
            # seed 1: constant operands; seed 7: operands whose bits differ from lane to lane like real data - the
            # chip runs these loops against its power limit and clocks by how much toggles (the clock a wave
            # saw over the kernel's life comes back in sink[1])
            for seed, suffix in ((1, ""), (7, "_random_operands")):
                best, mhz = 0.0, None
                for w in waves:
                    sink.zero_()
                    t = time_run(lambda: BL().L.mnnqb_peak_mfma(kind, epi, w, 2000, seed, sink.data_ptr(), stream_ptr()), 3) * 1e-3
                    rate = cus * 4 * w * 2000 * 16 * ops[kind] / t / 1e12
                    if rate > best:
                        best, mhz = rate, float(sink[1].item())
                achievable[key + suffix] = round(best, 1)
                achievable[key + suffix + "_shader_mhz"] = round(mhz)

    pack_gbs = round(mdl.pack_bytes_in / (mdl.pack_ms * 1e-3) / 1e9, 1)
    # The load-time kernels in steady state: the largest layer of the block quantized and stored into buffers
    # allocated before (the set-up figure above includes the allocations and, with the plane, both kernels).
    note("load-time kernels")
    name_p, N_p, K_p = max(mdl.layers, key=lambda l: l[1] * l[2])
    srcs = [torch.randn((N_p, K_p), dtype=torch.float32, device=dev) * 0.02 for _ in range(2)]
    mode_c = mdl.mode & ~B.WITH_MATRIX_PLANE      # the chunk layout alone
    dsts = [torch.empty(B.mnnq_packed_size(N_p, K_p, 64, mode_c), dtype=torch.uint8, device=dev) for _ in range(2)]
    t_pack = time_run(lambda: [B.mnnq_pack_weights(s, out=d, mode=mode_c) for s, d in zip(srcs, dsts)], 5) / 2
    pack = {"layer": name_p, "quantize_and_store_us": round(t_pack * 1e3, 1),
            "bytes": 4 * N_p * K_p + dsts[0].numel(),
            "gbs": round((4 * N_p * K_p + dsts[0].numel()) / (t_pack * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round((4 * N_p * K_p + dsts[0].numel()) / (t_pack * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "set_up_gbs_fp32_in": pack_gbs}
    if mdl.plane:
        dsts6 = [torch.empty(B.mnnq_packed_size(N_p, K_p, 64, mdl.mode), dtype=torch.uint8, device=dev) for _ in range(2)]
        t6 = time_run(lambda: [B.mnnq_pack_weights(s, out=d, mode=mdl.mode) for s, d in zip(srcs, dsts6)], 5) / 2
        pack["with_matrix_plane_us"] = round(t6 * 1e3, 1)
        del dsts6
    del srcs, dsts
    setup_s = mdl.setup_s
    n_blocks, M_pre, has_lm, plane = mdl.n_blocks, mdl.M, mdl.lm is not None, mdl.plane
    packed_bytes_per_weight = round(sum(mdl.packed[name][0].numel() for name, _, _ in mdl.layers) /
                                    sum(N * K for _, N, K in mdl.layers), 4)

    # ================================================================== the other BASELINE configurations
    configs = None
    if not args.no_configs and args.phase == "both" and headline_cfg:
        del mdl, run_dec, run_pre
        torch.cuda.empty_cache()
        configs = {}

        note("config 1")
        # --- config 1: a single 8960 x 1536 layer, decode, seed 0: cold (64 packed copies, 0.5 GB, round-robin) and warm
        W1, x1 = synth.config1()
        Wd, xd = torch.from_numpy(W1).to(dev), torch.from_numpy(x1).to(dev)
        N1, K1 = W1.shape
        copies = [B.mnnq_pack_weights(Wd) for _ in range(64)]
        y1 = torch.empty((1, N1), dtype=torch.float32, device=dev)
        ws1 = torch.empty(B.mnnq_workspace_size(1, N1, K1), dtype=torch.uint8, device=dev)
        tc = time_graph([(lambda p=p: B.mnnq_linear_decode_fused(p, N1, K1, xd, out=y1, workspace=ws1)) for p in copies], 8)
        tw = time_graph([lambda: B.mnnq_linear_decode_fused(copies[0], N1, K1, xd, out=y1, workspace=ws1)] * 64, 8)
        b1 = decode_bytes(N1, K1)
        configs["config1_single_8960x1536_decode"] = {
            "algorithmic_bytes": b1,
            "cold_us": round(tc * 1e3, 2), "cold_gbs": round(b1 / (tc * 1e-3) / 1e9, 1), "cold_frac_of_hbm_peak": round(b1 / (tc * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "warm_us": round(tw * 1e3, 2), "warm_gbs": round(b1 / (tw * 1e-3) / 1e9, 1), "warm_is_cache_resident": True,
            "call": "mnnq_linear_decode_fused, 64 launches per graph replay; cold: 64 distinct packed copies (0.51 GB)"}
        del copies, Wd, xd, y1, ws1
        torch.cuda.empty_cache()

        def model_summary(model, a16):
            note("configuration", model)
            m = Model(model, "zp", True)
            m.make_decode_io(outliers=(model != "llama3-8b"))
            m.make_prefill_io(outliers=(model != "llama3-8b"))
            out = {}
            note(model, "decode pass")
            rd = capture(lambda: m.decode_pass(True))
            td = time_run(rd, 10)
            out["decode_ms"] = round(td, 4)
            out["decode_gbs"] = round(m.dec_bytes() / (td * 1e-3) / 1e9, 1)
            out["decode_frac_of_hbm_peak"] = round(out["decode_gbs"] / HBM_PEAK_GBS, 4)
            note(model, "prefill pass")
            rp = capture(m.prefill_pass)
            tp = time_run(rp, 3)
            out["prefill_m"] = m.M
            out["prefill_ms"] = round(tp, 4)
            out["prefill_tops"] = round(m.pre_ops() / (tp * 1e-3) / 1e12, 1)
            out["prefill_frac_of_int8_peak"] = round(out["prefill_tops"] / INT8_PEAK_TOPS, 4)
            # bytes a prefill pass has to move at least: packed weights, int8 activations, fp32 output
            pre_bytes = m.n_blocks * sum(decode_bytes(N, K) - K - 4 * N + m.M * K + 4 * m.M * N for _, N, K in m.layers)
            out["prefill_frac_of_hbm_peak"] = round(pre_bytes / (tp * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
            per, t, n = m.prefill_kernels()
            out["prefill_gemm_tops"] = round(m.pre_ops() / n / (t * 1e-3) / 1e12, 1)
            out["per_layer"] = {k: {"gemm_us": v["gemm_us"], "gemm_tops": v["gemm_tops"]} for k, v in per.items()}
            if a16:
                note(model, "fp16 activations")
                # the same layers with fp16 activations (W4A16): decode and prefill passes of the _f16 calls
                x16d = {name: m.io_dec[name][0].to(torch.float16) for name, _, _ in m.layers}
                x16p = {name: m.io_pre[name][0][0].to(torch.float16) for name, _, _ in m.layers}

                def dec16():
                    for b in range(m.n_blocks):
                        for name, N, K in m.layers:
                            B.mnnq_linear_decode_f16(m.packed[name][b], N, K, x16d[name][0], out=m.io_dec[name][3][0], mode=m.mode)

                def pre16():
                    for b in range(m.n_blocks):
                        for name, N, K in m.layers:
                            B.mnnq_linear_prefill_f16(m.packed[name][b], N, K, x16p[name], out=m.io_pre[name][3], mode=m.mode)
                td16 = time_run(capture(dec16), 10)
                tp16 = time_run(capture(pre16), 3)
                b16 = m.n_blocks * sum(decode_bytes(N, K, "zp", 2) for _, N, K in m.layers)
                out["w4a16"] = {"decode_ms": round(td16, 4), "decode_gbs": round(b16 / (td16 * 1e-3) / 1e9, 1),
                                "decode_frac_of_hbm_peak": round(b16 / (td16 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                "prefill_ms": round(tp16, 4),
                                "prefill_tflops": round(m.pre_ops() / (tp16 * 1e-3) / 1e12, 1),
                                "prefill_frac_of_fp16_peak": round(m.pre_ops() / (tp16 * 1e-3) / 1e12 / FP16_PEAK_TFLOPS, 4)}
            del m
            torch.cuda.empty_cache()
            return out

        configs["qwen2-1.5b_w4a8_decode_and_prefill_m512"] = model_summary("qwen2-1.5b", False)
        configs["llama3-8b_w4a8_and_w4a16_decode_and_prefill_m2048"] = model_summary("llama3-8b", True)

    # ================================================================== CPU baseline: the oracle on the host cores
    cpu = None
    if not args.no_cpu_baseline:
        note("cpu baseline (oracle on the host cores)")
        import oracle
        cores = len(os.sched_getaffinity(0))
        try:
            cpu_model = [l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name")][0]
        except (OSError, IndexError):
            cpu_model = "unknown"
        spec = synth.MODELS[args.model]
        shapes = {}     # distinct (N, K) -> [count per block, name of one projection]
        for p_, (N, K) in spec["layers"].items():
            shapes.setdefault((N, K), [0, p_])[0] += 1
        rows_cap = 4096          # a layer is timed on its first rows_cap output rows and scaled by N / rows
        budget = {"dec1": 0.0, "decN": 0.0, "pre1": 0.0, "preN": 0.0}
        m1, mN = 4, 48           # token rows of the prefill samples (1 thread / all cores), scaled by M / rows
        sample_s = 0.0
        for (N, K), (cnt, p_) in shapes.items():
            rows = min(N, rows_cap)
            Wc = synth.weights(N, K, synth.layer_seed(args.model, 0, p_))[:rows]
            q, s, z = oracle.quant_weights(Wc)
            xs_ = synth.activations(mN, K, 9001, outliers=True)
            xq_o, sx_o, _ = oracle.quant_act(xs_)
            scale = cnt * spec["blocks"] * (N / rows)
            for key, threads, xr in (("dec1", 1, 1), ("decN", cores, 1), ("pre1", 1, m1), ("preN", cores, mN)):
                oracle.set_threads(threads)
                oracle.linear_w4a8(xq_o[:xr], sx_o[:xr], q, s, z, want_acc=False)   # warm
                t1 = time.perf_counter(); reps = 0
                while reps < 1 or time.perf_counter() - t1 < 1.0:
                    oracle.linear_w4a8(xq_o[:xr], sx_o[:xr], q, s, z, want_acc=False); reps += 1
                dt = (time.perf_counter() - t1) / reps
                sample_s += dt * reps
                budget[key] += dt * scale * ((spec["prefill_m"] / xr) if key.startswith("pre") else 1.0)
            del Wc, q, s, z
        blk_bytes = spec["blocks"] * sum(decode_bytes(N, K) for N, K in spec["layers"].values())
        blk_ops = spec["blocks"] * sum(prefill_ops(spec["prefill_m"], N, K) for N, K in spec["layers"].values())
        cpu = {"value": round(blk_bytes / budget["decN"] / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
               "cpu_model": cpu_model,
               "decode_pass_s": {"threads_1": round(budget["dec1"], 3), "threads_all": round(budget["decN"], 3)},
               "decode_gbs": {"threads_1": round(blk_bytes / budget["dec1"] / 1e9, 3), "threads_all": round(blk_bytes / budget["decN"] / 1e9, 3)},
               "prefill_pass_s": {"threads_1": round(budget["pre1"], 1), "threads_all": round(budget["preN"], 1)},
               "prefill_tops": {"threads_1": round(blk_ops / budget["pre1"] / 1e12, 6), "threads_all": round(blk_ops / budget["preN"] / 1e12, 6)},
               "prefill_value": round(blk_ops / budget["preN"] / 1e12, 6), "prefill_unit": "TOP/s",
               "sample": "oracle O4 (plain scalar C; OpenMP over output rows for the all-cores figure) on one instance per "
                         "distinct layer shape of a %s block (%s), seeded like the GPU leg, timed on the first %d output rows "
                         "(scaled by N / rows), decode with 1 token, prefill with %d (1 thread) / %d (all cores) tokens "
                         "(scaled by %d / tokens), each multiplied by its count per block x %d blocks: extrapolated; "
                         "%.1f s of CPU work measured" % (args.model, ", ".join("%dx%d" % k for k in shapes), rows_cap, m1, mN,
                                                            spec["prefill_m"], spec["blocks"], sample_s)}

    out = {
        "metric": "decode GEMV HBM GB/s (% peak); prefill W4A8 GEMM int8 TOPS (% MFMA peak)",
        "value": round(dec_gbs, 1) if do_dec else round(pre_tops, 1),
        "unit": "GB/s" if do_dec else "TOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8",   # int8 x int4 -> int32 group sums (exact in fp32 on the fp6 matrix instructions), fp32 epilogue
        "data": "synthetic: N(0,0.02) weights of one block drawn on the host (seeded) and packed into "
                "%d distinct buffers, N(0,1) activations with 0.1%% outlier channels x20, a buffer per block" % n_blocks,
        "config": {"workload": "%s-shaped W4A8 linears: decode batch 1 (%d blocks%s) + prefill M=%d (%d blocks), "
                               "q|k|v and gate|up concatenated along N" %
                               (args.model, n_blocks, " + lm_head" if has_lm else "", M_pre, n_blocks),
                   "arithmetic": "int8 x int4 -> int32 group sums, fp32 epilogue",
                   "group": 64, "graph": use_graph, "phase": args.phase,
                   "fused_decode_quant": bool(fused_dec), "weight_mode": args.weight_mode,
                   "matrix_core_plane": plane, "packed_bytes_per_weight": packed_bytes_per_weight,
                   "concatenated_projections": not args.separate_projections},
        "decode_ms": round(dec_mean, 4) if do_dec else None,
        "decode_gbs": round(dec_gbs, 1) if do_dec else None,
        "decode_frac_of_hbm_peak": round(dec_gbs / HBM_PEAK_GBS, 4) if do_dec else None,
        "decode_decomposition": dec_decomp,
        "prefill_ms": round(pre_mean, 4) if do_pre else None,
        "prefill_value": round(pre_tops, 1) if do_pre else None, "prefill_unit": "TOP/s",
        "prefill_frac_of_int8_peak": round(pre_tops / INT8_PEAK_TOPS, 4) if do_pre else None,
        "prefill_decomposition": pre_decomp,
        "roofline": roof_pre if roof_pre is not None else roof_dec,
        "roofline_decode": roof_dec,
        "per_layer": per_layer,
        "configs": configs,
        "cpu_baseline": cpu,
        "achievable": achievable,
        "pack": pack,
        "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
