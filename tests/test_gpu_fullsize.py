"""GPU parity at the full layer sizes of the benchmark configurations, in the launch configuration
bench.py times (same entry points, same shapes, q|k|v and gate|up concatenated, packed buffers with
the matrix-core plane: the fp6 GEMM when the call gets its workspace, the int8 GEMM without).

Codes, zero points, scales and int8 activations are compared in full (bit-exact).
Prefill outputs are compared on (m, n) pairs the oracle computes one by one: one pair, at a random
place, in every 16 x 16 block of the output - so every matrix-instruction tile of every workgroup
tile is checked - plus the corners; decode outputs in full; integer group accumulators on a subset
of token rows.  Tolerances: 1e-5 * max|y| (W4A8), 1e-3 * max|y| (W4A16)."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2506_10443_amd import binding as B, synth

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def note(*a):
    print(*a, flush=True)


MODE_PLANE = B.MODE_W4_ZP_INT | B.WITH_MATRIX_PLANE


def stratified_pairs(M, N, rng, tile=16):
    """One (m, n) at a random place in every tile x tile block of an M x N output, plus the corners."""
    mt, nt = -(-M // tile), -(-N // tile)
    m = np.minimum(np.arange(mt)[:, None] * tile + rng.integers(0, tile, (mt, nt)), M - 1)
    n = np.minimum(np.arange(nt)[None, :] * tile + rng.integers(0, tile, (mt, nt)), N - 1)
    ms = np.concatenate([m.ravel(), [0, 0, M - 1, M - 1]])
    ns = np.concatenate([n.ravel(), [0, N - 1, 0, N - 1]])
    return ms.astype(np.int64), ns.astype(np.int64)


def fused_weights(model, name):
    parts = [synth.weights(*synth.MODELS[model]["layers"][p], synth.layer_seed(model, 0, p))
             for p in synth.fused_parts(name)]
    return np.concatenate(parts) if len(parts) > 1 else parts[0]


def check_w4a8_layer(model, name, M, seed, acc_rows=8):
    W = fused_weights(model, name)
    N, K = W.shape
    note("full-size W4A8", model, name, "M", M, "N", N, "K", K)
    x = synth.activations(M, K, seed, outliers=True)
    q, s, z = oracle.quant_weights(W)
    xq_o, sx_o, _ = oracle.quant_act(x)

    packed = B.mnnq_pack_weights(dev(W), mode=MODE_PLANE)
    del W
    qg, sg, zg = B.mnnq_unpack_weights(packed, N, K, mode=MODE_PLANE)
    assert np.array_equal(zg.cpu().numpy(), z)
    assert np.array_equal(sg.cpu().numpy().view(np.uint32), s.view(np.uint32))
    assert np.array_equal(qg.cpu().numpy(), q)
    del qg, sg, zg
    xq, sx, _ = B.mnnq_quant_act(dev(x), want_xsum=False)
    assert np.array_equal(xq.cpu().numpy(), xq_o)
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), sx_o.view(np.uint32))

    # prefill, both GEMMs: one output per 16 x 16 block, plus the corners
    rng = np.random.default_rng(seed)
    ms, ns = stratified_pairs(M, N, rng)
    _, y_s = oracle.linear_w4a8_sampled(xq_o, sx_o, q, s, z, ms, ns, want_acc=False)
    ws = torch.empty(B.mnnq_workspace_size(M, N, K, 64, MODE_PLANE), dtype=torch.uint8, device="cuda:0")
    # the fp6 GEMM, except where the shape has too few output tiles for it (Qwen2-1.5B's down: 48 tiles)
    fp6 = B.mnnq_plan_debug(0, M, N, K, mode=MODE_PLANE)[7] == 6
    assert fp6 == ((model, name) != ("qwen2-1.5b", "down"))
    y6 = B.mnnq_linear_prefill(packed, N, K, xq, sx, mode=MODE_PLANE, workspace=ws).cpu().numpy()
    ymax = np.abs(y6).max()
    err = np.abs(y6[ms, ns] - y_s).max()
    assert err <= 1e-5 * ymax, ("fp6 GEMM", err, ymax)
    assert np.isfinite(y6).all()
    y = B.mnnq_linear_prefill(packed, N, K, xq, sx, mode=MODE_PLANE).cpu().numpy()   # no workspace: the int8 GEMM
    err = np.abs(y[ms, ns] - y_s).max()
    assert err <= 1e-5 * ymax, ("int8 GEMM", err, ymax)
    assert np.isfinite(y).all()
    assert np.abs(y6 - y).max() <= 2e-5 * ymax
    del y6, ws

    # integer accumulators of both matrix-instruction loops on a few token rows
    rows = np.sort(rng.choice(M, size=min(acc_rows, M), replace=False))
    acc = B.mnnq_linear_acc_debug(packed, N, K, dev(xq_o[rows]), True, mode=MODE_PLANE).cpu().numpy()
    pm = np.repeat(np.arange(len(rows)), 512)
    pn = rng.integers(0, N, len(pm))
    acc_s, _ = oracle.linear_w4a8_sampled(xq_o[rows], sx_o[rows], q, s, z, pm, pn)
    assert np.array_equal(acc[pm, pn], acc_s)
    del acc
    rows6 = np.sort(rng.choice(M, size=min(40, M), replace=False))          # (the fp6 GEMM wants more than 32 rows)
    acc6 = B.mnnq_linear_acc_debug_planes(packed, N, K, dev(xq_o[rows6]), MODE_PLANE).cpu().numpy()
    pm6 = np.repeat(np.arange(len(rows6)), 128)
    pn6 = rng.integers(0, N, len(pm6))
    acc_s6, _ = oracle.linear_w4a8_sampled(xq_o[rows6], sx_o[rows6], q, s, z, pm6, pn6)
    assert np.array_equal(acc6[pm6, pn6], acc_s6)
    del acc6

    # decode: row 0 in full, through both the two-call and the fused entry point
    _, y0 = oracle.linear_w4a8(xq_o[:1], sx_o[:1], q, s, z, want_acc=False)
    yd = B.mnnq_linear_decode(packed, N, K, xq[0].contiguous(), sx[:1].contiguous(), mode=MODE_PLANE).cpu().numpy()
    tol0 = 1e-5 * np.abs(y0).max()
    assert np.abs(yd - y0[0]).max() <= tol0
    yf = B.mnnq_linear_decode_fused(packed, N, K, dev(x[0]), mode=MODE_PLANE).cpu().numpy()
    assert np.abs(yf - y0[0]).max() <= tol0
    # with a workspace the fused call may run the quantizer as its own kernel (large layers):
    # same codes, same GEMV kernel as the two-call form, hence the same bits; otherwise the same tolerance
    ws = torch.empty(B.mnnq_workspace_size(1, N, K), dtype=torch.uint8, device="cuda:0")
    yw = B.mnnq_linear_decode_fused(packed, N, K, dev(x[0]), workspace=ws, mode=MODE_PLANE).cpu().numpy()
    assert np.abs(yw - y0[0]).max() <= tol0
    if B.mnnq_packed_size(N, K) > (96 << 20):
        assert np.array_equal(yw, yd)
    B.mnnq_debug_set("MNNQ_FUSED_TWO_KERNEL_MIB", "0")       # ... forced for any size
    try:
        yw = B.mnnq_linear_decode_fused(packed, N, K, dev(x[0]), workspace=ws, mode=MODE_PLANE).cpu().numpy()
    finally:
        B.mnnq_debug_set("MNNQ_FUSED_TWO_KERNEL_MIB", None)
    assert np.array_equal(yw, yd)
    # the same row out of the prefill kernel agrees with the decode kernel to the same bound
    assert np.abs(y[0] - y0[0]).max() <= tol0


@pytest.mark.parametrize("name", ["qkv", "o", "gateup", "down"])
def test_qwen2_7b_block_layers(name):
    check_w4a8_layer("qwen2-7b", name, 1024, {"qkv": 11, "o": 12, "gateup": 13, "down": 14}[name])


@pytest.mark.parametrize("name", ["qkv", "o", "gateup", "down"])
def test_qwen2_1p5b_block_layers(name):
    check_w4a8_layer("qwen2-1.5b", name, 512, {"qkv": 21, "o": 22, "gateup": 23, "down": 24}[name])


def test_qwen2_7b_lm_head_through_the_prefill_gemm():
    """The LM head (N = 152064) at M = 1024 through mnnq_linear_prefill, as `bench.py --lm-head-prefill`
    times it: one output per 16 x 16 block against the oracle, for the fp6 GEMM."""
    N, K = synth.MODELS["qwen2-7b"]["lm_head"]
    M = 1024
    note("full-size lm_head prefill", M, N, K)
    W = synth.weights(N, K, synth.layer_seed("qwen2-7b", 0, "lm_head"))
    x = synth.activations(M, K, 32, outliers=True)
    q, s, z = oracle.quant_weights(W)
    xq_o, sx_o, _ = oracle.quant_act(x)
    packed = B.mnnq_pack_weights(dev(W), mode=MODE_PLANE)
    del W
    ws = torch.empty(B.mnnq_workspace_size(M, N, K, 64, MODE_PLANE), dtype=torch.uint8, device="cuda:0")
    y = B.mnnq_linear_prefill(packed, N, K, dev(xq_o), dev(sx_o), mode=MODE_PLANE, workspace=ws)
    rng = np.random.default_rng(33)
    ms, ns = stratified_pairs(M, N, rng)
    got = y[torch.from_numpy(ms).to("cuda:0"), torch.from_numpy(ns).to("cuda:0")].cpu().numpy()
    ymax = float(y.abs().max())
    assert bool(torch.isfinite(y).all())
    del y
    _, y_s = oracle.linear_w4a8_sampled(xq_o, sx_o, q, s, z, ms, ns, want_acc=False)
    assert np.abs(got - y_s).max() <= 1e-5 * ymax
    # the int8 GEMM on the same packed buffer (no workspace), on a thinner sample
    y8 = B.mnnq_linear_prefill(packed, N, K, dev(xq_o), dev(sx_o), mode=MODE_PLANE)
    got8 = y8[torch.from_numpy(ms[::8]).to("cuda:0"), torch.from_numpy(ns[::8]).to("cuda:0")].cpu().numpy()
    assert np.abs(got8 - y_s[::8]).max() <= 1e-5 * ymax


def test_qwen2_7b_lm_head_decode():
    N, K = synth.MODELS["qwen2-7b"]["lm_head"]
    note("full-size lm_head decode", N, K)
    W = synth.weights(N, K, synth.layer_seed("qwen2-7b", 0, "lm_head"))
    x = synth.activations(1, K, 31)
    q, s, z = oracle.quant_weights(W)
    xq_o, sx_o, _ = oracle.quant_act(x)
    _, y_o = oracle.linear_w4a8(xq_o, sx_o, q, s, z, want_acc=False)
    packed = B.mnnq_pack_weights(dev(W))
    del W
    xq, sx, _ = B.mnnq_quant_act(dev(x), want_xsum=False)
    y = B.mnnq_linear_decode(packed, N, K, xq, sx).cpu().numpy()
    assert np.abs(y - y_o[0]).max() <= 1e-5 * np.abs(y_o).max()
    rng = np.random.default_rng(5)
    pn = rng.integers(0, N, 4096)
    acc = B.mnnq_linear_acc_debug(packed, N, K, xq, False).cpu().numpy()
    acc_s, _ = oracle.linear_w4a8_sampled(xq_o, sx_o, q, s, z, np.zeros_like(pn), pn)
    assert np.array_equal(acc[0, pn], acc_s)


@pytest.mark.parametrize("name", ["qkv", "o", "gateup", "down"])
def test_llama3_8b_w4a16_and_w4a8_side_by_side(name):
    model, M = "llama3-8b", 2048
    W = fused_weights(model, name)
    N, K = W.shape
    note("full-size W4A16 + W4A8", model, name, "M", M, "N", N, "K", K)
    x = synth.activations(M, K, 41, outliers=False)
    x16 = x.astype(np.float16)
    q, s, z = oracle.quant_weights(W)
    packed = B.mnnq_pack_weights(dev(W), mode=MODE_PLANE)
    del W
    rng = np.random.default_rng(42)
    ms, ns = stratified_pairs(M, N, rng, tile=32)
    # W4A16
    y16 = B.mnnq_linear_prefill_f16(packed, N, K, dev(x16), mode=MODE_PLANE).cpu().numpy()
    y16_s = oracle.linear_w4a16_sampled(x16, q, s, z, ms, ns)
    assert np.abs(y16[ms, ns] - y16_s).max() <= 1e-3 * np.abs(y16).max()
    y16_0 = oracle.linear_w4a16(x16[:1], q, s, z)
    yd = B.mnnq_linear_decode_f16(packed, N, K, dev(x16[0]), mode=MODE_PLANE).cpu().numpy()
    assert np.abs(yd - y16_0[0]).max() <= 1e-3 * np.abs(y16_0).max()
    # W4A8 on the same activations
    xq_o, sx_o, _ = oracle.quant_act(x)
    xq, sx, _ = B.mnnq_quant_act(dev(x), want_xsum=False)
    assert np.array_equal(xq.cpu().numpy(), xq_o)
    ws = torch.empty(B.mnnq_workspace_size(M, N, K, 64, MODE_PLANE), dtype=torch.uint8, device="cuda:0")
    y8 = B.mnnq_linear_prefill(packed, N, K, xq, sx, mode=MODE_PLANE, workspace=ws).cpu().numpy()    # the fp6 GEMM
    _, y8_s = oracle.linear_w4a8_sampled(xq_o, sx_o, q, s, z, ms, ns, want_acc=False)
    assert np.abs(y8[ms, ns] - y8_s).max() <= 1e-5 * np.abs(y8).max()
    y8i = B.mnnq_linear_prefill(packed, N, K, xq, sx, mode=MODE_PLANE).cpu().numpy()                  # the int8 GEMM
    assert np.abs(y8i[ms, ns] - y8_s).max() <= 1e-5 * np.abs(y8).max()
    del y8i, ws
    # the two variants see the same weights: they differ only by the activation rounding
    assert np.abs(y8[ms, ns] - y16[ms, ns]).max() < 0.05 * np.abs(y16).max()


@pytest.mark.parametrize("name", ["gateup", "down"])
@pytest.mark.parametrize("form", ["minfloat", "int8"])
def test_qwen2_7b_other_weight_forms(form, name):
    """Float-minimum int4 and int8 weights at the sizes and launch plans `bench.py --weight-mode` times:
    sampled prefill outputs (M = 1024) and the first row through both single-token calls."""
    model, M, seed = "qwen2-7b", 1024, 77
    W = fused_weights(model, name)
    N, K = W.shape
    note("full-size", form, model, name, "M", M, "N", N, "K", K)
    x = synth.activations(M, K, seed, outliers=True)
    if form == "minfloat":
        mode, quant, sampled = B.MODE_W4_MIN_FLOAT, oracle.quant_weights_minf, oracle.linear_w4a8_minf_sampled
    else:
        mode, quant, sampled = B.MODE_W8_MIN_FLOAT, oracle.quant_weights8, oracle.linear_w8a8_sampled
    q, s, mn = quant(W)
    xq_o, sx_o, _ = oracle.quant_act(x)
    packed = B.mnnq_pack_weights(dev(W), mode=mode)
    del W
    xq, sx = dev(xq_o), dev(sx_o)
    y = B.mnnq_linear_prefill(packed, N, K, xq, sx, mode=mode).cpu().numpy()
    rng = np.random.default_rng(seed)
    ms = np.concatenate([rng.integers(0, M, 4096), [0, 0, M - 1, M - 1]])
    ns = np.concatenate([rng.integers(0, N, 4096), [0, N - 1, 0, N - 1]])
    _, y_s = sampled(xq_o, sx_o, q, s, mn, ms, ns, want_acc=False)
    ymax = np.abs(y).max()
    assert np.isfinite(y).all()
    assert np.abs(y[ms, ns] - y_s).max() <= 1e-5 * ymax
    # the first token in full through the GEMV and the fused GEMV
    n_all = np.arange(N)
    _, y0 = sampled(xq_o, sx_o, q, s, mn, np.zeros(N, dtype=np.int64), n_all, want_acc=False)
    tol0 = 1e-5 * np.abs(y0).max()
    yd = B.mnnq_linear_decode(packed, N, K, xq[0].contiguous(), sx[:1].contiguous(), mode=mode).cpu().numpy()
    assert np.abs(yd - y0).max() <= tol0
    yf = B.mnnq_linear_decode_fused(packed, N, K, dev(x[0]), mode=mode).cpu().numpy()
    assert np.abs(yf - y0).max() <= tol0
    assert np.abs(y[0] - y0).max() <= tol0


def test_batch_beyond_one_launch_is_processed_in_slabs():
    """(M + 256) * N * 4 bytes of output beyond 2 GiB: the call runs slab by slab (32512 rows here);
    sampled outputs, with rows on both sides of the slab boundary and the last row."""
    M, N, K = 40000, 16384, 64
    note("slabs", M, N, K)
    W = synth.weights(N, K, 91)
    x = synth.activations(M, K, 92, outliers=False)
    q, s, z = oracle.quant_weights(W)
    xq_o, sx_o, _ = oracle.quant_act(x)
    packed = B.mnnq_pack_weights(dev(W))
    bias = synth.weights(1, N, 93)[0] * 10
    y = B.mnnq_linear_prefill(packed, N, K, dev(xq_o), dev(sx_o), bias=dev(bias))
    rng = np.random.default_rng(94)
    ms = np.concatenate([rng.integers(0, M, 4096), [0, 32511, 32511, 32512, 32512, M - 1, M - 1]])
    ns = np.concatenate([rng.integers(0, N, 4096), [0, 0, N - 1, 0, N - 1, 0, N - 1]])
    got = y[torch.from_numpy(ms).to("cuda:0"), torch.from_numpy(ns).to("cuda:0")].cpu().numpy()
    _, y_s = oracle.linear_w4a8_sampled(xq_o, sx_o, q, s, z, ms, ns, bias=bias, want_acc=False)
    assert np.abs(got - y_s).max() <= 1e-5 * np.abs(y_s).max()
    del y
    # the fused call and the fp16-activation call take the same route
    ws = torch.empty(B.mnnq_workspace_size(M, N, K), dtype=torch.uint8, device="cuda:0")
    yf = B.mnnq_linear_prefill_fused(packed, N, K, dev(x), bias=dev(bias), workspace=ws)
    got = yf[torch.from_numpy(ms).to("cuda:0"), torch.from_numpy(ns).to("cuda:0")].cpu().numpy()
    assert np.abs(got - y_s).max() <= 1e-5 * np.abs(y_s).max()
    del yf, ws
    x16 = x.astype(np.float16)
    y16 = B.mnnq_linear_prefill_f16(packed, N, K, dev(x16), bias=dev(bias))
    got = y16[torch.from_numpy(ms).to("cuda:0"), torch.from_numpy(ns).to("cuda:0")].cpu().numpy()
    y_s16 = oracle.linear_w4a16_sampled(x16, q, s, z, ms, ns, bias=bias)
    assert np.abs(got - y_s16).max() <= 1e-3 * np.abs(y_s16).max()
