"""GPU parity of the Eq.-1-literal weight form (float group minimum, no integer zero point)
against the oracle's O6..O8, through the C-ABI.  Codes, steps and minima bit-exact; the
integer sums A[m,n,g] bit-exact; y within 1e-5 * max|y|."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2506_10443_amd import binding as B, synth

pytestmark = pytest.mark.gpu
MINF = B.MODE_W4_MIN_FLOAT
TOL = 1e-5


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.cpu().numpy()


def note(*a):
    print(*a, flush=True)


def _weights(N, K, seed):
    W = synth.weights(N, K, seed)
    W[0, :64] = 0.25                      # constant group
    W[1, :64] = np.abs(W[1, :64]) + 0.5   # group far from zero: the integer zero point form would widen it
    W[2, :64] = 0.0
    return W


@pytest.mark.parametrize("N,K", [(16, 64), (48, 192), (272, 1536), (1024, 4096)])
def test_pack_unpack_import_bit_exact(N, K):
    note("minfloat pack", N, K)
    W = _weights(N, K, 700 + N + K)
    q, s, mn = oracle.quant_weights_minf(W)
    packed = B.mnnq_pack_weights(dev(W), mode=MINF)
    Gp = (K // 64 + 1) // 2 * 2                       # an odd number of groups gets a padding group
    assert packed.numel() == N * Gp * 32 + 8 * N * Gp    # codes + fp32 step + fp32 minimum
    q2, s2, m2 = B.mnnq_unpack_weights(packed, N, K, mode=MINF)
    assert np.array_equal(host(q2), q)
    assert np.array_equal(host(s2).view(np.uint32), s.view(np.uint32))
    assert np.array_equal(host(m2).view(np.uint32), mn.view(np.uint32))
    # import of the oracle's arrays gives the same bytes
    assert torch.equal(B.mnnq_pack_from_quantized(dev(q), dev(s), dev(mn), mode=MINF), packed)


SHAPES = [(1, 16, 64), (7, 48, 192), (16, 144, 18944), (33, 272, 448), (130, 144, 1536), (300, 400, 1024),
          (64, 1024, 4096)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_linear_matches_oracle(M, N, K):
    note("minfloat linear", M, N, K)
    W = _weights(N, K, 710 + M + N + K)
    x = synth.activations(M, K, 711 + M + N + K, outliers=True)
    q, s, mn = oracle.quant_weights_minf(W)
    xq, sx, _ = oracle.quant_act(x)
    bias = synth.weights(1, N, 9)[0] * 10
    acc_o, y_o = oracle.linear_w4a8_minf(xq, sx, q, s, mn, bias=bias)
    tol = TOL * np.abs(y_o).max()
    packed = B.mnnq_pack_weights(dev(W), mode=MINF)
    xqd, sxd, bd = dev(xq), dev(sx), dev(bias)
    # integer sums from both kernels' inner loops
    assert np.array_equal(host(B.mnnq_linear_acc_debug(packed, N, K, xqd, True, mode=MINF)), acc_o)
    assert np.array_equal(host(B.mnnq_linear_acc_debug(packed, N, K, xqd, False, mode=MINF)), acc_o)
    # prefill, every tile / split choice
    y = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd, mode=MINF))
    assert np.abs(y - y_o).max() <= tol, (np.abs(y - y_o).max(), tol)
    B.mnnq_debug_set("MNNQ_NO_SKINNY", "1")     # M <= 16 would otherwise bypass the tiled kernel
    try:
        for cfg in ("b1", "s1", "b1k", "s1k", "s2", "b2k", "w1", "w2", "v1k", "v2k", "w1k", "t1", "t1k", "t2q", "n1", "n2q"):
            B.mnnq_debug_set("MNNQ_PREFILL_TILE", cfg)
            try:
                y2 = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd, mode=MINF))
            finally:
                B.mnnq_debug_set("MNNQ_PREFILL_TILE", None)
            assert np.abs(y2 - y_o).max() <= tol, cfg
    finally:
        B.mnnq_debug_set("MNNQ_NO_SKINNY", None)
    # decode of a few rows, every K split, and the fused quantizer
    for m in sorted({0, M // 2, M - 1}):
        for ks in ("", "1", "2", "4", "8", "16"):
            if ks:
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", ks)
            try:
                y0 = host(B.mnnq_linear_decode(packed, N, K, xqd[m].contiguous(), sxd[m:m + 1].contiguous(),
                                               bias=bd, mode=MINF))
            except B.MnnqError as e:
                # a forced split that leaves a wave more of the row than its LDS slice holds is refused
                assert ks and e.status == -3 and K > 8192, (ks, e)
                continue
            finally:
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", None)
            assert np.abs(y0 - y_o[m]).max() <= tol, (m, ks)
        yf = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x[m]), bias=bd, mode=MINF))
        assert np.abs(yf - y_o[m]).max() <= tol, m


def test_all_positive_weights_and_extreme_codes():
    # Weights in [1, 2): every code 0..15 occurs, the minimum term dominates the sum.
    N, K, M = 32, 256, 48
    rng = np.random.default_rng(5)
    W = (1.0 + rng.integers(0, 16, (N, K)) / 16.0).astype(np.float32)
    W[:, ::64] = 1.0
    W[:, 1::64] = 1.9375
    x = np.where(rng.random((M, K)) < 0.5, -1.0, 1.0).astype(np.float32)      # xq = +-127
    q, s, mn = oracle.quant_weights_minf(W)
    assert q.min() == 0 and q.max() == 15 and (mn == 1.0).all()
    xq, sx, _ = oracle.quant_act(x)
    acc_o, y_o = oracle.linear_w4a8_minf(xq, sx, q, s, mn)
    packed = B.mnnq_pack_weights(dev(W), mode=MINF)
    assert np.array_equal(host(B.mnnq_linear_acc_debug(packed, N, K, dev(xq), True, mode=MINF)), acc_o)
    y = host(B.mnnq_linear_prefill(packed, N, K, dev(xq), dev(sx), mode=MINF))
    assert np.abs(y - y_o).max() <= TOL * np.abs(y_o).max()
    y0 = host(B.mnnq_linear_decode(packed, N, K, dev(xq[0]), dev(sx[:1]), mode=MINF))
    assert np.abs(y0 - y_o[0]).max() <= TOL * np.abs(y_o).max()
    # the result is the product with the dequantized weights, which here are W itself
    assert np.array_equal(oracle.dequant_minf(q, s, mn), W)
    ref = (xq.astype(np.float64) * sx[:, None]) @ W.astype(np.float64).T
    assert np.abs(y - ref).max() <= TOL * np.abs(ref).max()


def test_full_size_gateup_sampled():
    model, M = "qwen2-7b", 1024
    parts = [synth.weights(*synth.MODELS[model]["layers"][p], synth.layer_seed(model, 0, p))
             for p in synth.fused_parts("gateup")]
    W = np.concatenate(parts)
    N, K = W.shape
    note("minfloat full size", N, K)
    x = synth.activations(M, K, 55, outliers=True)
    q, s, mn = oracle.quant_weights_minf(W)
    xq_o, sx_o, _ = oracle.quant_act(x)
    packed = B.mnnq_pack_weights(dev(W), mode=MINF)
    del W
    q2, s2, m2 = B.mnnq_unpack_weights(packed, N, K, mode=MINF)
    assert np.array_equal(host(q2), q) and np.array_equal(host(m2).view(np.uint32), mn.view(np.uint32))
    assert np.array_equal(host(s2).view(np.uint32), s.view(np.uint32))
    del q2, s2, m2
    y = host(B.mnnq_linear_prefill(packed, N, K, dev(xq_o), dev(sx_o), mode=MINF))
    rng = np.random.default_rng(56)
    ms = np.concatenate([rng.integers(0, M, 4096), [0, 0, M - 1, M - 1]])
    ns = np.concatenate([rng.integers(0, N, 4096), [0, N - 1, 0, N - 1]])
    _, y_s = oracle.linear_w4a8_minf_sampled(xq_o, sx_o, q, s, mn, ms, ns, want_acc=False)
    assert np.abs(y[ms, ns] - y_s).max() <= TOL * np.abs(y).max()
    _, y0 = oracle.linear_w4a8_minf(xq_o[:1], sx_o[:1], q, s, mn, want_acc=False)
    yd = host(B.mnnq_linear_decode(packed, N, K, dev(xq_o[0]), dev(sx_o[:1]), mode=MINF))
    assert np.abs(yd - y0[0]).max() <= TOL * np.abs(y0).max()
    ws = torch.empty(B.mnnq_workspace_size(1, N, K), dtype=torch.uint8, device="cuda:0")
    yf = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x[0]), workspace=ws, mode=MINF))
    assert np.array_equal(yf, yd)
