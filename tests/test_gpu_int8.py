"""GPU parity of the int8 weight path (mode MNNQ_W8_MIN_FLOAT: Eq. 1 with clip range 0..255 and a
float group minimum, stored as two 4-bit planes on the int4 kernels) against the oracle's O9 / O10,
through the C-ABI.  Codes, steps and minima bit-exact; integer sums bit-exact; y within 1e-5 * max|y|."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2506_10443_amd import binding as B, synth

pytestmark = pytest.mark.gpu
W8 = B.MODE_W8_MIN_FLOAT
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
    W[1, :64] = np.abs(W[1, :64]) + 0.5   # group far from zero
    return W


@pytest.mark.parametrize("N,K", [(16, 128), (48, 384), (272, 1536), (1024, 4096)])
def test_pack_unpack_import_bit_exact(N, K):
    note("int8 pack", N, K)
    W = _weights(N, K, 900 + N + K)
    q, s, mn = oracle.quant_weights8(W)
    assert q.max() == 255
    packed = B.mnnq_pack_weights(dev(W), mode=W8)
    assert packed.numel() == N * K + 16 * N * (K // 64)       # two nibble planes, each with fp32 step and minimum
    assert packed.numel() == B.mnnq_packed_size(N, K, 64, W8)
    q2, s2, m2 = B.mnnq_unpack_weights(packed, N, K, mode=W8)
    assert np.array_equal(host(q2), q)
    assert np.array_equal(host(s2).view(np.uint32), s.view(np.uint32))
    assert np.array_equal(host(m2).view(np.uint32), mn.view(np.uint32))
    assert torch.equal(B.mnnq_pack_from_quantized(dev(q), dev(s), dev(mn), mode=W8), packed)
    with pytest.raises(B.MnnqError):
        B.mnnq_pack_weights(dev(W[:, :64].copy()), mode=W8)    # K must be a multiple of 128


SHAPES = [(1, 16, 128), (7, 48, 384), (16, 144, 9472), (33, 272, 640), (130, 144, 1536), (300, 400, 1024),
          (64, 1024, 4096), (129, 144, 8192), (513, 1040, 896)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_linear_matches_oracle(M, N, K):
    note("int8 linear", M, N, K)
    W = _weights(N, K, 910 + M + N + K)
    x = synth.activations(M, K, 911 + M + N + K, outliers=True)
    q, s, mn = oracle.quant_weights8(W)
    xq, sx, _ = oracle.quant_act(x)
    bias = synth.weights(1, N, 9)[0] * 10
    acc_o, y_o = oracle.linear_w8a8(xq, sx, q, s, mn, bias=bias)
    tol = TOL * np.abs(y_o).max()
    G = K // 64
    packed = B.mnnq_pack_weights(dev(W), mode=W8)
    xqd, sxd, bd = dev(xq), dev(sx), dev(bias)
    for use_prefill in (True, False):
        planes = host(B.mnnq_linear_acc_debug(packed, N, K, xqd, use_prefill, mode=W8)).astype(np.int64)
        assert np.array_equal(16 * planes[:, :, :G] + planes[:, :, G:], acc_o)
    y = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd, mode=W8))
    assert np.abs(y - y_o).max() <= tol, (np.abs(y - y_o).max(), tol)
    # every tile plan, with both nibble planes merged into one matrix instruction per group (the
    # default) and with one per plane; "2" splits K over two workgroups (long rows only)
    B.mnnq_debug_set("MNNQ_NO_SKINNY", "1")
    try:
        for planes in ("0", "1"):
            for cfg in ("b1", "s1", "b1k", "s1k", "s2", "s2k", "v1k", "v2k"):
                B.mnnq_debug_set("MNNQ_PREFILL_TILE", cfg)
                B.mnnq_debug_set("MNNQ_W8_PLANES", planes)
                try:
                    y2 = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd, mode=W8))
                finally:
                    B.mnnq_debug_set("MNNQ_PREFILL_TILE", None)
                    B.mnnq_debug_set("MNNQ_W8_PLANES", None)
                assert np.abs(y2 - y_o).max() <= tol, (planes, cfg)
    finally:
        B.mnnq_debug_set("MNNQ_NO_SKINNY", None)
    if M <= 16:
        for staged in ("0", "1"):
            B.mnnq_debug_set("MNNQ_SKINNY_STAGED", staged)
            try:
                y3 = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd, mode=W8))
            finally:
                B.mnnq_debug_set("MNNQ_SKINNY_STAGED", None)
            assert np.abs(y3 - y_o).max() <= tol, staged
    for m in sorted({0, M - 1}):
        y0 = host(B.mnnq_linear_decode(packed, N, K, xqd[m].contiguous(), sxd[m:m + 1].contiguous(), bias=bd, mode=W8))
        assert np.abs(y0 - y_o[m]).max() <= tol, m
        yf = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x[m]), bias=bd, mode=W8))
        assert np.abs(yf - y_o[m]).max() <= tol, m


def test_full_size_lm_head_decode():
    # The layer the paper singles out for int8: the LM head.
    N, K = synth.MODELS["qwen2-7b"]["lm_head"]
    note("int8 lm_head", N, K)
    W = synth.weights(N, K, synth.layer_seed("qwen2-7b", 0, "lm_head"))
    x = synth.activations(1, K, 61)
    q, s, mn = oracle.quant_weights8(W)
    xq_o, sx_o, _ = oracle.quant_act(x)
    _, y_o = oracle.linear_w8a8(xq_o, sx_o, q, s, mn, want_acc=False)
    packed = B.mnnq_pack_weights(dev(W), mode=W8)
    del W
    q2, s2, m2 = B.mnnq_unpack_weights(packed, N, K, mode=W8)
    assert np.array_equal(host(q2), q) and np.array_equal(host(m2).view(np.uint32), mn.view(np.uint32))
    assert np.array_equal(host(s2).view(np.uint32), s.view(np.uint32))
    del q2, s2, m2
    y = host(B.mnnq_linear_decode(packed, N, K, dev(xq_o[0]), dev(sx_o), mode=W8))
    assert np.abs(y - y_o[0]).max() <= TOL * np.abs(y_o).max()
    ws = torch.empty(B.mnnq_workspace_size(1, N, K), dtype=torch.uint8, device="cuda:0")
    yf = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x[0]), workspace=ws, mode=W8))
    assert np.array_equal(yf, y)
    # 8-bit weights track the fp32 layer 16 times closer than 4-bit ones
    ref = (xq_o.astype(np.float64) * sx_o[:, None]) @ synth.weights(N, K, synth.layer_seed("qwen2-7b", 0, "lm_head")).astype(np.float64).T
    e8 = np.abs(y - ref[0]).max()
    p4 = B.mnnq_pack_weights(dev(synth.weights(N, K, synth.layer_seed("qwen2-7b", 0, "lm_head"))), mode=B.MODE_W4_MIN_FLOAT)
    y4 = host(B.mnnq_linear_decode(p4, N, K, dev(xq_o[0]), dev(sx_o), mode=B.MODE_W4_MIN_FLOAT))
    e4 = np.abs(y4 - ref[0]).max()
    assert e8 < e4 / 8
