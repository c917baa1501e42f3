"""GPU parity of the binary16-output calls (Section 4.2: the GPU path runs in fp16) through the
C-ABI.  The sums are those of the fp32-output calls, rounded once to nearest even: the result must
equal the fp32 call's output converted to half bit for bit, and lie within the linear layer's
tolerance plus half a binary16 unit (2^-11 relative, 2^-25 absolute in the subnormal range) of the
oracle."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2506_10443_amd import binding as B, synth

pytestmark = pytest.mark.gpu
TOL_A8, TOL_A16 = 1e-5, 1e-3


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.cpu().numpy()


def note(*a):
    print(*a, flush=True)


def close_to_oracle(y16, y_o, tol):
    err = np.abs(y16.astype(np.float64) - y_o.astype(np.float64))
    bound = tol * np.abs(y_o).max() + 2.0 ** -11 * np.abs(y_o) * 1.001 + 2.0 ** -25
    assert (err <= bound).all(), float((err - bound).max())


SHAPES = [(1, 16, 64), (4, 48, 192), (16, 272, 1536), (33, 272, 640), (130, 144, 1536), (300, 400, 1024),
          (513, 1040, 448),
          (100, 144, 8192)]   # few tiles, long rows: the fp32 call splits K over two workgroups, this one must not


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_w4a8_out16(M, N, K):
    note("out16 w4a8", M, N, K)
    W = synth.weights(N, K, 300 + M + N + K)
    x = synth.activations(M, K, 301 + M + N + K, outliers=True)
    q, s, z = oracle.quant_weights(W)
    xq, sx, _ = oracle.quant_act(x)
    bias = synth.weights(1, N, 5)[0] * 10
    y_o = oracle.linear_w4a8(xq, sx, q, s, z, bias=bias, want_acc=False)[1]
    packed = B.mnnq_pack_weights(dev(W))
    xqd, sxd, bd = dev(xq), dev(sx), dev(bias)
    for cfg in ("", "b1", "s1", "b1k", "s1k", "w1", "v1k", "w1k", "t1", "t1q", "n1", "n1q"):
        if cfg:
            B.mnnq_debug_set("MNNQ_PREFILL_TILE", cfg)
            B.mnnq_debug_set("MNNQ_NO_SKINNY", "1")
        try:
            y32 = B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd)
            y16 = B.mnnq_linear_prefill_o16(packed, N, K, xqd, sxd, bias=bd)
        finally:
            B.mnnq_debug_set("MNNQ_PREFILL_TILE", None)
            B.mnnq_debug_set("MNNQ_NO_SKINNY", None)
        assert y16.dtype == torch.float16
        if K < 8192 or cfg:       # same tile plan and summation order as the fp32 call
            assert torch.equal(y16, y32.to(torch.float16)), cfg
        else:                     # the fp32 call adds two K halves in the output array
            assert (y16.float() - y32).abs().max().item() <= 2.0 ** -10 * y32.abs().max().item()
        close_to_oracle(host(y16), y_o, TOL_A8)
    y32 = B.mnnq_linear_decode(packed, N, K, xqd[0].contiguous(), sxd[:1].contiguous(), bias=bd)
    y16 = B.mnnq_linear_decode_o16(packed, N, K, xqd[0].contiguous(), sxd[:1].contiguous(), bias=bd)
    assert torch.equal(y16, y32.to(torch.float16))
    close_to_oracle(host(y16), y_o[0], TOL_A8)
    if M <= 16 and K <= 4096:
        # both few-token kernels (the persistent one is normally reserved for large layers)
        for staged in ("0", "1"):
            B.mnnq_debug_set("MNNQ_SKINNY_STAGED", staged)
            try:
                y32 = B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd)
                y16 = B.mnnq_linear_prefill_o16(packed, N, K, xqd, sxd, bias=bd)
            finally:
                B.mnnq_debug_set("MNNQ_SKINNY_STAGED", None)
            assert torch.equal(y16, y32.to(torch.float16)), staged
            close_to_oracle(host(y16), y_o, TOL_A8)


@pytest.mark.parametrize("M,N,K", [(1, 16, 64), (9, 48, 192), (130, 272, 1536), (300, 272, 448)])
def test_w4a16_out16(M, N, K):
    note("out16 w4a16", M, N, K)
    W = synth.weights(N, K, 320 + M + N + K)
    x16 = synth.activations_f16(M, K, 321 + M + N + K)
    q, s, z = oracle.quant_weights(W)
    bias = synth.weights(1, N, 6)[0] * 10
    y_o = oracle.linear_w4a16(x16, q, s, z, bias=bias)
    packed = B.mnnq_pack_weights(dev(W))
    xd, bd = dev(x16), dev(bias)
    for cfg in ("", "s1", "b1", "s1k", "b1k"):       # tile and K parts of the fp16 GEMM
        if cfg:
            B.mnnq_debug_set("MNNQ_PREFILL_TILE", cfg)
        try:
            y32 = B.mnnq_linear_prefill_f16(packed, N, K, xd, bias=bd)
            y16 = B.mnnq_linear_prefill_f16_o16(packed, N, K, xd, bias=bd)
        finally:
            B.mnnq_debug_set("MNNQ_PREFILL_TILE", None)
        assert torch.equal(y16, y32.to(torch.float16)), cfg
        close_to_oracle(host(y16), y_o, TOL_A16)
    y32 = B.mnnq_linear_decode_f16(packed, N, K, xd[0].contiguous(), bias=bd)
    y16 = B.mnnq_linear_decode_f16_o16(packed, N, K, xd[0].contiguous(), bias=bd)
    assert torch.equal(y16, y32.to(torch.float16))
    close_to_oracle(host(y16), y_o[0], TOL_A16)


def test_other_weight_forms_and_neighbours_untouched():
    # float-minimum and 8-bit forms go through the same store; the halves must land densely: the
    # elements around the output array stay as they were
    M, N, K = 70, 48, 256
    x = synth.activations(M, K, 341, outliers=True)
    xq, sx, _ = oracle.quant_act(x)
    W = synth.weights(N, K, 340)
    for mode, quant, lin in ((B.MODE_W4_MIN_FLOAT, oracle.quant_weights_minf, oracle.linear_w4a8_minf),
                             (B.MODE_W8_MIN_FLOAT, oracle.quant_weights8, oracle.linear_w8a8)):
        q, s, mn = quant(W)
        y_o = lin(xq, sx, q, s, mn, want_acc=False)[1]
        packed = B.mnnq_pack_weights(dev(W), mode=mode)
        buf = torch.full((M * N + 16,), 7.0, dtype=torch.float16, device="cuda:0")
        out = buf[8:8 + M * N].view(M, N)          # 16-byte aligned
        B.mnnq_linear_prefill_o16(packed, N, K, dev(xq), dev(sx), out=out, mode=mode)
        assert (host(buf[:8]) == 7).all() and (host(buf[-8:]) == 7).all()
        close_to_oracle(host(out), y_o, TOL_A8)


def test_values_beyond_half_range_become_infinite():
    N, K = 16, 64
    W = np.full((N, K), 0.5, np.float32)
    W[:, 0] = -0.5
    x = np.full((1, K), 3000.0, np.float32)
    packed = B.mnnq_pack_weights(dev(W))
    xq, sx, _ = B.mnnq_quant_act(dev(x), want_xsum=False)
    y32 = host(B.mnnq_linear_decode(packed, N, K, xq[0], sx))
    y16 = host(B.mnnq_linear_decode_o16(packed, N, K, xq[0], sx))
    assert (y32 > 65504 * 1.01).all() and np.isinf(y16).all()


@pytest.mark.parametrize("M,N,K", [(1, 48, 192), (1, 272, 1536), (7, 144, 640), (130, 144, 1536), (300, 400, 1024)])
def test_fused_calls_out16(M, N, K):
    """fp32 activations in, binary16 out: the fused calls with the suffix give the fp32 fused call's
    result converted to half, with and without a workspace for the single-token call."""
    note("out16 fused", M, N, K)
    W = synth.weights(N, K, 340 + M + N + K)
    x = synth.activations(M, K, 341 + M + N + K, outliers=True)
    q, s, z = oracle.quant_weights(W)
    xq, sx, _ = oracle.quant_act(x)
    bias = synth.weights(1, N, 6)[0] * 10
    y_o = oracle.linear_w4a8(xq, sx, q, s, z, bias=bias, want_acc=False)[1]
    packed = B.mnnq_pack_weights(dev(W))
    xd, bd = dev(x), dev(bias)
    y32 = B.mnnq_linear_prefill_fused(packed, N, K, xd, bias=bd)
    y16 = B.mnnq_linear_prefill_fused_o16(packed, N, K, xd, bias=bd)
    assert y16.dtype == torch.float16 and torch.equal(y16, y32.to(torch.float16))
    close_to_oracle(host(y16), y_o, TOL_A8)
    ws = torch.empty(B.mnnq_workspace_size(1, N, K), dtype=torch.uint8, device="cuda:0")
    for workspace, two_kernel in ((None, None), (ws, "0")):
        if two_kernel is not None:
            B.mnnq_debug_set("MNNQ_FUSED_TWO_KERNEL_MIB", two_kernel)   # quantizer as a kernel of its own
        try:
            r32 = B.mnnq_linear_decode_fused(packed, N, K, xd[0].contiguous(), bias=bd, workspace=workspace)
            r16 = B.mnnq_linear_decode_fused_o16(packed, N, K, xd[0].contiguous(), bias=bd, workspace=workspace)
        finally:
            B.mnnq_debug_set("MNNQ_FUSED_TWO_KERNEL_MIB", None)
        assert r16.dtype == torch.float16 and torch.equal(r16, r32.to(torch.float16))
        close_to_oracle(host(r16), y_o[0], TOL_A8)
