"""GPU parity of fp16 activations on the float-minimum weight forms (MNNQ_W4_MIN_FLOAT: Eq. 1 as
printed; MNNQ_W8_MIN_FLOAT: 8-bit codes, i.e. W8A16) against the oracle's O11, through the C-ABI.
y within 1e-3 * max|y| (the W4A16 bar); with integer activations the fp16 kernels must reproduce
the int8 kernels' result to fp32 rounding."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2506_10443_amd import binding as B, synth

pytestmark = pytest.mark.gpu
TOL_A16 = 1e-3
MODES = [(B.MODE_W4_MIN_FLOAT, oracle.quant_weights_minf), (B.MODE_W8_MIN_FLOAT, oracle.quant_weights8)]


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.cpu().numpy()


def note(*a):
    print(*a, flush=True)


SHAPES = [(1, 16, 128), (9, 48, 384), (130, 272, 1536), (64, 1024, 4096), (300, 272, 640), (700, 144, 1664),
          (40, 32, 192)]


@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("which", [0, 1])
def test_a16_matches_oracle(M, N, K, which):
    mode, quant = MODES[which]
    if mode == B.MODE_W8_MIN_FLOAT and K % 128:
        pytest.skip("8-bit codes need whole chunks per plane")
    note("a16 minfloat", mode, M, N, K)
    W = synth.weights(N, K, 700 + M + N + K)
    W[0, :64] = 0.25                      # constant group
    W[1, :64] = np.abs(W[1, :64]) + 0.5   # group far from zero: a large minimum
    x16 = synth.activations_f16(M, K, 701 + M + N + K)
    q, s, mn = quant(W)
    bias = synth.weights(1, N, 6)[0] * 10
    y_o = oracle.linear_a16_minf(x16, q, s, mn, bias=bias)
    packed = B.mnnq_pack_weights(dev(W), mode=mode)
    xd = dev(x16)
    tol = TOL_A16 * np.abs(y_o).max()
    for tile in ("", "b", "s", "b1k", "s1k"):
        if tile:
            B.mnnq_debug_set("MNNQ_PREFILL_TILE", tile)
        try:
            y = host(B.mnnq_linear_prefill_f16(packed, N, K, xd, bias=dev(bias), mode=mode))
        finally:
            B.mnnq_debug_set("MNNQ_PREFILL_TILE", None)
        assert np.abs(y - y_o).max() <= tol, (tile, np.abs(y - y_o).max(), tol)
    for ks in ("", "1", "2", "4", "8", "16"):
        if ks:
            B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", ks)
        try:
            y0 = host(B.mnnq_linear_decode_f16(packed, N, K, xd[0].contiguous(), bias=dev(bias), mode=mode))
        except B.MnnqError as e:
            # a forced split can ask for more LDS than a workgroup has; the library's own choice never does
            assert ks and e.status == -3, (ks, e)
            continue
        finally:
            B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", None)
        assert np.abs(y0 - y_o[0]).max() <= TOL_A16 * np.abs(y_o[0]).max(), ks


@pytest.mark.parametrize("which", [0, 1])
def test_integer_activations_reproduce_the_int8_kernels(which):
    # int8 codes are exact in fp16 and the group sums are integers below 2^24, so only the fp32
    # epilogue order differs between the two routes.
    mode, _ = MODES[which]
    M, N, K = 200, 272, 1536
    W = synth.weights(N, K, 720)
    x = synth.activations(M, K, 721, outliers=True)
    packed = B.mnnq_pack_weights(dev(W), mode=mode)
    xq, sx, _ = B.mnnq_quant_act(dev(x), want_xsum=False)
    y8 = host(B.mnnq_linear_prefill(packed, N, K, xq, sx, mode=mode))
    y16 = host(B.mnnq_linear_prefill_f16(packed, N, K, xq.to(torch.float16), row_scale=sx, mode=mode))
    assert np.abs(y16 - y8).max() <= 2e-6 * np.abs(y8).max()


@pytest.mark.parametrize("which", [0, 1])
def test_one_hot_returns_the_weight_column(which):
    mode, quant = MODES[which]
    N, K = 32, 256
    W = synth.weights(N, K, 77)
    q, s, mn = quant(W)
    what = oracle.dequant_minf(q, s, mn)
    packed = B.mnnq_pack_weights(dev(W), mode=mode)
    atol = 2e-7 * np.abs(mn).max()     # q * step and the minimum cancel: fp32 rounding at the minimum's size
    for j in (0, 17, 64, 255):
        x16 = np.zeros((1, K), np.float16); x16[0, j] = 1.0
        y = host(B.mnnq_linear_decode_f16(packed, N, K, dev(x16[0]), mode=mode))
        np.testing.assert_allclose(y, what[:, j], rtol=2e-6, atol=atol)
        y = host(B.mnnq_linear_prefill_f16(packed, N, K, dev(x16), mode=mode))
        np.testing.assert_allclose(y[0], what[:, j], rtol=2e-6, atol=atol)


def test_rows_do_not_leak_with_an_odd_group_count():
    M, N, K = 40, 32, 192
    W = synth.weights(N, K, 910)
    x16 = synth.activations_f16(M, K, 911)
    q, s, mn = oracle.quant_weights_minf(W)
    y_o = oracle.linear_a16_minf(x16, q, s, mn)
    bad = x16.copy()
    bad[7, :] = np.float16(np.inf)
    packed = B.mnnq_pack_weights(dev(W), mode=B.MODE_W4_MIN_FLOAT)
    y = host(B.mnnq_linear_prefill_f16(packed, N, K, dev(bad), mode=B.MODE_W4_MIN_FLOAT))
    keep = np.arange(M) != 7
    assert np.isfinite(y[keep]).all()
    assert np.abs(y[keep] - y_o[keep]).max() <= TOL_A16 * np.abs(y_o).max()
