"""Pins for the oracle's linear layers (O4 W4A8, O5 W4A16).

Given the codes, both layers reach exactly (up to one final rounding) the plain
product y = x^ . w^T of the dequantized operands, so they are pinned against:
brute force in Python integers / exact rationals on tiny shapes, an independent
library route (numpy int64 / float64 matmul), a one-hot input that must return
a dequantized weight column, the hand-worked group of tests/golden, and
metamorphic relations (power-of-two scaling, row permutation, concatenation
along N).  Shapes follow Section 5.1: activations [e, l], weights [h, l],
result [e, h].
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2506_10443_amd import synth


def _setup(M, N, K, seed, outliers=True):
    W = synth.weights(N, K, seed)
    x = synth.activations(M, K, seed + 1000, outliers=outliers)
    q, s, z = oracle.quant_weights(W)
    xq, sx, xsum = oracle.quant_act(x)
    return W, x, q, s, z, xq, sx, xsum


def test_brute_force_tiny_integers_and_rationals():
    M, N, K = 3, 4, 128
    W, x, q, s, z, xq, sx, xsum = _setup(M, N, K, 21)
    bias = np.array([0.5, -0.25, 0.0, 3.0], np.float32)
    acc, y = oracle.linear_w4a8(xq, sx, q, s, z, bias=bias)
    for m in range(M):
        for n in range(N):
            total = Fraction(0)
            for g in range(K // 64):
                I = 0
                for k in range(64 * g, 64 * g + 64):
                    I += int(xq[m, k]) * (int(q[n, k]) - int(z[n, g]))
                assert acc[m, n, g] == I
                total += Fraction(float(s[n, g])) * I
            exact = Fraction(float(sx[m])) * total + Fraction(float(bias[n]))
            assert y[m, n] == np.float32(float(exact))  # correctly rounded once


@pytest.mark.parametrize("M,N,K", [(1, 48, 192), (5, 33, 256), (17, 16, 1536)])
def test_integer_accumulators_library_route(M, N, K):
    W, x, q, s, z, xq, sx, xsum = _setup(M, N, K, 31)
    acc, y = oracle.linear_w4a8(xq, sx, q, s, z)
    G = K // 64
    d = q.astype(np.int64).reshape(N, G, 64) - z.astype(np.int64)[:, :, None]
    a = xq.astype(np.int64).reshape(M, G, 64)
    ref = np.einsum("mgk,ngk->mng", a, d)
    assert np.array_equal(acc, ref)
    assert np.abs(acc).max() <= 64 * 127 * 15
    # identity: I = sum xq*q - z * xsum
    A = np.einsum("mgk,ngk->mng", a, q.astype(np.int64).reshape(N, G, 64))
    assert np.array_equal(acc, A - z.astype(np.int64)[None] * xsum.astype(np.int64)[:, None, :])
    # float part: y == sx * (xq . w^T) with w^ from O2, via float64 matmul
    what = oracle.dequant(q, s, z).astype(np.float64)
    yref = sx.astype(np.float64)[:, None] * (xq.astype(np.float64) @ what.T)
    np.testing.assert_allclose(y, yref, rtol=0, atol=1e-6 * np.abs(yref).max())


def test_one_hot_returns_dequantized_column():
    N, K = 40, 256
    W = synth.weights(N, K, 41)
    q, s, z = oracle.quant_weights(W)
    what = oracle.dequant(q, s, z)
    for j, c in [(0, 1.0), (63, -2.5), (64, 0.375), (255, 100.0)]:
        x = np.zeros((1, K), np.float32)
        x[0, j] = c
        xq, sx, _ = oracle.quant_act(x)
        assert abs(int(xq[0, j])) == 127 and np.count_nonzero(xq) == 1
        _, y = oracle.linear_w4a8(xq, sx, q, s, z)
        np.testing.assert_allclose(y[0], c * what[:, j].astype(np.float64), rtol=1e-6, atol=0)


def test_worked_group_closed_form():
    # Weights: the hand-worked group (scale 1/8, zero 7, codes k mod 16), twice
    # with the second row negated.  Activations: integers with |x| max 127, so
    # the activation scale is exactly 1.  y is an exact dyadic rational.
    w = np.array([((k % 16) - 7) * 0.125 for k in range(128)], np.float32)
    W = np.stack([w, -w])
    q, s, z = oracle.quant_weights(W)
    x = np.array([[(k % 5) - 2 for k in range(128)]], np.float32)
    x[0, 0] = 127.0
    xq, sx, _ = oracle.quant_act(x)
    assert sx[0] == 1.0
    _, y = oracle.linear_w4a8(xq, sx, q, s, z)
    expect = sum(Fraction(int(x[0, k])) * Fraction((k % 16) - 7, 8) for k in range(128))
    assert Fraction(float(y[0, 0])) == expect
    # -w has min -1.0, max 0.875 -> zero = 8, codes 15 - (k mod 16), still exact
    assert Fraction(float(y[0, 1])) == -expect


def test_metamorphic_relations():
    M, N, K = 4, 64, 512
    W, x, q, s, z, xq, sx, xsum = _setup(M, N, K, 51)
    acc, y = oracle.linear_w4a8(xq, sx, q, s, z)
    # power-of-two scaling of x scales y exactly
    xq2, sx2, _ = oracle.quant_act(x * np.float32(4.0))
    _, y2 = oracle.linear_w4a8(xq2, sx2, q, s, z)
    assert np.array_equal(y2, y * np.float32(4.0))
    # permuting weight rows permutes outputs
    perm = np.random.default_rng(0).permutation(N)
    qp, sp, zp = oracle.quant_weights(W[perm])
    accp, yp = oracle.linear_w4a8(xq, sx, qp, sp, zp)
    assert np.array_equal(yp, y[:, perm]) and np.array_equal(accp, acc[:, perm])
    # concatenation along N == separate calls
    _, ya = oracle.linear_w4a8(xq, sx, q[:24], s[:24], z[:24])
    _, yb = oracle.linear_w4a8(xq, sx, q[24:], s[24:], z[24:])
    assert np.array_equal(np.concatenate([ya, yb], axis=1), y)
    # tokens are independent
    _, y1 = oracle.linear_w4a8(xq[1:2], sx[1:2], q, s, z)
    assert np.array_equal(y1[0], y[1])
    # bias is added last
    bias = np.linspace(-1, 1, N).astype(np.float32)
    _, yb = oracle.linear_w4a8(xq, sx, q, s, z, bias=bias)
    np.testing.assert_allclose(yb, y.astype(np.float64) + bias, rtol=0, atol=2e-7 * np.abs(y).max() + 1e-7)


def test_against_real_valued_product_bound():
    M, N, K = 4, 32, 1536
    W, x, q, s, z, xq, sx, xsum = _setup(M, N, K, 61)
    _, y = oracle.linear_w4a8(xq, sx, q, s, z)
    exact = x.astype(np.float64) @ W.astype(np.float64).T
    what = oracle.dequant(q, s, z).astype(np.float64)
    srep = np.repeat(s.astype(np.float64), 64, axis=1)               # [N,K]
    bound = np.abs(x).astype(np.float64) @ (srep / 2).T + \
        (sx.astype(np.float64)[:, None] / 2) * np.abs(what).sum(axis=1)[None, :]
    assert np.all(np.abs(y - exact) <= bound * (1 + 1e-4))
    # and the quantized product is a useful approximation, not noise
    assert np.abs(y - exact).max() < 0.2 * np.abs(exact).max()


def test_sampled_variant_matches_full():
    M, N, K = 6, 50, 320
    W, x, q, s, z, xq, sx, xsum = _setup(M, N, K, 71)
    acc, y = oracle.linear_w4a8(xq, sx, q, s, z)
    rng = np.random.default_rng(5)
    ms = rng.integers(0, M, 40)
    ns = rng.integers(0, N, 40)
    a2, y2 = oracle.linear_w4a8_sampled(xq, sx, q, s, z, ms, ns)
    assert np.array_equal(a2, acc[ms, ns]) and np.array_equal(y2, y[ms, ns])
    x16 = synth.activations_f16(M, K, 72)
    yf = oracle.linear_w4a16(x16, q, s, z)
    yf2 = oracle.linear_w4a16_sampled(x16, q, s, z, ms, ns)
    assert np.array_equal(yf2, yf[ms, ns])


# ------------------------------------------------------------------ O5

@pytest.mark.parametrize("M,N,K", [(1, 24, 128), (7, 40, 448)])
def test_w4a16_is_float64_matmul_of_dequantized(M, N, K):
    W = synth.weights(N, K, 81)
    q, s, z = oracle.quant_weights(W)
    x16 = synth.activations_f16(M, K, 82)
    bias = np.linspace(0.5, -0.5, N).astype(np.float32)
    y = oracle.linear_w4a16(x16, q, s, z, bias=bias)
    what = oracle.dequant(q, s, z).astype(np.float64)
    ref = x16.astype(np.float64) @ what.T + bias
    np.testing.assert_allclose(y, ref, rtol=0, atol=2e-7 * np.abs(ref).max())


def test_w4a16_one_hot_and_half_decoding():
    N, K = 16, 128
    W = synth.weights(N, K, 91)
    q, s, z = oracle.quant_weights(W)
    what = oracle.dequant(q, s, z).astype(np.float64)
    # normal, subnormal, negative, large: each fp16 value must be widened exactly
    for j, v in [(3, np.float16(1.0009765625)), (64, np.float16(-5.96e-8)),
                 (100, np.float16(6.1e-5)), (127, np.float16(-65504.0))]:
        x16 = np.zeros((1, K), np.float16)
        x16[0, j] = v
        y = oracle.linear_w4a16(x16, q, s, z)
        np.testing.assert_allclose(y[0], float(v) * what[:, j], rtol=1e-6, atol=0)


def test_w4a16_close_to_w4a8_on_same_input():
    # Same weights, same activations: the two variants differ only by the
    # activation rounding (int8 vs fp16), so they agree to about sx/2 per term.
    M, N, K = 2, 64, 1024
    W = synth.weights(N, K, 95)
    x = synth.activations(M, K, 96, outliers=False)
    q, s, z = oracle.quant_weights(W)
    xq, sx, _ = oracle.quant_act(x)
    _, y8 = oracle.linear_w4a8(xq, sx, q, s, z)
    y16 = oracle.linear_w4a16(x.astype(np.float16), q, s, z)
    assert np.abs(y8 - y16).max() < 0.05 * np.abs(y16).max()
