"""Pins for O11, fp16 activations on float-minimum weights (Section 4.2: quantized weights meet
fp16 activations on the GPU path; Eq. 1 defines the weight a code stands for), 4- and 8-bit codes:
exact rational brute force, the library matmul the definition reduces to, one-hot inputs, the
integer-activation special case that must agree with the W4A8 / W8A8 oracles, the zero-point
form on a group where both forms describe the same weights, and exact scaling."""
from fractions import Fraction

import numpy as np

import oracle


def _case(rng, M, N, K, bits):
    x16 = rng.standard_normal((M, K)).astype(np.float16)
    q = rng.integers(0, 1 << bits, (N, K)).astype(np.uint8)
    s = rng.uniform(1e-3, 1e-2, (N, K // 64)).astype(np.float32)
    mn = rng.uniform(-0.1, 0.05, (N, K // 64)).astype(np.float32)
    return x16, q, s, mn


def test_brute_force_exact_rational():
    rng = np.random.default_rng(5)
    for bits in (4, 8):
        M, N, K = 2, 3, 128
        x16, q, s, mn = _case(rng, M, N, K, bits)
        bias = rng.standard_normal(N).astype(np.float32)
        y = oracle.linear_a16_minf(x16, q, s, mn, bias=bias)
        for m in range(M):
            for n in range(N):
                tot = Fraction(float(bias[n]))
                for k in range(K):
                    g = k // 64
                    w = int(q[n, k]) * Fraction(float(s[n, g])) + Fraction(float(mn[n, g]))
                    tot += Fraction(float(x16[m, k])) * w
                assert abs(Fraction(float(y[m, n])) - tot) <= abs(tot) * Fraction(1, 2 ** 22) + Fraction(1, 10 ** 9)


def test_reduces_to_float64_matmul_and_one_hot():
    rng = np.random.default_rng(6)
    for bits in (4, 8):
        M, N, K = 5, 16, 256
        x16, q, s, mn = _case(rng, M, N, K, bits)
        w = q.astype(np.float64).reshape(N, K // 64, 64) * s[..., None] + mn[..., None].astype(np.float64)
        ref = x16.astype(np.float64) @ w.reshape(N, K).T
        y = oracle.linear_a16_minf(x16, q, s, mn)
        assert np.allclose(y, ref, rtol=3e-7, atol=1e-9)
        ys = oracle.linear_a16_minf_sampled(x16, q, s, mn, np.array([0, 4, 2]), np.array([15, 0, 7]))
        assert np.array_equal(ys, y[[0, 4, 2], [15, 0, 7]])
        # one-hot row: returns the weight column times the activation
        j, c = 77, np.float16(-1.5)
        e = np.zeros((1, K), np.float16)
        e[0, j] = c
        col = oracle.linear_a16_minf(e, q, s, mn)[0]
        assert np.allclose(col, float(c) * w.reshape(N, K)[:, j], rtol=2e-7, atol=0)


def test_integer_activations_agree_with_the_int8_activation_oracles():
    rng = np.random.default_rng(7)
    M, N, K = 4, 8, 192
    xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
    one = np.ones(M, np.float32)
    for bits, lin8 in ((4, oracle.linear_w4a8_minf), (8, oracle.linear_w8a8)):
        _, q, s, mn = _case(rng, M, N, K, bits)
        y8 = lin8(xq, one, q, s, mn, want_acc=False)[1]
        y16 = oracle.linear_a16_minf(xq.astype(np.float16), q, s, mn)     # |x| <= 127 is exact in fp16
        assert np.allclose(y16, y8, rtol=1e-6, atol=1e-7)


def test_zero_point_form_on_a_group_both_forms_describe():
    # w_k = ((k mod 16) - 7) / 8: scale 1/8, zero 7, minimum -7/8 = -zero * scale exactly, so the
    # integer-zero-point oracle (O5) and this one must give the same numbers
    K, N = 64, 2
    w = (((np.arange(K) % 16) - 7) * 0.125).astype(np.float32)
    W = np.stack([w, w[::-1]])
    q, s, z = oracle.quant_weights(W)
    qm, sm, mn = oracle.quant_weights_minf(W)
    assert np.array_equal(q, qm) and np.array_equal(s, sm) and np.array_equal(mn, -(z * s))
    rng = np.random.default_rng(8)
    x16 = rng.standard_normal((3, K)).astype(np.float16)
    assert np.array_equal(oracle.linear_w4a16(x16, q, s, z), oracle.linear_a16_minf(x16, qm, sm, mn))


def test_scaling_by_a_power_of_two_is_exact():
    rng = np.random.default_rng(9)
    x16, q, s, mn = _case(rng, 3, 4, 128, 8)
    y = oracle.linear_a16_minf(x16, q, s, mn)
    y4 = oracle.linear_a16_minf((x16.astype(np.float32) * 4).astype(np.float16), q, s, mn)
    assert np.array_equal(y4, 4 * y)
