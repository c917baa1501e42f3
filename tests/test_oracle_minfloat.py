"""Pins for the oracle's Eq.-1-literal form (O6 weights, O7 dequant, O8 linear):
the group minimum stays a float offset, w^ = q * step + w_min.

None of these re-types the oracle's formula: hand-derived groups (tests/golden),
exact rational arithmetic, invariants of Eq. 1 of Section 4.2, brute force in
Python integers, and the cases in which the form coincides with the integer
zero point form, which is pinned separately.
"""
import os
from fractions import Fraction

import numpy as np

import oracle
from paper_2506_10443_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    scale = mn = None
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] == "scale":
                scale = float(tok[1])
            elif tok[0] == "min":
                mn = float(tok[1])
            else:
                rows.append([float(t) for t in tok])
    return scale, mn, rows


def test_worked_group_is_exact():
    scale, mn, rows = _read_golden("eq1_minfloat_worked_group.txt")
    table = {int(r[0]): (r[1], int(r[2])) for r in rows}
    w = np.array([table[k % 16][0] for k in range(64)], np.float32)[None, :]
    q, s, m = oracle.quant_weights_minf(w)
    assert s[0, 0] == np.float32(scale) and m[0, 0] == np.float32(mn)
    assert q[0].tolist() == [table[k % 16][1] for k in range(64)]
    assert np.array_equal(oracle.dequant_minf(q, s, m), w)       # bit for bit
    # the integer-zero-point form is a different quantizer on this group
    q0, s0, z0 = oracle.quant_weights(w)
    assert not np.array_equal(q0, q) and s0[0, 0] != s[0, 0]


def test_ties_round_half_to_even():
    scale, mn, rows = _read_golden("eq1_minfloat_ties_group.txt")
    w = np.full((1, 64), 3.0, np.float32)
    for i, (val, _) in enumerate(rows):
        w[0, i] = val
    q, s, m = oracle.quant_weights_minf(w)
    assert s[0, 0] == np.float32(scale) and m[0, 0] == np.float32(mn)
    for i, (val, code) in enumerate(rows):
        assert q[0, i] == int(code), (val, q[0, i], code)
    assert (q[0, len(rows):] == 4).all()


def _eq1_exact(w):
    """Eq. 1 in exact rational arithmetic with round-half-even, for one group."""
    w = [Fraction(float(v)) for v in w]
    mn, mx = min(w), max(w)
    step = (mx - mn) / 15
    return [int(round((v - mn) / step)) for v in w], step, mn     # Python's round() is half-even


def test_against_exact_rational_eq1_on_dyadic_inputs():
    # Multiples of 2^-6 in a range whose width is 15 * 2^-j: every binary32 operation of the
    # quantizer is then exact, so the codes must equal Eq. 1 evaluated over the rationals.
    rng = np.random.default_rng(11)
    for trial in range(40):
        j = int(rng.integers(0, 4))
        width = 15.0 / (1 << j)
        lo = float(rng.integers(-64, 64)) / 8.0
        w = lo + np.round(rng.uniform(0, width, 64) * 64) / 64
        w[0], w[1] = lo, lo + width
        w = np.clip(w, lo, lo + width).astype(np.float32)
        codes, step, mn = _eq1_exact(w)
        q, s, m = oracle.quant_weights_minf(w[None, :])
        assert Fraction(float(s[0, 0])) == step and Fraction(float(m[0, 0])) == mn
        assert q[0].tolist() == codes


def test_invariants_on_random_groups():
    W = synth.weights(64, 512, 5)
    q, s, m = oracle.quant_weights_minf(W)
    G = 512 // 64
    Wg = W.reshape(64, G, 64)
    qg = q.reshape(64, G, 64)
    assert np.array_equal(m, Wg.min(axis=2))                      # the offset is the group minimum
    assert q.min() == 0 and q.max() == 15
    # minimum -> code 0, maximum -> code 15, in every group; codes are monotone in w
    assert (np.take_along_axis(qg, Wg.argmin(axis=2)[..., None], 2) == 0).all()
    assert (np.take_along_axis(qg, Wg.argmax(axis=2)[..., None], 2) == 15).all()
    order = np.argsort(Wg, axis=2, kind="stable")
    assert (np.diff(np.take_along_axis(qg, order, 2).astype(int), axis=2) >= 0).all()
    # reconstruction error at most half a step (plus binary32 rounding of the quantizer's operations)
    What = oracle.dequant_minf(q, s, m).reshape(64, G, 64)
    assert (np.abs(What.astype(np.float64) - Wg) <= 0.5 * s[..., None].astype(np.float64) * (1 + 1e-5)).all()
    # the minimum is reproduced exactly
    assert np.array_equal(np.take_along_axis(What, Wg.argmin(axis=2)[..., None], 2)[..., 0], m)
    # step is (max - min) / 15 per (row, group): a transposed axis or a per-row step fails here
    ref = ((Wg.max(axis=2).astype(np.float64) - Wg.min(axis=2)) / 15)
    assert np.allclose(s, ref, rtol=1e-6, atol=0)


def test_shift_and_scale_covariance():
    # Eq. 1 depends on w only through (w - w_min) / (w_max - w_min): a shift of the group by a
    # constant and a scaling by a power of two leave the codes alone (values chosen so that the
    # shifted and scaled inputs are exact in binary32).
    rng = np.random.default_rng(3)
    w = (rng.integers(-2000, 2000, (4, 128)) / 1024.0).astype(np.float32)
    q, s, m = oracle.quant_weights_minf(w)
    q2, s2, m2 = oracle.quant_weights_minf(w + np.float32(3.0))
    assert np.array_equal(q2, q) and np.array_equal(s2, s) and np.array_equal(m2, m + np.float32(3.0))
    q3, s3, m3 = oracle.quant_weights_minf(w * np.float32(0.25))
    assert np.array_equal(q3, q) and np.array_equal(s3, s * np.float32(0.25)) and np.array_equal(m3, m * np.float32(0.25))
    # the integer-zero-point form is not shift covariant
    assert not np.array_equal(oracle.quant_weights(w + np.float32(3.0))[0], oracle.quant_weights(w)[0])


def test_constant_group_and_tiny_range():
    w = np.full((1, 128), -0.375, np.float32)
    w[0, 64:] = 0.0
    q, s, m = oracle.quant_weights_minf(w)
    assert (q == 0).all() and s.tolist() == [[1.0, 1.0]] and m.tolist() == [[-0.375, 0.0]]
    assert np.array_equal(oracle.dequant_minf(q, s, m), w)
    w2 = np.full((1, 64), 1.0, np.float32)
    w2[0, 7] = np.nextafter(np.float32(1.0), np.float32(2.0))
    q2, s2, m2 = oracle.quant_weights_minf(w2)
    assert q2[0, 7] == 15 and (np.delete(q2[0], 7) == 0).all() and m2[0, 0] == 1.0


def test_coincides_with_zero_point_form_when_the_minimum_is_a_multiple_of_the_step():
    # eq1_worked_group: w_min = -7 steps, so zero = 7 and (q - 7) * step = q * step + w_min.
    w = np.array([((k % 16) - 7) * 0.125 for k in range(64)], np.float32)[None, :]
    q0, s0, z0 = oracle.quant_weights(w)
    q1, s1, m1 = oracle.quant_weights_minf(w)
    assert np.array_equal(q0, q1) and np.array_equal(s0, s1) and m1[0, 0] == -(z0[0, 0] * s0[0, 0])
    assert np.array_equal(oracle.dequant(q0, s0, z0), oracle.dequant_minf(q1, s1, m1))


def _rand_layer(M, N, K, seed):
    rng = np.random.default_rng(seed)
    xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
    sx = rng.uniform(0.01, 0.1, M).astype(np.float32)
    q = rng.integers(0, 16, (N, K)).astype(np.uint8)
    s = rng.uniform(1e-3, 1e-2, (N, K // 64)).astype(np.float32)
    mn = rng.uniform(-0.1, 0.05, (N, K // 64)).astype(np.float32)
    return xq, sx, q, s, mn


def test_linear_integer_part_by_brute_force():
    xq, sx, q, s, mn = _rand_layer(3, 5, 128, 1)
    acc, _ = oracle.linear_w4a8_minf(xq, sx, q, s, mn)
    for m in range(3):
        for n in range(5):
            for g in range(2):
                want = sum(int(xq[m, 64 * g + k]) * int(q[n, 64 * g + k]) for k in range(64))
                assert acc[m, n, g] == want
    # an independent library route: int64 einsum per group
    ref = np.einsum("mgk,ngk->mng", xq.reshape(3, 2, 64).astype(np.int64), q.reshape(5, 2, 64).astype(np.int64))
    assert np.array_equal(acc, ref)


def test_linear_is_the_correctly_rounded_product_with_the_dequantized_weights():
    # y[m,n] = sum_k (sx[m] xq[m,k]) * (q[n,k] step + w_min), evaluated over the rationals.
    xq, sx, q, s, mn = _rand_layer(2, 3, 128, 2)
    bias = np.array([0.5, -0.25, 0.125], np.float32)
    _, y = oracle.linear_w4a8_minf(xq, sx, q, s, mn, bias=bias)
    for m in range(2):
        for n in range(3):
            tot = Fraction(0)
            for k in range(128):
                g = k // 64
                what = int(q[n, k]) * Fraction(float(s[n, g])) + Fraction(float(mn[n, g]))
                tot += int(xq[m, k]) * what
            exact = Fraction(float(sx[m])) * tot + Fraction(float(bias[n]))
            # binary64 accumulation, one rounding to binary32: within one binary32 ulp of the exact value
            assert abs(Fraction(float(y[m, n])) - exact) <= abs(exact) * Fraction(1, 2 ** 23)
            assert np.float32(float(exact)) == y[m, n] or abs(float(y[m, n]) - float(exact)) <= abs(float(exact)) * 2 ** -24 * 1.01


def test_linear_matches_float64_matmul_and_zero_point_form():
    xq, sx, q, s, mn = _rand_layer(4, 6, 256, 3)
    _, y = oracle.linear_w4a8_minf(xq, sx, q, s, mn)
    what = q.astype(np.float64).reshape(6, 4, 64) * s[..., None].astype(np.float64) + mn[..., None].astype(np.float64)
    ref = (xq.astype(np.float64) * sx[:, None].astype(np.float64)) @ what.reshape(6, 256).T
    assert np.allclose(y, ref, rtol=3e-7, atol=1e-9)
    # one-hot activation returns the dequantized column
    e = np.zeros((1, 256), np.int8); e[0, 70] = 1
    _, y1 = oracle.linear_w4a8_minf(e, np.ones(1, np.float32), q, s, mn)
    assert np.array_equal(y1[0], oracle.dequant_minf(q, s, mn)[:, 70])
    # with w_min = -zero * step (exactly representable here) the two forms are the same function
    z = np.random.default_rng(4).integers(0, 16, (6, 4)).astype(np.uint8)
    s2 = (np.random.default_rng(5).integers(1, 64, (6, 4)) / 1024.0).astype(np.float32)
    mn2 = -(z.astype(np.float32) * s2)
    _, ya = oracle.linear_w4a8_minf(xq, sx, q, s2, mn2)
    _, yb = oracle.linear_w4a8(xq, sx, q, s2, z)
    assert np.allclose(ya, yb, rtol=1e-6, atol=1e-7)


def test_sampled_variant_agrees_with_full():
    xq, sx, q, s, mn = _rand_layer(5, 7, 192, 6)
    acc, y = oracle.linear_w4a8_minf(xq, sx, q, s, mn)
    ms = np.array([0, 4, 2, 2]); ns = np.array([6, 0, 3, 3])
    a2, y2 = oracle.linear_w4a8_minf_sampled(xq, sx, q, s, mn, ms, ns)
    assert np.array_equal(a2, acc[ms, ns]) and np.array_equal(y2, y[ms, ns])
