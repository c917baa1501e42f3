"""Pins for the oracle's int8 weight path (O9 quantizer, O10 linear): Eq. 1 of Section 4.2 with
clip range 0..255 and the group minimum as a float offset.  Hand-derived group, exact rational
arithmetic, invariants, brute force; the linear part is also tied to the 4-bit float-minimum
form (pinned separately) through the split of a code into two nibbles."""
import os
from fractions import Fraction

import numpy as np

import oracle
from paper_2506_10443_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_worked_group_is_exact():
    scale = mn = None
    rows = []
    for line in open(os.path.join(GOLD, "eq1_int8_worked_group.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0] == "scale":
            scale = float(tok[1])
        elif tok[0] == "min":
            mn = float(tok[1])
        else:
            rows.append((int(tok[0]), float(tok[1]), int(tok[2])))
    w = np.array([r[1] for r in rows], np.float32)[None, :]
    q, s, m = oracle.quant_weights8(w)
    assert s[0, 0] == np.float32(scale) and m[0, 0] == np.float32(mn)
    assert q[0].tolist() == [r[2] for r in rows]
    assert np.array_equal(oracle.dequant_minf(q, s, m), w)


def test_against_exact_rational_eq1_on_dyadic_inputs():
    rng = np.random.default_rng(21)
    for trial in range(40):
        j = int(rng.integers(0, 4))
        width = 255.0 / (64 << j)                       # step = 2^-(6+j)
        lo = float(rng.integers(-64, 64)) / 8.0
        w = lo + np.round(rng.uniform(0, width, 64) * 1024) / 1024
        w[0], w[1] = lo, lo + width
        w = np.clip(w, lo, lo + width).astype(np.float32)
        fr = [Fraction(float(v)) for v in w]
        step = (max(fr) - min(fr)) / 255
        codes = [int(round((v - min(fr)) / step)) for v in fr]       # round() is half-even
        q, s, m = oracle.quant_weights8(w[None, :])
        assert Fraction(float(s[0, 0])) == step and Fraction(float(m[0, 0])) == min(fr)
        assert q[0].tolist() == codes


def test_invariants_on_random_groups():
    W = synth.weights(32, 512, 8)
    q, s, m = oracle.quant_weights8(W)
    Wg = W.reshape(32, 8, 64)
    qg = q.reshape(32, 8, 64)
    assert np.array_equal(m, Wg.min(axis=2))
    assert (np.take_along_axis(qg, Wg.argmin(axis=2)[..., None], 2) == 0).all()
    assert (np.take_along_axis(qg, Wg.argmax(axis=2)[..., None], 2) == 255).all()
    What = oracle.dequant_minf(q, s, m).reshape(32, 8, 64)
    assert (np.abs(What.astype(np.float64) - Wg) <= 0.5 * s[..., None].astype(np.float64) * (1 + 1e-4)).all()
    ref = (Wg.max(axis=2).astype(np.float64) - Wg.min(axis=2)) / 255
    assert np.allclose(s, ref, rtol=1e-6, atol=0)
    # 16 times finer than the 4-bit grid on the same data (same range, 255 vs 15 steps)
    s4 = oracle.quant_weights_minf(W)[1]
    assert np.allclose(s4 / s, 17.0, rtol=1e-5)
    # constant group
    c = np.full((1, 64), 0.5, np.float32)
    qc, sc, mc = oracle.quant_weights8(c)
    assert (qc == 0).all() and sc[0, 0] == 1.0 and mc[0, 0] == 0.5


def test_linear_brute_force_and_nibble_split():
    rng = np.random.default_rng(9)
    M, N, K = 3, 4, 128
    xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
    sx = rng.uniform(0.01, 0.1, M).astype(np.float32)
    q = rng.integers(0, 256, (N, K)).astype(np.uint8)
    q[0, :4] = [0, 255, 15, 16]
    s = rng.uniform(1e-4, 1e-3, (N, K // 64)).astype(np.float32)
    mn = rng.uniform(-0.1, 0.05, (N, K // 64)).astype(np.float32)
    acc, y = oracle.linear_w8a8(xq, sx, q, s, mn)
    for m in range(M):
        for n in range(N):
            tot = Fraction(0)
            for g in range(K // 64):
                A = sum(int(xq[m, 64 * g + k]) * int(q[n, 64 * g + k]) for k in range(64))
                assert acc[m, n, g] == A
                xs = sum(int(xq[m, 64 * g + k]) for k in range(64))
                tot += Fraction(float(s[n, g])) * A + Fraction(float(mn[n, g])) * xs
            exact = Fraction(float(sx[m])) * tot
            assert abs(Fraction(float(y[m, n])) - exact) <= abs(exact) * Fraction(1, 2 ** 23)
    # q = 16 hi + lo: the same layer as two 4-bit planes over the doubled reduction axis, steps
    # 16 s and s, minimum carried by the high plane only
    hi, lo = q >> 4, q & 15
    q2 = np.concatenate([hi, lo], axis=1)
    s2 = np.concatenate([16 * s, s], axis=1)
    mn2 = np.concatenate([mn, np.zeros_like(mn)], axis=1)
    xq2 = np.concatenate([xq, xq], axis=1)
    acc2, y2 = oracle.linear_w4a8_minf(xq2, sx, q2, s2, mn2)
    G = K // 64
    assert np.array_equal(16 * acc2[:, :, :G] + acc2[:, :, G:], acc)
    assert np.allclose(y2, y, rtol=1e-6, atol=1e-9)
    # float64 matmul with the dequantized weights
    what = oracle.dequant_minf(q, s, mn).astype(np.float64)
    exact_w = q.astype(np.float64).reshape(N, G, 64) * s[..., None] + mn[..., None].astype(np.float64)
    ref = (xq.astype(np.float64) * sx[:, None]) @ exact_w.reshape(N, K).T
    assert np.allclose(y, ref, rtol=3e-7, atol=1e-9)
    assert np.allclose(what, exact_w.reshape(N, K), rtol=1e-7)
    a3, y3 = oracle.linear_w8a8_sampled(xq, sx, q, s, mn, np.array([0, 2]), np.array([3, 1]))
    assert np.array_equal(a3, acc[[0, 2], [3, 1]]) and np.array_equal(y3, y[[0, 2], [3, 1]])
