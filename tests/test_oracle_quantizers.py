"""Pins for the oracle's quantizers (O1 weights, O2 dequant, O3 activations).

None of these re-types the oracle's formula: they check hand-derived examples
(tests/golden), invariants that follow from Eq. 1 of Section 4.2, and special
cases, chosen so that a dropped term, a wrong sign, a wrong rounding mode or a
transposed axis fails at least one.
"""
import os

import numpy as np
import pytest

import oracle
from paper_2506_10443_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    scale = zero = None
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] == "scale":
                scale = float(tok[1])
            elif tok[0] == "zero":
                zero = int(tok[1])
            else:
                rows.append([float(t) for t in tok])
    return scale, zero, rows


def test_worked_group_is_exact():
    scale, zero, rows = _read_golden("eq1_worked_group.txt")
    table = {int(r[0]): (r[1], int(r[2])) for r in rows}
    w = np.array([table[k % 16][0] for k in range(64)], np.float32)[None, :]
    q, s, z = oracle.quant_weights(w)
    assert s[0, 0] == np.float32(scale) and z[0, 0] == zero
    assert q[0].tolist() == [table[k % 16][1] for k in range(64)]
    assert np.array_equal(oracle.dequant(q, s, z), w)  # bit for bit


def test_ties_round_half_to_even_and_clip():
    scale, zero, rows = _read_golden("eq1_ties_group.txt")
    w = np.zeros((1, 64), np.float32)
    for i, (val, _) in enumerate(rows):
        w[0, i] = val
    q, s, z = oracle.quant_weights(w)
    assert s[0, 0] == np.float32(scale) and z[0, 0] == zero
    for i, (val, code) in enumerate(rows):
        assert q[0, i] == int(code), (val, q[0, i], code)
    # the clipped top element sits exactly half a step away
    what = oracle.dequant(q, s, z)
    assert abs(float(what[0, 1]) - 11.5) == 0.5


def test_zero_point_tie_rounds_to_even():
    scale, zero, rows = _read_golden("eq1_zero_tie_group.txt")
    w = np.zeros((1, 64), np.float32)
    for i, (val, _) in enumerate(rows):
        w[0, i] = val
    q, s, z = oracle.quant_weights(w)
    assert s[0, 0] == np.float32(scale) and z[0, 0] == zero
    assert [int(c) for c in q[0, :len(rows)]] == [int(r[1]) for r in rows]
    assert np.all(q[0, len(rows):] == zero)


def test_group_axis_is_k_and_rows_are_independent():
    # Two rows with very different ranges, two groups each with different
    # ranges: scale must differ per (row, group) and follow the K axis.
    w = np.zeros((2, 128), np.float32)
    w[0, :64] = np.linspace(-1, 1.5, 64)
    w[0, 64:] = np.linspace(-10, 20, 64)
    w[1, :64] = np.linspace(-0.01, 0.02, 64)
    w[1, 64:] = np.linspace(-300, 0, 64)
    q, s, z = oracle.quant_weights(w)
    np.testing.assert_allclose(s, [[2.5 / 15, 30 / 15], [0.03 / 15, 300 / 15]], rtol=1e-6)
    assert z.tolist() == [[6, 5], [5, 15]]
    # a transposed implementation would quantize columns: check one element
    assert q[0, 0] == 0 and q[0, 63] == 15 and q[1, 64] == 0 and q[1, 127] == 15


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_round_trip_within_half_step_and_code_range(seed):
    W = synth.weights(96, 512, seed)
    q, s, z = oracle.quant_weights(W)
    assert q.max() <= 15 and z.max() <= 15
    G = W.shape[1] // 64
    what = oracle.dequant(q, s, z)
    err = np.abs(what.astype(np.float64) - W.astype(np.float64)).reshape(96, G, 64)
    half = (s.astype(np.float64) / 2)[:, :, None]
    assert np.all(err <= half * (1 + 1e-5))
    # the error is not trivially small either: some element is beyond 0.45 step
    assert (err / half).max() > 0.9
    Wg = W.reshape(96, G, 64)
    qg = q.reshape(96, G, 64)
    imin = Wg.argmin(axis=2)
    imax = Wg.argmax(axis=2)
    rows, grp = np.indices((96, G))
    assert np.all(qg[rows, grp, imin] == 0)       # minimum element -> lowest code
    assert np.all(qg[rows, grp, imax] >= 14)      # maximum -> top code (15 unless a tie clips z)
    assert np.mean(qg[rows, grp, imax] == 15) > 0.9
    # codes are monotone in w inside a group
    order = np.argsort(Wg, axis=2, kind="stable")
    sorted_codes = np.take_along_axis(qg, order, axis=2).astype(np.int32)
    assert np.all(np.diff(sorted_codes, axis=2) >= 0)


def test_scale_matches_range_over_15():
    W = synth.weights(8, 256, 5)
    _, s, z = oracle.quant_weights(W)
    Wg = W.reshape(8, 4, 64).astype(np.float64)
    rng = Wg.max(axis=2) - Wg.min(axis=2)
    np.testing.assert_allclose(s, rng / 15, rtol=3e-7)
    np.testing.assert_array_equal(z, np.rint(-Wg.min(axis=2) / s.astype(np.float64)).astype(np.uint8))


def test_groups_not_straddling_zero_and_zero_group():
    w = np.zeros((4, 64), np.float32)
    w[0] = np.linspace(1.0, 16.0, 64)     # all positive: range widened down to 0
    w[1] = np.linspace(-16.0, -1.0, 64)   # all negative: range widened up to 0
    w[2] = 0.0                            # all zero
    w[3] = 3.0                            # constant positive
    q, s, z = oracle.quant_weights(w)
    assert z[0, 0] == 0 and s[0, 0] == np.float32(16.0 / 15.0)
    assert z[1, 0] == 15 and s[1, 0] == np.float32(16.0 / 15.0)
    assert s[2, 0] == 1.0 and z[2, 0] == 0 and not q[2].any()
    assert z[3, 0] == 0 and s[3, 0] == np.float32(0.2) and np.all(q[3] == 15)
    what = oracle.dequant(q, s, z)
    assert np.all(np.abs(what - w) <= s[:, :1] / 2 * (1 + 1e-5))
    assert np.array_equal(what[2], w[2])
    np.testing.assert_allclose(what[3], w[3], rtol=1e-6)


def test_weight_codes_scale_invariance():
    # Scaling a group by a power of two scales s exactly and leaves codes alone.
    W = synth.weights(4, 128, 9)
    q1, s1, z1 = oracle.quant_weights(W)
    q2, s2, z2 = oracle.quant_weights(W * np.float32(8.0))
    assert np.array_equal(q1, q2) and np.array_equal(z1, z2)
    assert np.array_equal(s2, s1 * np.float32(8.0))
    # Negating weights mirrors the codes inside the used range.
    q3, s3, z3 = oracle.quant_weights(-W)
    assert np.array_equal(s3, s1)
    w1 = oracle.dequant(q1, s1, z1)
    w3 = oracle.dequant(q3, s3, z3)
    # dequantized values mirror up to one step where -min/s sits on a tie
    assert np.all(np.abs(w1 + w3) <= np.repeat(s1, 64, axis=1) * (1 + 1e-5))


# ------------------------------------------------------------------ O3

def test_act_integer_example():
    # amax = 127 -> scale exactly 1, codes equal the (integer) inputs.
    rng = np.random.default_rng(3)
    x = rng.integers(-127, 128, size=(3, 128)).astype(np.float32)
    x[:, 5] = [127, -127, 127]
    xq, sx, xsum = oracle.quant_act(x)
    assert np.all(sx == 1.0)
    assert np.array_equal(xq.astype(np.float32), x)
    assert np.array_equal(xsum, x.reshape(3, 2, 64).sum(axis=2).astype(np.int32))


@pytest.mark.parametrize("outliers", [False, True])
def test_act_invariants(outliers):
    x = synth.activations(5, 1536, 7, outliers=outliers)
    xq, sx, xsum = oracle.quant_act(x)
    amax = np.abs(x).max(axis=1)
    np.testing.assert_allclose(sx, amax / 127.0, rtol=2e-7)
    assert xq.min() >= -127 and xq.max() <= 127
    # the largest element maps to +-127 exactly
    idx = np.abs(x).argmax(axis=1)
    assert np.all(np.abs(xq[np.arange(5), idx].astype(np.int32)) == 127)
    assert np.all(np.sign(xq[np.arange(5), idx]) == np.sign(x[np.arange(5), idx]))
    err = np.abs(x.astype(np.float64) - sx[:, None].astype(np.float64) * xq)
    assert np.all(err <= sx[:, None] / 2 * (1 + 1e-5))
    assert (err / (sx[:, None] / 2)).max() > 0.9
    assert np.array_equal(xsum, xq.astype(np.int32).reshape(5, -1, 64).sum(axis=2))
    # per-token: rows are quantized independently
    xq1, sx1, _ = oracle.quant_act(x[2:3])
    assert np.array_equal(xq1[0], xq[2]) and sx1[0] == sx[2]


def test_act_power_of_two_scaling_and_zero_row():
    x = synth.activations(3, 256, 11)
    x[1] = 0.0
    xq, sx, xsum = oracle.quant_act(x)
    assert sx[1] == 0.0 and not xq[1].any() and not xsum[1].any()
    xq2, sx2, _ = oracle.quant_act(x * np.float32(2.0 ** -7))
    assert np.array_equal(xq, xq2)
    assert np.array_equal(sx2, sx * np.float32(2.0 ** -7))
    xq3, _, _ = oracle.quant_act(-x)
    assert np.array_equal(xq3, -xq)


def test_act_ties_half_to_even():
    # amax = 127 -> scale 1; x = j + 0.5 must go to the even neighbour.
    x = np.zeros((1, 64), np.float32)
    x[0, 0] = 127.0
    vals = [0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 125.5, 126.5]
    x[0, 1:1 + len(vals)] = vals
    xq, sx, _ = oracle.quant_act(x)
    assert sx[0] == 1.0
    assert xq[0, 1:1 + len(vals)].tolist() == [0, 2, 2, 0, -2, -2, 126, 126]
