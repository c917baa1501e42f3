"""GPU parity: every entry point of libmnnq.so against the CPU oracle on the
same seeded inputs.  Integer results (codes, zero points, int8 activations,
int32 group accumulators) and the fp32 scales must be bit-exact; fp32 outputs
must be within 1e-5 * max|y| (W4A8) resp. 1e-3 * max|y| (W4A16)."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2506_10443_amd import binding as B, synth

pytestmark = pytest.mark.gpu

TOL_A8 = 1e-5
TOL_A16 = 1e-3


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.cpu().numpy()


def note(*a):
    print(*a, flush=True)


def special_weights(N, K, seed):
    """Random weights with the quantizer's corner cases planted in the first rows."""
    W = synth.weights(N, K, seed)
    W[0, :64] = 0.0                                   # all-zero group
    W[1, :64] = np.abs(W[1, :64]) + 0.01              # all positive
    W[2, :64] = -np.abs(W[2, :64]) - 0.01             # all negative
    W[3, :64] = 3.0                                   # constant
    t = np.zeros(64, np.float32); t[:9] = [-3.5, 11.5, 0.5, 1.5, 2.5, -0.5, -2.5, -1.5, 0.0]
    W[4, :64] = t                                     # exact ties, scale 1
    t = np.zeros(64, np.float32); t[:4] = [-2.5, 12.5, 3.0, 0.0]
    W[5, :64] = t
    W[6, :64] = [((k % 16) - 7) * 0.125 for k in range(64)]
    return W


PACK_SHAPES = [(16, 64), (32, 192), (48, 128), (512, 1536), (272, 3584), (1536, 8960)]


@pytest.mark.parametrize("N,K", PACK_SHAPES)
def test_pack_unpack_bit_exact(N, K):
    note("pack", N, K)
    W = special_weights(N, K, 100 + N + K)
    q, s, z = oracle.quant_weights(W)
    packed = B.mnnq_pack_weights(dev(W))
    assert packed.numel() == B.mnnq_packed_size(N, K)
    qg, sg, zg = B.mnnq_unpack_weights(packed, N, K)
    assert np.array_equal(host(zg), z)
    assert np.array_equal(host(sg).view(np.uint32), s.view(np.uint32))
    assert np.array_equal(host(qg), q)


def test_pack_is_deterministic_and_concatenation_holds():
    Wa = synth.weights(64, 512, 7)
    Wb = synth.weights(32, 512, 8)
    pa = B.mnnq_pack_weights(dev(Wa))
    pa2 = B.mnnq_pack_weights(dev(Wa))
    assert torch.equal(pa, pa2)
    pcat = B.mnnq_pack_weights(dev(np.concatenate([Wa, Wb])))
    qc, sc, zc = B.mnnq_unpack_weights(pcat, 96, 512)
    qa, sa, za = B.mnnq_unpack_weights(pa, 64, 512)
    qb, sb, zb = B.mnnq_unpack_weights(B.mnnq_pack_weights(dev(Wb)), 32, 512)
    assert torch.equal(qc, torch.cat([qa, qb])) and torch.equal(sc, torch.cat([sa, sb]))
    assert torch.equal(zc, torch.cat([za, zb]))


@pytest.mark.parametrize("N,K", [(16, 64), (48, 192), (272, 1536), (1024, 4096)])
def test_pack_from_quantized_is_the_inverse_of_unpack(N, K):
    # Import of weights quantized elsewhere (here: by the oracle on the CPU): the packed buffer
    # must be byte-identical to the one the GPU quantizer writes, and unpack must return the inputs.
    note("pack_from_quantized", N, K)
    W = synth.weights(N, K, 600 + N + K)
    q, s, z = oracle.quant_weights(W)
    packed_ref = B.mnnq_pack_weights(dev(W))
    packed = B.mnnq_pack_from_quantized(dev(q), dev(s), dev(z))
    assert torch.equal(packed, packed_ref)
    q2, s2, z2 = B.mnnq_unpack_weights(packed, N, K)
    assert np.array_equal(host(q2), q) and np.array_equal(host(z2), z)
    assert np.array_equal(host(s2).view(np.uint32), s.view(np.uint32))
    # arbitrary codes / scales / zero points (nothing ties them to a float matrix)
    rng = np.random.default_rng(N * K)
    qr = rng.integers(0, 16, (N, K), dtype=np.uint8)
    sr = rng.uniform(1e-4, 1e-1, (N, K // 64)).astype(np.float32)
    zr = rng.integers(0, 16, (N, K // 64), dtype=np.uint8)
    pr = B.mnnq_pack_from_quantized(dev(qr), dev(sr), dev(zr))
    q3, s3, z3 = B.mnnq_unpack_weights(pr, N, K)
    assert np.array_equal(host(q3), qr) and np.array_equal(host(z3), zr)
    assert np.array_equal(host(s3).view(np.uint32), sr.view(np.uint32))
    # ... and the linear layer on them matches the oracle on the same arrays
    x = synth.activations(3, K, 601)
    xq, sx, _ = oracle.quant_act(x)
    acc_o, y_o = oracle.linear_w4a8(xq, sx, qr, sr, zr)
    assert np.array_equal(host(B.mnnq_linear_acc_debug(pr, N, K, dev(xq), True)), acc_o)
    y = host(B.mnnq_linear_prefill(pr, N, K, dev(xq), dev(sx)))
    assert np.abs(y - y_o).max() <= TOL_A8 * np.abs(y_o).max()
    y0 = host(B.mnnq_linear_decode(pr, N, K, dev(xq[0]), dev(sx[:1])))
    assert np.abs(y0 - y_o[0]).max() <= TOL_A8 * np.abs(y_o).max()
    # out-of-range inputs: codes are taken modulo 16, zero points saturate at 15
    pm = B.mnnq_pack_from_quantized(dev(qr | 0xa0), dev(sr), dev(np.where(zr == 15, 200, zr).astype(np.uint8)))
    assert torch.equal(pm, pr)


@pytest.mark.parametrize("M,K,outliers", [(1, 1536, False), (1, 64, True), (5, 192, True), (40, 3584, True),
                                          (3, 18944, True), (257, 1536, True), (33, 64, True), (20, 18944, True),
                                          (17, 20480, False), (18, 20544, True), (19, 8960, True)])
def test_quant_act_bit_exact(M, K, outliers):
    note("quant_act", M, K)
    x = synth.activations(M, K, 200 + M + K, outliers=outliers)
    if M >= 3:
        x[1] = 0.0                                   # zero row
        x[2, :8] = [127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5]
        x[2, 8:] = np.clip(np.rint(x[2, 8:] * 10), -127, 127)  # amax = 127 -> scale 1, ties above
    xq_o, sx_o, xs_o = oracle.quant_act(x)
    xq, sx, xs = B.mnnq_quant_act(dev(x))
    assert np.array_equal(host(sx).view(np.uint32), sx_o.view(np.uint32))
    assert np.array_equal(host(xq), xq_o)
    assert np.array_equal(host(xs), xs_o)
    xq2, sx2, none = B.mnnq_quant_act(dev(x), want_xsum=False)
    assert none is None and torch.equal(xq2, xq) and torch.equal(sx2, sx)


@pytest.mark.parametrize("M", [1, 24])
def test_quant_act_is_exact_at_rounding_boundaries(M):
    # The kernels round x * fl(1/scale) and do the division of the definition only next to a
    # half-integer.  Rows of values on and within a few ulps of every tie, for scales of many
    # magnitudes (also where 1/scale is not a normal number): the codes must be the oracle's.
    K = 1536
    rng = np.random.default_rng(11)
    rows = []
    for amax in (127.0, 3.3, 1e-3, 517.25, 1e-30, 3e-38, 1e-40, 2.5e38, 0.9999999, 64.0):
        scale = np.float32(amax) / np.float32(127.0)
        for ulps in (0, 1, -1, 2, -2, 7, -7):
            n = rng.integers(-126, 126, K).astype(np.float32)
            xv = ((n + np.float32(0.5)) * scale).astype(np.float32)
            if ulps:
                xv = (xv.view(np.int32) + np.where(xv >= 0, ulps, -ulps)).astype(np.int32).view(np.float32)
            xv[0] = amax
            rows.append(xv)
    x = np.stack(rows)
    for lo in range(0, len(rows), M):
        xb = x[lo:lo + M]
        xq_o, sx_o, xs_o = oracle.quant_act(xb)
        xq, sx, xs = B.mnnq_quant_act(dev(xb))
        assert np.array_equal(host(sx).view(np.uint32), sx_o.view(np.uint32))
        assert np.array_equal(host(xq), xq_o), lo
        assert np.array_equal(host(xs), xs_o)


def _layer(N, K, M, seed, outliers=True):
    W = synth.weights(N, K, seed)
    x = synth.activations(M, K, seed + 1, outliers=outliers)
    q, s, z = oracle.quant_weights(W)
    xq, sx, _ = oracle.quant_act(x)
    return W, x, q, s, z, xq, sx


DECODE_SHAPES = [(16, 64), (32, 192), (48, 1536), (8960, 1536), (1536, 8960), (528, 3584), (4096, 4096),
                 (80, 14336)]     # (seven chunks on each of sixteen waves)


@pytest.mark.parametrize("N,K", DECODE_SHAPES)
def test_decode_matches_oracle(N, K):
    note("decode", N, K)
    W, x, q, s, z, xq, sx = _layer(N, K, 1, 300 + N + K, outliers=(N, K) != (8960, 1536))
    acc_o, y_o = oracle.linear_w4a8(xq, sx, q, s, z)
    packed = B.mnnq_pack_weights(dev(W))
    xqd, sxd = dev(xq[0]), dev(sx)
    acc = B.mnnq_linear_acc_debug(packed, N, K, xqd, False)
    assert np.array_equal(host(acc), acc_o)
    tol = TOL_A8 * np.abs(y_o).max()
    results = []
    for ks in ("", "1", "2", "4", "8", "16"):
        if ks:
            B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", ks)
        else:
            B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", None)
        try:
            y = host(B.mnnq_linear_decode(packed, N, K, xqd, sxd))
        finally:
            B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", None)
        err = np.abs(y - y_o[0]).max()
        assert err <= tol, (ks, err, tol)
        results.append(y)
    y2 = host(B.mnnq_linear_decode(packed, N, K, xqd, sxd))
    assert np.array_equal(results[0], y2)          # run-to-run identical
    # the row staged under the weight stream (small layers) or after it: the same sums
    for ks in ("", "1", "4", "16"):
        pair = []
        for early in ("0", "1"):
            B.mnnq_debug_set("MNNQ_DECODE_EARLY", early)
            if ks:
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", ks)
            try:
                pair.append(host(B.mnnq_linear_decode(packed, N, K, xqd, sxd)))
            finally:
                B.mnnq_debug_set("MNNQ_DECODE_EARLY", None)
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", None)
        assert np.array_equal(pair[0], pair[1]), ks
        assert np.abs(pair[1] - y_o[0]).max() <= tol, ks
    # fused activation quantizer: same codes -> same result up to the summation order
    yf = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x)))
    assert np.abs(yf - y_o[0]).max() <= tol, (np.abs(yf - y_o[0]).max(), tol)
    assert np.abs(yf - results[0]).max() <= 2e-6 * np.abs(y_o).max()
    # ... with the quantizer run under the weight stream (small layers) or after it: the same sums
    xd = dev(x)
    for ks in ("", "1", "4", "8", "16"):
        pair = []
        for early in ("0", "1"):
            B.mnnq_debug_set("MNNQ_DECODE_EARLY", early)
            if ks:
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", ks)
            try:
                pair.append(host(B.mnnq_linear_decode_fused(packed, N, K, xd)))
            finally:
                B.mnnq_debug_set("MNNQ_DECODE_EARLY", None)
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", None)
        assert np.array_equal(pair[0], pair[1]), ks
        assert np.abs(pair[1] - y_o[0]).max() <= tol, ks


def test_config1_single_layer_seed0():
    # First benchmark configuration: x [1,1536] ~ N(0,1), W [8960,1536] ~ N(0,0.02), seed 0, whole path on the GPU.
    W, x = synth.config1()
    q, s, z = oracle.quant_weights(W)
    xq_o, sx_o, _ = oracle.quant_act(x)
    acc_o, y_o = oracle.linear_w4a8(xq_o, sx_o, q, s, z)
    packed = B.mnnq_pack_weights(dev(W))
    xq, sx, _ = B.mnnq_quant_act(dev(x))
    y = host(B.mnnq_linear_decode(packed, 8960, 1536, xq, sx))
    assert np.array_equal(host(xq), xq_o)
    assert np.array_equal(host(B.mnnq_linear_acc_debug(packed, 8960, 1536, xq, False)), acc_o)
    assert np.abs(y - y_o[0]).max() <= TOL_A8 * np.abs(y_o).max()


def test_decode_fused_zero_row_and_bias():
    N, K = 48, 320
    W = synth.weights(N, K, 43)
    packed = B.mnnq_pack_weights(dev(W))
    bias = np.linspace(-2, 2, N).astype(np.float32)
    y = host(B.mnnq_linear_decode_fused(packed, N, K, dev(np.zeros((1, K), np.float32)), bias=dev(bias)))
    assert np.array_equal(y, bias)
    x = synth.activations(1, K, 44)
    q, s, z = oracle.quant_weights(W)
    xq, sx, _ = oracle.quant_act(x)
    _, y_o = oracle.linear_w4a8(xq, sx, q, s, z, bias=bias)
    y = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x), bias=dev(bias)))
    assert np.abs(y - y_o[0]).max() <= TOL_A8 * np.abs(y_o).max()


def test_decode_fused_quantizer_is_exact_at_rounding_boundaries():
    # The fused kernel rounds x * (1/scale) and falls back to the division only near
    # half-integers.  Feed it values on and next to every tie: the codes, and with them
    # y, must equal those of the two-call path (a single differing code moves y by
    # about 1e-3 * max|y|).
    N, K = 64, 1536
    W = synth.weights(N, K, 47)
    packed = B.mnnq_pack_weights(dev(W))
    rng = np.random.default_rng(3)
    for amax in (127.0, 3.3, 1e-3, 517.25):
        scale = np.float32(amax) / np.float32(127.0)
        n = rng.integers(-126, 126, K).astype(np.float32)
        x = ((n + np.float32(0.5)) * scale).astype(np.float32)
        for ulps in (0, 1, -1, 2, -2, 5, -5):
            xv = x.copy()
            if ulps:
                xv = np.nextafter(xv, np.float32(np.inf if ulps > 0 else -np.inf)) if abs(ulps) == 1 else \
                    (xv.view(np.int32) + np.where(xv >= 0, ulps, -ulps)).astype(np.int32).view(np.float32)
            xv[0] = amax
            xq_o, sx_o, _ = oracle.quant_act(xv[None, :])
            xq, sx, _ = B.mnnq_quant_act(dev(xv[None, :]))
            assert np.array_equal(host(xq), xq_o)
            yu = host(B.mnnq_linear_decode(packed, N, K, xq, sx))
            yf = host(B.mnnq_linear_decode_fused(packed, N, K, dev(xv)))
            assert np.abs(yf - yu).max() <= 2e-6 * np.abs(yu).max(), (amax, ulps)


def test_decode_bias_and_one_hot():
    N, K = 64, 256
    W = synth.weights(N, K, 41)
    q, s, z = oracle.quant_weights(W)
    what = oracle.dequant(q, s, z)
    packed = B.mnnq_pack_weights(dev(W))
    bias = np.linspace(-1, 1, N).astype(np.float32)
    for j, c in [(0, 1.0), (63, -2.5), (64, 0.375), (255, 100.0)]:
        x = np.zeros((1, K), np.float32); x[0, j] = c
        xq, sx, _ = B.mnnq_quant_act(dev(x))
        y = host(B.mnnq_linear_decode(packed, N, K, xq, sx))
        np.testing.assert_allclose(y, c * what[:, j].astype(np.float64), rtol=2e-6, atol=0)
        yb = host(B.mnnq_linear_decode(packed, N, K, xq, sx, bias=dev(bias)))
        np.testing.assert_allclose(yb, c * what[:, j].astype(np.float64) + bias, rtol=2e-6, atol=1e-7)


PREFILL_SHAPES = [(1, 16, 64), (17, 144, 192), (128, 128, 128), (200, 512, 1536), (130, 272, 3584),
                  (512, 1536, 1536), (64, 256, 8960), (33, 400, 1536), (48, 144, 18944), (20, 4608, 1024)]


@pytest.mark.parametrize("M,N,K", PREFILL_SHAPES)
def test_prefill_matches_oracle(M, N, K):
    note("prefill", M, N, K)
    W, x, q, s, z, xq, sx = _layer(N, K, M, 400 + M + N + K)
    bias = synth.weights(1, N, 5)[0] * 10
    acc_o, y_o = oracle.linear_w4a8(xq, sx, q, s, z, bias=bias)
    packed = B.mnnq_pack_weights(dev(W))
    xqd, sxd = dev(xq), dev(sx)
    acc = B.mnnq_linear_acc_debug(packed, N, K, xqd, True)
    assert np.array_equal(host(acc), acc_o)
    acc_d = B.mnnq_linear_acc_debug(packed, N, K, xqd, False)
    assert np.array_equal(host(acc_d), acc_o)
    y = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=dev(bias)))
    tol = TOL_A8 * np.abs(y_o).max()
    assert np.abs(y - y_o).max() <= tol, (np.abs(y - y_o).max(), tol)
    y2 = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=dev(bias)))
    assert np.array_equal(y, y2)
    # every tile / split choice gives the same result to the same tolerance
    for cfg in ("b1", "b2", "s1", "s2", "b1k", "s1k", "b2k", "s2k", "w1", "w2", "v1k", "v2k", "w1k", "w2k", "t1", "t2", "t1k", "t1q", "t2q", "n1", "n2", "n1k", "n1q", "n2q"):
        B.mnnq_debug_set("MNNQ_PREFILL_TILE", cfg)
        try:
            y3 = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=dev(bias)))
            y4 = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=dev(bias)))
        finally:
            B.mnnq_debug_set("MNNQ_PREFILL_TILE", None)
        assert np.abs(y3 - y_o).max() <= tol, cfg
        assert np.array_equal(y3, y4), cfg           # two commuting addends: still reproducible
    # decode of row 0 agrees with prefill row 0 to the same tolerance
    y0 = host(B.mnnq_linear_decode(packed, N, K, xqd[0].contiguous(), sxd[:1].contiguous(), bias=dev(bias)))
    assert np.abs(y0 - y_o[0]).max() <= tol


@pytest.mark.parametrize("M", [1, 2, 5, 16])
@pytest.mark.parametrize("N,K", [(16, 64), (48, 192), (272, 1536), (144, 18944), (1024, 4096)])
def test_few_tokens_share_one_pass_over_the_weights(M, N, K):
    # M <= 16 goes through the streaming kernel (one MFMA per group and row tile for all tokens).
    note("few tokens", M, N, K)
    W, x, q, s, z, xq, sx = _layer(N, K, M, 800 + M + N + K)
    bias = synth.weights(1, N, 10)[0] * 10
    _, y_o = oracle.linear_w4a8(xq, sx, q, s, z, bias=bias, want_acc=False)
    tol = TOL_A8 * np.abs(y_o).max()
    packed = B.mnnq_pack_weights(dev(W))
    xqd, sxd, bd = dev(xq), dev(sx), dev(bias)
    for staged in ("0", "1"):        # activations straight from L2, or shared through LDS
        B.mnnq_debug_set("MNNQ_SKINNY_STAGED", staged)
        for ks in ("", "1", "2", "4", "8"):
            if ks:
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", ks)
            try:
                y = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd))
                y2 = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd))
            finally:
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", None)
            assert np.abs(y - y_o).max() <= tol, (staged, ks)
            assert np.array_equal(y, y2), (staged, ks)
        B.mnnq_debug_set("MNNQ_SKINNY_STAGED", None)
    # the tiled GEMM kernel on the same input
    B.mnnq_debug_set("MNNQ_NO_SKINNY", "1")
    try:
        y3 = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd))
    finally:
        B.mnnq_debug_set("MNNQ_NO_SKINNY", None)
    assert np.abs(y3 - y_o).max() <= tol
    # every token agrees with the one-token GEMV to the same bound
    for m in range(M):
        y0 = host(B.mnnq_linear_decode(packed, N, K, xqd[m].contiguous(), sxd[m:m + 1].contiguous(), bias=bd))
        assert np.abs(y0 - y_o[m]).max() <= tol


@pytest.mark.parametrize("M,N,K", [(1, 48, 192), (5, 272, 1536), (16, 144, 640), (130, 272, 1536), (300, 400, 1024)])
def test_prefill_fused_equals_the_two_calls(M, N, K):
    # activation quantizer inside the call: the codes pass through the caller's workspace and the
    # same kernels run, so the result is that of mnnq_quant_act + mnnq_linear_prefill bit for bit
    note("prefill fused", M, N, K)
    W, x, q, s, z, xq, sx = _layer(N, K, M, 650 + M + N + K, outliers=True)
    _, y_o = oracle.linear_w4a8(xq, sx, q, s, z, want_acc=False)
    packed = B.mnnq_pack_weights(dev(W))
    xd = dev(x)
    xq_g, sx_g, _ = B.mnnq_quant_act(xd, want_xsum=False)
    y2 = B.mnnq_linear_prefill(packed, N, K, xq_g, sx_g)
    ws = torch.full((B.mnnq_workspace_size(M, N, K) + 32,), 0x5a, dtype=torch.uint8, device="cuda:0")
    yf = B.mnnq_linear_prefill_fused(packed, N, K, xd, workspace=ws[:B.mnnq_workspace_size(M, N, K)])
    assert torch.equal(yf, y2)
    assert np.abs(host(yf) - y_o).max() <= TOL_A8 * np.abs(y_o).max()
    assert (host(ws[-32:]) == 0x5a).all()                      # nothing past the stated size is touched
    with pytest.raises(B.MnnqError):
        B.mnnq_linear_prefill_fused(packed, N, K, xd, workspace=ws[:16])


def test_prefill_many_tiles_ragged_last_column():
    # More 256-row tiles than the GPU holds at once (several rounds of workgroups), N not a
    # multiple of the tile width: every output is compared.
    M, N, K = 1024, 20496, 128
    note("prefill many tiles", M, N, K)
    W = synth.weights(N, K, 321)
    x = synth.activations(M, K, 322, outliers=True)
    q, s, z = oracle.quant_weights(W)
    xq, sx, _ = oracle.quant_act(x)
    bias = synth.weights(1, N, 8)[0] * 10
    _, y_o = oracle.linear_w4a8(xq, sx, q, s, z, bias=bias, want_acc=False)
    packed = B.mnnq_pack_weights(dev(W))
    y = host(B.mnnq_linear_prefill(packed, N, K, dev(xq), dev(sx), bias=dev(bias)))
    assert np.abs(y - y_o).max() <= TOL_A8 * np.abs(y_o).max()


def test_prefill_extreme_codes_accumulator_bound():
    # |I| reaches 64 * 127 * 15: all activations +-127, weights at the ends of the code range.
    N, K, M = 32, 256, 16
    W = np.zeros((N, K), np.float32)
    W[:, :] = 1.0          # range widened to [0, 1]: codes 15, zero 0
    W[1::2] = -1.0         # range widened to [-1, 0]: codes 0, zero 15
    x = np.full((M, K), 5.0, np.float32)
    x[1::2] = -5.0
    q, s, z = oracle.quant_weights(W)
    xq, sx, _ = oracle.quant_act(x)
    acc_o, y_o = oracle.linear_w4a8(xq, sx, q, s, z)
    assert np.abs(acc_o).max() == 64 * 127 * 15 and acc_o.min() < 0 < acc_o.max()
    packed = B.mnnq_pack_weights(dev(W))
    assert np.array_equal(host(B.mnnq_linear_acc_debug(packed, N, K, dev(xq), True)), acc_o)
    assert np.array_equal(host(B.mnnq_linear_acc_debug(packed, N, K, dev(xq), False)), acc_o)
    y = host(B.mnnq_linear_prefill(packed, N, K, dev(xq), dev(sx)))
    assert np.abs(y - y_o).max() <= TOL_A8 * np.abs(y_o).max()


F16_SHAPES = [(1, 16, 64), (9, 48, 192), (130, 272, 1536), (64, 1024, 4096), (300, 272, 448), (700, 144, 1600)]


@pytest.mark.parametrize("M,N,K", F16_SHAPES)
def test_w4a16_matches_oracle(M, N, K):
    note("w4a16", M, N, K)
    W = synth.weights(N, K, 500 + M + N + K)
    x16 = synth.activations_f16(M, K, 501 + M + N + K)
    q, s, z = oracle.quant_weights(W)
    bias = synth.weights(1, N, 6)[0] * 10
    y_o = oracle.linear_w4a16(x16, q, s, z, bias=bias)
    packed = B.mnnq_pack_weights(dev(W))
    xd = dev(x16)
    y = host(B.mnnq_linear_prefill_f16(packed, N, K, xd, bias=dev(bias)))
    tol = TOL_A16 * np.abs(y_o).max()
    assert np.abs(y - y_o).max() <= tol, (np.abs(y - y_o).max(), tol)
    for ks in ("", "1", "2", "4", "8", "16"):
        pair = []
        for early in ("0", "1"):     # x staged after or under the weight stream: the same sums
            B.mnnq_debug_set("MNNQ_DECODE_EARLY", early)
            if ks:
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", ks)
            try:
                pair.append(host(B.mnnq_linear_decode_f16(packed, N, K, xd[0].contiguous(), bias=dev(bias))))
            finally:
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", None)
                B.mnnq_debug_set("MNNQ_DECODE_EARLY", None)
        assert np.array_equal(pair[0], pair[1]), ks
        assert np.abs(pair[1] - y_o[0]).max() <= TOL_A16 * np.abs(y_o[0]).max(), ks
    y0 = host(B.mnnq_linear_decode_f16(packed, N, K, xd[0].contiguous(), bias=dev(bias)))
    assert np.abs(y0 - y_o[0]).max() <= TOL_A16 * np.abs(y_o[0]).max()


@pytest.mark.parametrize("M,N,K", [(17, 16, 64), (300, 272, 448), (513, 400, 1536), (1024, 512, 3584)])
@pytest.mark.parametrize("tile", ["", "b", "s", "b1k", "s1k"])
def test_prefill_f16_with_integer_codes_equals_int8_prefill(M, N, K, tile):
    # int8 codes are exact in fp16 and every group sum is an integer below 2^24: the fp16
    # matrix cores give the int32 accumulators exactly, hence bit-identical y - as long as the
    # fp32 sums over the groups are added in the same order: by one wave in sequence ("s1"), or in
    # two halves of the chunks that are added at the end ("s1k"; the fp16 kernel's own choice for
    # shapes with few tiles).
    note("f16 == int8", M, N, K, tile)
    W = synth.weights(N, K, 900 + M)
    x = synth.activations(M, K, 901 + M, outliers=True)
    packed = B.mnnq_pack_weights(dev(W))
    xq, sx, _ = B.mnnq_quant_act(dev(x), want_xsum=False)
    bias = dev(synth.weights(1, N, 7)[0] * 10)
    y8 = {}
    for plan in ("s1", "s1k"):
        B.mnnq_debug_set("MNNQ_PREFILL_TILE", plan)
        try:
            y8[plan] = B.mnnq_linear_prefill(packed, N, K, xq, sx, bias=bias)
        finally:
            B.mnnq_debug_set("MNNQ_PREFILL_TILE", None)
    if tile:
        B.mnnq_debug_set("MNNQ_PREFILL_TILE", tile)
    try:
        y16 = B.mnnq_linear_prefill_f16(packed, N, K, xq.to(torch.float16), bias=bias, row_scale=sx)
    finally:
        B.mnnq_debug_set("MNNQ_PREFILL_TILE", None)
    if tile == "":
        assert torch.equal(y8["s1"], y16) or torch.equal(y8["s1k"], y16)
    else:
        assert torch.equal(y8["s1k" if tile.endswith("k") else "s1"], y16)


def test_prefill_f16_rows_do_not_leak_into_each_other():
    # Odd number of groups: the padding group of a row must not pick up the next row's data.
    M, N, K = 40, 32, 192
    W = synth.weights(N, K, 910)
    x16 = synth.activations_f16(M, K, 911)
    q, s, z = oracle.quant_weights(W)
    y_o = oracle.linear_w4a16(x16, q, s, z)
    bad = x16.copy()
    bad[7, :] = np.float16(np.inf)
    packed = B.mnnq_pack_weights(dev(W))
    y = host(B.mnnq_linear_prefill_f16(packed, N, K, dev(bad)))
    keep = np.arange(M) != 7
    assert np.isfinite(y[keep]).all()
    assert np.abs(y[keep] - y_o[keep]).max() <= TOL_A16 * np.abs(y_o).max()


def test_w4a16_one_hot_exact_weights():
    # x = e_j in fp16: the result is the dequantized column, to fp32 rounding.
    N, K = 32, 128
    W = synth.weights(N, K, 77)
    q, s, z = oracle.quant_weights(W)
    what = oracle.dequant(q, s, z)
    packed = B.mnnq_pack_weights(dev(W))
    for j in (0, 17, 64, 127):
        x16 = np.zeros((1, K), np.float16); x16[0, j] = 1.0
        y = host(B.mnnq_linear_decode_f16(packed, N, K, dev(x16[0])))
        np.testing.assert_allclose(y, what[:, j], rtol=1e-6, atol=0)
        y = host(B.mnnq_linear_prefill_f16(packed, N, K, dev(x16)))
        np.testing.assert_allclose(y[0], what[:, j], rtol=1e-6, atol=0)


@pytest.mark.parametrize("K", [53248, 79872, 126976])
def test_decode_rows_beyond_64k_of_lds(K):
    """Rows whose int8 image needs more than the default 64 KiB of LDS (e.g. K = 53248, the down projection
    of a 405B-class model): plain and fused GEMV, a few tokens, the accumulators and the fp16-activation GEMV."""
    N, M = 144, 3
    note("long rows", N, K)
    W, x, q, s, z, xq, sx = _layer(N, K, M, 1300 + K)
    acc_o, y_o = oracle.linear_w4a8(xq, sx, q, s, z)
    tol = TOL_A8 * np.abs(y_o).max()
    packed = B.mnnq_pack_weights(dev(W))
    xqd, sxd = dev(xq), dev(sx)
    y0 = host(B.mnnq_linear_decode(packed, N, K, xqd[0].contiguous(), sxd[:1].contiguous()))
    assert np.abs(y0 - y_o[0]).max() <= tol
    yf = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x[0])))
    assert np.abs(yf - y_o[0]).max() <= tol
    ws = torch.empty(B.mnnq_workspace_size(1, N, K), dtype=torch.uint8, device="cuda:0")
    yw = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x[0]), workspace=ws))
    assert np.abs(yw - y_o[0]).max() <= tol
    assert np.array_equal(host(B.mnnq_linear_acc_debug(packed, N, K, xqd, False)), acc_o)
    ys = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd))          # few tokens: the streaming kernel
    assert np.abs(ys - y_o).max() <= tol
    if K <= 79872:
        x16 = x.astype(np.float16)
        y16_o = oracle.linear_w4a16(x16, q, s, z)
        y16 = host(B.mnnq_linear_decode_f16(packed, N, K, dev(x16[0])))
        assert np.abs(y16 - y16_o[0]).max() <= TOL_A16 * np.abs(y16_o).max()
    else:
        with pytest.raises(B.MnnqError):
            B.mnnq_linear_decode_f16(packed, N, K, dev(x.astype(np.float16)[0]))
