"""GPU parity of the byte form of int8 weights (mode MNNQ_W8_MIN_FLOAT | MNNQ_NATIVE_8BIT: the codes of
Eq. 1 with clip range 0..255 stored as bytes q8 - 128, 1.125 bytes per weight) against the oracle's
O9 / O10, through the C-ABI.  Codes, steps and minima bit-exact; y within 1e-5 * max|y|; the calls that
read the plane form refuse it."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_10443_amd import binding as B, synth

pytestmark = pytest.mark.gpu
W8 = B.MODE_W8_MIN_FLOAT
W8N = B.MODE_W8_MIN_FLOAT | B.NATIVE_8BIT
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
    note("int8 bytes pack", N, K)
    W = _weights(N, K, 1900 + N + K)
    q, s, mn = oracle.quant_weights8(W)
    assert q.max() == 255 and q.min() == 0
    packed = B.mnnq_pack_weights(dev(W), mode=W8N)
    assert packed.numel() == N * K + 8 * N * (K // 64)        # a byte per code, fp32 step and minimum per group
    assert packed.numel() == B.mnnq_packed_size(N, K, 64, W8N) < B.mnnq_packed_size(N, K, 64, W8)
    q2, s2, m2 = B.mnnq_unpack_weights(packed, N, K, mode=W8N)
    assert np.array_equal(host(q2), q)
    assert np.array_equal(host(s2).view(np.uint32), s.view(np.uint32))
    assert np.array_equal(host(m2).view(np.uint32), mn.view(np.uint32))
    assert torch.equal(B.mnnq_pack_from_quantized(dev(q), dev(s), dev(mn), mode=W8N), packed)
    # the same canonical arrays as the plane form holds
    qp, sp, mp = B.mnnq_unpack_weights(B.mnnq_pack_weights(dev(W), mode=W8), N, K, mode=W8)
    assert torch.equal(qp, q2) and torch.equal(sp, s2) and torch.equal(mp, m2)
    with pytest.raises(B.MnnqError):
        B.mnnq_pack_weights(dev(W[:, :64].copy()), mode=W8N)   # K must be a multiple of 128
    with pytest.raises(B.MnnqError):
        B.mnnq_pack_weights(dev(W), mode=B.MODE_W4_MIN_FLOAT | B.NATIVE_8BIT)   # a form of the int8 weights only


SHAPES = [(1, 16, 128), (7, 48, 384), (16, 144, 9472), (33, 272, 640), (130, 144, 1536), (300, 400, 1024),
          (64, 1024, 4096), (129, 144, 8192), (513, 1040, 896), (3, 64, 18944), (2, 32, 53248)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_linear_matches_oracle(M, N, K):
    note("int8 bytes linear", M, N, K)
    W = _weights(N, K, 1910 + M + N + K)
    x = synth.activations(M, K, 1911 + M + N + K, outliers=True)
    q, s, mn = oracle.quant_weights8(W)
    xq, sx, _ = oracle.quant_act(x)
    bias = synth.weights(1, N, 9)[0] * 10
    _, y_o = oracle.linear_w8a8(xq, sx, q, s, mn, bias=bias, want_acc=False)
    tol = TOL * np.abs(y_o).max()
    packed = B.mnnq_pack_weights(dev(W), mode=W8N)
    xqd, sxd, bd = dev(xq), dev(sx), dev(bias)
    y = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd, mode=W8N))
    assert np.abs(y - y_o).max() <= tol, (np.abs(y - y_o).max(), tol)
    # the tile plans of the int8 GEMM for this weight form: one or two K parts, four or eight waves per part,
    # K split over two workgroups (long rows only)
    for cfg in ("s1", "s1k", "s2", "s2k", "v1", "v1k"):
        B.mnnq_debug_set("MNNQ_PREFILL_TILE", cfg)
        try:
            y2 = host(B.mnnq_linear_prefill(packed, N, K, xqd, sxd, bias=bd, mode=W8N))
        finally:
            B.mnnq_debug_set("MNNQ_PREFILL_TILE", None)
        assert np.abs(y2 - y_o).max() <= tol, cfg
    # fused call (quantizer as a kernel of its own, through the workspace)
    yf = host(B.mnnq_linear_prefill_fused(packed, N, K, dev(x), bias=bd, mode=W8N))
    assert np.array_equal(yf, y)
    # decode: every K split the kernel is built for, plain and with the quantizer inside
    for m in sorted({0, M - 1}):
        for ks in (None, "1", "2", "4", "8", "16"):
            B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", ks)
            try:
                # (a forced split whose staging of the row does not fit the LDS is refused, not run)
                if ks is not None and B.mnnq_plan_debug(1, 1, N, K, mode=W8N)[4] > 160 * 1024:
                    with pytest.raises(B.MnnqError):
                        B.mnnq_linear_decode(packed, N, K, xqd[m].contiguous(), sxd[m:m + 1].contiguous(), bias=bd, mode=W8N)
                    continue
                y0 = host(B.mnnq_linear_decode(packed, N, K, xqd[m].contiguous(), sxd[m:m + 1].contiguous(), bias=bd, mode=W8N))
                yq = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x[m]), bias=bd, mode=W8N))
            finally:
                B.mnnq_debug_set("MNNQ_DECODE_KSPLIT", None)
            assert np.abs(y0 - y_o[m]).max() <= tol, (m, ks)
            assert np.abs(yq - y_o[m]).max() <= tol, (m, ks)
    # binary16 output: the fp32 result rounded once
    y16 = host(B.mnnq_linear_decode_o16(packed, N, K, xqd[0].contiguous(), sxd[:1].contiguous(), bias=bd, mode=W8N))
    y32 = host(B.mnnq_linear_decode(packed, N, K, xqd[0].contiguous(), sxd[:1].contiguous(), bias=bd, mode=W8N))
    assert np.array_equal(y16, y32.astype(np.float16))
    p16 = host(B.mnnq_linear_prefill_o16(packed, N, K, xqd, sxd, bias=bd, mode=W8N))
    # (long rows: the fp32 call may split K over two workgroups, the binary16 call never does - same sums
    # in another order, so the comparison allows the fp32 tolerance next to half a binary16 unit)
    assert (np.abs(p16.astype(np.float32) - y) <= tol + 2.0 ** -11 * np.abs(y)).all()


def test_calls_that_read_the_plane_form_refuse_the_byte_form():
    N, K, M = 64, 256, 40
    W = _weights(N, K, 1950)
    packed = B.mnnq_pack_weights(dev(W), mode=W8N)
    x16 = dev(synth.activations_f16(M, K, 1951))
    xq = dev(oracle.quant_act(synth.activations(M, K, 1952))[0])
    for call in (lambda: B.mnnq_linear_prefill_f16(packed, N, K, x16, mode=W8N),
                 lambda: B.mnnq_linear_decode_f16(packed, N, K, x16[0].contiguous(), mode=W8N),
                 lambda: B.mnnq_linear_acc_debug(packed, N, K, xq, True, mode=W8N),
                 lambda: B.mnnq_linear_acc_debug(packed, N, K, xq, False, mode=W8N)):
        with pytest.raises(B.MnnqError) as e:
            call()
        assert e.value.status == -3


@pytest.mark.parametrize("name", ["gateup", "down"])
def test_full_size_block_layers(name):
    """Qwen2-7B's gate|up and down in the byte form at the sizes `bench.py --weight-mode int8n` times:
    sampled prefill outputs (M = 1024) and the first row through both single-token calls."""
    model, M, seed = "qwen2-7b", 1024, 1977
    parts = [synth.weights(*synth.MODELS[model]["layers"][p], synth.layer_seed(model, 0, p)) for p in synth.fused_parts(name)]
    W = np.concatenate(parts) if len(parts) > 1 else parts[0]
    del parts
    N, K = W.shape
    note("full-size int8 bytes", name, M, N, K)
    x = synth.activations(M, K, seed, outliers=True)
    q, s, mn = oracle.quant_weights8(W)
    xq_o, sx_o, _ = oracle.quant_act(x)
    packed = B.mnnq_pack_weights(dev(W), mode=W8N)
    del W
    xq, sx = dev(xq_o), dev(sx_o)
    y = host(B.mnnq_linear_prefill(packed, N, K, xq, sx, mode=W8N))
    rng = np.random.default_rng(seed)
    ms = np.concatenate([rng.integers(0, M, 8192), [0, 0, M - 1, M - 1]])
    ns = np.concatenate([rng.integers(0, N, 8192), [0, N - 1, 0, N - 1]])
    _, y_s = oracle.linear_w8a8_sampled(xq_o, sx_o, q, s, mn, ms, ns, want_acc=False)
    ymax = np.abs(y).max()
    assert np.isfinite(y).all()
    assert np.abs(y[ms, ns] - y_s).max() <= TOL * ymax
    n_all = np.arange(N)
    _, y0 = oracle.linear_w8a8_sampled(xq_o, sx_o, q, s, mn, np.zeros(N, dtype=np.int64), n_all, want_acc=False)
    tol0 = TOL * np.abs(y0).max()
    yd = host(B.mnnq_linear_decode(packed, N, K, xq[0].contiguous(), sx[:1].contiguous(), mode=W8N))
    assert np.abs(yd - y0).max() <= tol0
    yf = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x[0]), mode=W8N))
    assert np.abs(yf - y0).max() <= tol0
    assert np.abs(y[0] - y0).max() <= tol0


def test_full_size_lm_head_decode():
    # The layer the paper singles out for int8: the LM head.
    N, K = synth.MODELS["qwen2-7b"]["lm_head"]
    note("int8 bytes lm_head", N, K)
    W = synth.weights(N, K, synth.layer_seed("qwen2-7b", 0, "lm_head"))
    x = synth.activations(1, K, 61)
    q, s, mn = oracle.quant_weights8(W)
    xq_o, sx_o, _ = oracle.quant_act(x)
    _, y_o = oracle.linear_w8a8(xq_o, sx_o, q, s, mn, want_acc=False)
    packed = B.mnnq_pack_weights(dev(W), mode=W8N)
    del W
    q2, s2, m2 = B.mnnq_unpack_weights(packed, N, K, mode=W8N)
    assert np.array_equal(host(q2), q) and np.array_equal(host(m2).view(np.uint32), mn.view(np.uint32))
    assert np.array_equal(host(s2).view(np.uint32), s.view(np.uint32))
    del q2, s2, m2
    y = host(B.mnnq_linear_decode(packed, N, K, dev(xq_o[0]), dev(sx_o), mode=W8N))
    assert np.abs(y - y_o[0]).max() <= TOL * np.abs(y_o).max()
    ws = torch.empty(B.mnnq_workspace_size(1, N, K, 64, W8N), dtype=torch.uint8, device="cuda:0")
    yf = host(B.mnnq_linear_decode_fused(packed, N, K, dev(x[0]), workspace=ws, mode=W8N))
    assert np.array_equal(yf, y)      # beyond 96 MiB the fused call runs the quantizer as a kernel of its own
