"""GPU parity of the GEMM on the fp6 matrix instructions (packed buffers with the matrix-core plane,
mode MNNQ_W4_ZP_INT | MNNQ_WITH_MATRIX_PLANE) against the CPU oracle: the int32 group accumulators
bit-exact for every tile plan, y within 1e-5 * max|y|, and bit-identical codes in front of the plane."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_10443_amd import binding as B, synth

pytestmark = pytest.mark.gpu

MODE = B.MODE_W4_ZP_INT | B.WITH_MATRIX_PLANE
TOL_A8 = 1e-5


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def note(*a):
    print(*a, flush=True)


@pytest.fixture(autouse=True)
def _auto_plan():
    yield
    B.mnnq_debug_set("MNNQ_PREFILL6_PLAN", None)


def make(N, K, M, seed, special=False):
    W = synth.weights(N, K, seed)
    if special:
        W[0, :64] = 0.0
        W[1, :64] = np.abs(W[1, :64]) + 0.01
        W[2, :64] = -np.abs(W[2, :64]) - 0.01
        t = np.zeros(64, np.float32); t[:9] = [-3.5, 11.5, 0.5, 1.5, 2.5, -0.5, -2.5, -1.5, 0.0]
        W[4, :64] = t
    x = synth.activations(M, K, seed + 1, outliers=True)
    if special:
        x[0, :] = 0.0                       # zero row
        x[1, :] = 127.0                     # every code at the top of the range
        x[2, ::2] = -127.0; x[2, 1::2] = 127.0
        x[3, :] = -1.0
    q, s, z = oracle.quant_weights(W)
    xq, sx, _ = oracle.quant_act(x)
    return W, x, q, s, z, xq, sx


def test_plane_leaves_the_chunk_layout_alone():
    N, K = 272, 1536
    W = synth.weights(N, K, 4101)
    p0 = B.mnnq_pack_weights(dev(W))
    p1 = B.mnnq_pack_weights(dev(W), mode=MODE)
    assert p1.numel() == B.mnnq_packed_size(N, K, 64, MODE) > p0.numel()
    assert torch.equal(p1[:p0.numel()], p0)
    q, s, z = oracle.quant_weights(W)
    qg, sg, zg = B.mnnq_unpack_weights(p1, N, K, mode=MODE)
    assert np.array_equal(qg.cpu().numpy(), q) and np.array_equal(sg.cpu().numpy(), s) and np.array_equal(zg.cpu().numpy(), z)
    # the import call builds the same plane
    p2 = B.mnnq_pack_from_quantized(dev(q), dev(s), dev(z), mode=MODE)
    assert torch.equal(p2, p1)


@pytest.mark.parametrize("plan", [0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("M,N,K", [(200, 400 - 400 % 16, 1536), (129, 592, 448), (40, 48, 64), (333, 1024, 192), (150, 704, 320)])
def test_prefill6_every_plan(plan, M, N, K):
    note("prefill6 plan", plan, "M", M, "N", N, "K", K)
    W, x, q, s, z, xq, sx = make(N, K, M, 4200 + plan, special=True)
    acc_o, y_o = oracle.linear_w4a8(xq, sx, q, s, z)
    packed = B.mnnq_pack_weights(dev(W), mode=MODE)
    ws = torch.empty(B.mnnq_workspace_size(M, N, K, 64, MODE), dtype=torch.uint8, device="cuda:0")
    B.mnnq_debug_set("MNNQ_PREFILL6_PLAN", plan)
    assert B.mnnq_plan_debug(0, M, N, K, mode=MODE)[7] == 6
    y = B.mnnq_linear_prefill(packed, N, K, dev(xq), dev(sx), mode=MODE, workspace=ws).cpu().numpy()
    err = np.abs(y - y_o).max()
    assert err <= TOL_A8 * np.abs(y_o).max(), (err, np.abs(y_o).max())
    # the same call again gives the same bits
    y2 = B.mnnq_linear_prefill(packed, N, K, dev(xq), dev(sx), mode=MODE, workspace=ws).cpu().numpy()
    assert np.array_equal(y, y2)


@pytest.mark.parametrize("M,N,K", [(200, 400 - 400 % 16, 1536), (129, 592, 448), (40, 48, 64)])
def test_prefill6_deeper_rings(M, N, K):
    """Three and four stages in the LDS rings (MNNQ_PREFILL6_STAGES) for the plans that have them."""
    W, x, q, s, z, xq, sx = make(N, K, M, 4250, special=True)
    _, y_o = oracle.linear_w4a8(xq, sx, q, s, z)
    packed = B.mnnq_pack_weights(dev(W), mode=MODE)
    ws = torch.empty(B.mnnq_workspace_size(M, N, K, 64, MODE), dtype=torch.uint8, device="cuda:0")
    try:
        for plan, stages in ((0, 3), (0, 4), (1, 3), (1, 4), (2, 3), (3, 3)):
            note("prefill6 plan", plan, "stages", stages, "M", M, "N", N, "K", K)
            B.mnnq_debug_set("MNNQ_PREFILL6_PLAN", plan)
            B.mnnq_debug_set("MNNQ_PREFILL6_STAGES", stages)
            y = B.mnnq_linear_prefill(packed, N, K, dev(xq), dev(sx), mode=MODE, workspace=ws).cpu().numpy()
            assert np.abs(y - y_o).max() <= TOL_A8 * np.abs(y_o).max(), (plan, stages)
    finally:
        B.mnnq_debug_set("MNNQ_PREFILL6_STAGES", None)


@pytest.mark.parametrize("M,N,K", [(200, 400 - 400 % 16, 1536), (129, 592, 448), (40, 48, 64)])
def test_prefill6_accumulators_bit_exact(M, N, K):
    note("prefill6 acc", "M", M, "N", N, "K", K)
    W, x, q, s, z, xq, sx = make(N, K, M, 4300, special=True)
    acc_o, _ = oracle.linear_w4a8(xq, sx, q, s, z)
    packed = B.mnnq_pack_weights(dev(W), mode=MODE)
    acc = B.mnnq_linear_acc_debug_planes(packed, N, K, dev(xq), MODE).cpu().numpy()
    assert np.array_equal(acc, acc_o)


def test_prefill6_every_int8_code_bit_exact():
    """Caller-supplied codes over the whole int8 range, -128 included (the activation quantizer never
    produces it): every value in every position of a group, accumulators against the oracle."""
    M, N, K = 64, 96, 256
    rng = np.random.default_rng(4350)
    W = synth.weights(N, K, 4351)
    q, s, z = oracle.quant_weights(W)
    xq = rng.integers(-128, 128, (M, K)).astype(np.int8)
    xq[0, :] = -128
    xq[1, :256] = np.arange(-128, 128).astype(np.int8)
    xq[2, :] = np.where(np.arange(K) % 2 == 0, -16, 16).astype(np.int8)
    xq[3, :] = np.where(np.arange(K) % 2 == 0, -15, 15).astype(np.int8)
    sx = np.ones(M, np.float32)
    acc_o, y_o = oracle.linear_w4a8(xq, sx, q, s, z)
    packed = B.mnnq_pack_weights(dev(W), mode=MODE)
    acc = B.mnnq_linear_acc_debug_planes(packed, N, K, dev(xq), MODE).cpu().numpy()
    assert np.array_equal(acc, acc_o)
    B.mnnq_debug_set("MNNQ_PREFILL6_PLAN", 0)
    ws = torch.empty(B.mnnq_workspace_size(M, N, K, 64, MODE), dtype=torch.uint8, device="cuda:0")
    y = B.mnnq_linear_prefill(packed, N, K, dev(xq), dev(sx), mode=MODE, workspace=ws).cpu().numpy()
    assert np.abs(y - y_o).max() <= TOL_A8 * np.abs(y_o).max()


def test_prefill6_bias_fused_and_fallbacks():
    M, N, K = 150, 512, 1536
    B.mnnq_debug_set("MNNQ_PREFILL6_PLAN", 0)       # (so few tiles would go to the int8 GEMM otherwise)
    W, x, q, s, z, xq, sx = make(N, K, M, 4400)
    bias = (0.5 * np.random.default_rng(4401).standard_normal(N)).astype(np.float32)
    _, y_o = oracle.linear_w4a8(xq, sx, q, s, z, bias=bias)
    packed = B.mnnq_pack_weights(dev(W), mode=MODE)
    tol = TOL_A8 * np.abs(y_o).max()
    # fused call (quantizer inside), workspace brought by the wrapper
    yf = B.mnnq_linear_prefill_fused(packed, N, K, dev(x), bias=dev(bias), mode=MODE).cpu().numpy()
    assert np.abs(yf - y_o).max() <= tol
    # no workspace: the int8 GEMM on the chunk layout in front of the plane
    y8 = B.mnnq_linear_prefill(packed, N, K, dev(xq), dev(sx), bias=dev(bias), mode=MODE).cpu().numpy()
    assert np.abs(y8 - y_o).max() <= tol
    # decode and the few-token path read the chunk layout too
    y1 = B.mnnq_linear_decode(packed, N, K, dev(xq[0]), dev(sx[:1]), bias=dev(bias), mode=MODE).cpu().numpy()
    assert np.abs(y1 - y_o[0]).max() <= TOL_A8 * np.abs(y_o[0]).max()
    # the entry point without allocations takes the plane too
    ys = B.mnnq_linear_prefill_fused_static(packed, N, K, dev(x), bias=dev(bias), mode=MODE).cpu().numpy()
    assert np.array_equal(ys, yf)


@pytest.mark.parametrize("plan", [0, 1, 2, 5])
def test_prefill6_binary16_output_and_bias(plan):
    """The output stage of the fp6 GEMM (row segments through an LDS patch, 128-bit stores; 64-bit ones for
    binary16) on ragged shapes: the binary16 call must give the fp32 result rounded once."""
    for M, N, K in ((150, 512, 1536), (333, 1040, 192), (77, 336, 320)):
        note("prefill6 out16 plan", plan, M, N, K)
        W, x, q, s, z, xq, sx = make(N, K, M, 4600 + plan)
        bias = (0.5 * np.random.default_rng(4601).standard_normal(N)).astype(np.float32)
        _, y_o = oracle.linear_w4a8(xq, sx, q, s, z, bias=bias)
        packed = B.mnnq_pack_weights(dev(W), mode=MODE)
        B.mnnq_debug_set("MNNQ_PREFILL6_PLAN", plan)
        assert B.mnnq_plan_debug(0, M, N, K, mode=MODE)[7] == 6
        y32 = B.mnnq_linear_prefill_fused(packed, N, K, dev(x), bias=dev(bias), mode=MODE).cpu().numpy()
        assert np.abs(y32 - y_o).max() <= TOL_A8 * np.abs(y_o).max()
        y16 = B.mnnq_linear_prefill_fused_o16(packed, N, K, dev(x), bias=dev(bias), mode=MODE).cpu().numpy()
        assert y16.dtype == np.float16 and np.array_equal(y16, y32.astype(np.float16))


def test_few_output_tiles_take_the_int8_gemm_unless_a_plan_is_forced():
    M, N, K = 150, 512, 4096
    assert B.mnnq_plan_debug(0, M, N, K, mode=MODE)[7] != 6
    assert B.mnnq_plan_debug(0, M, N, 1536, mode=MODE)[7] == 6      # short K: nothing to split
    assert B.mnnq_plan_debug(0, 1024, 4608, 3584, mode=MODE)[7] == 6
    B.mnnq_debug_set("MNNQ_PREFILL6_PLAN", 2)
    assert B.mnnq_plan_debug(0, M, N, K, mode=MODE)[:2] == [128, 256] and B.mnnq_plan_debug(0, M, N, K, mode=MODE)[7] == 6
    # the workspace size does not depend on the choice
    B.mnnq_debug_set("MNNQ_PREFILL6_PLAN", None)
    assert B.mnnq_workspace_size(M, N, K, 64, MODE) >= B.lib().mnnq_act_planes_size(M, K, 64) + M * K + 4 * M


def test_act_planes_and_gemm_as_separate_calls():
    M, N, K = 300, 768, 1536
    B.mnnq_debug_set("MNNQ_PREFILL6_PLAN", 0)       # (so few tiles would go to the int8 GEMM otherwise)
    W, x, q, s, z, xq, sx = make(N, K, M, 4500)
    _, y_o = oracle.linear_w4a8(xq, sx, q, s, z)
    packed = B.mnnq_pack_weights(dev(W), mode=MODE)
    ws = torch.empty(B.mnnq_workspace_size(M, N, K, 64, MODE), dtype=torch.uint8, device="cuda:0")
    y_ws = B.mnnq_linear_prefill(packed, N, K, dev(xq), dev(sx), mode=MODE, workspace=ws)
    planes = B.mnnq_act_planes(dev(xq))
    assert planes.numel() == B.lib().mnnq_act_planes_size(M, K, 64)
    y_pl = B.mnnq_linear_prefill_planes(packed, M, N, K, planes, dev(sx), mode=MODE)
    assert torch.equal(y_pl, y_ws)
    assert np.abs(y_pl.cpu().numpy() - y_o).max() <= TOL_A8 * np.abs(y_o).max()
