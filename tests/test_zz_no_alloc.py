"""The entry point that allocates nothing (mnnq_linear_prefill_fused_static) against the entry point
it is a variant of (mnnq_linear_prefill_fused with a caller's workspace), through the C-ABI: same
kernels, so the outputs must be identical bit for bit; both are also held to the oracle's tolerance.
Two calls in a row on the library's one scratch array, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2506_10443_amd import binding as B, synth

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def test_static_scratch_entry_point_matches_the_workspace_call():
    N, K = 1536, 1536
    W = synth.weights(N, K, 2201)
    q, s, z = oracle.quant_weights(W)
    packed = B.mnnq_pack_weights(dev(W))
    bias = (0.5 * np.random.default_rng(2202).standard_normal(N)).astype(np.float32)
    L = B.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for M, seed in ((200, 2203), (40, 2204)):     # the second call is smaller: stale codes lie behind its own
        print("static scratch call: M", M, "N", N, "K", K, flush=True)
        x = synth.activations(M, K, seed, outliers=True)
        xd, bd = dev(x), dev(bias)
        y_ws = B.mnnq_linear_prefill_fused(packed, N, K, xd, bias=bd)
        y_st = torch.empty((M, N), dtype=torch.float32, device="cuda:0")
        y_st.fill_(float("nan"))
        rc = L.mnnq_linear_prefill_fused_static(packed.data_ptr(), M, N, K, 64, 0, xd.data_ptr(), bd.data_ptr(),
                                                y_st.data_ptr(), stream)
        assert rc == 0, rc
        torch.cuda.synchronize()
        assert torch.equal(y_st, y_ws)
        xq_o, sx_o, _ = oracle.quant_act(x)
        _, y_o = oracle.linear_w4a8(xq_o, sx_o, q, s, z, bias=bias)
        err = np.abs(y_st.cpu().numpy() - y_o).max()
        assert err <= 1e-5 * np.abs(y_o).max(), (err, np.abs(y_o).max())


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    L = B.lib()
    cap = B.mnnq_static_scratch_bytes()
    assert cap == 32 << 20
    FAKE = 0x10000
    # 4096 x 8192 codes alone fill the array; the scales do not fit behind them
    assert L.mnnq_linear_prefill_fused_static(FAKE, 4096, 16, 8192, 64, 0, FAKE, None, FAKE, None) == -4
    assert L.mnnq_linear_prefill_fused_static(None, 4, 16, 128, 64, 0, FAKE, None, FAKE, None) == -1
    assert L.mnnq_linear_prefill_fused_static(FAKE, 4, 16, 128, 64, 0, FAKE + 4, None, FAKE, None) == -5
