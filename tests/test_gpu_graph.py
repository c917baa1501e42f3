"""The library's calls inside a HIP graph: the benchmark times graph replays, and callers capture
decode loops.  Every replay must reproduce the eager result bit for bit, also where a call issues
more than one kernel (split of K over two workgroups: a zero-fill kernel in front of the GEMM;
fused calls: quantizer kernel + GEMV / GEMM), with eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

from paper_2506_10443_amd import binding as B, synth

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def test_replays_equal_eager_results():
    print("graph replays", flush=True)
    cases = []
    # (M, N, K): few tokens, tiled GEMM, and a long-row shape that takes the two-workgroup K split
    for M, N, K in ((1, 272, 1536), (8, 272, 1536), (200, 400, 1024), (100, 144, 8192)):
        W = dev(synth.weights(N, K, 40 + M))
        x = dev(synth.activations(M, K, 41 + M, outliers=True))
        cases.append((M, N, K, B.mnnq_pack_weights(W), x))
    outs = []
    ws = torch.empty(max(B.mnnq_workspace_size(M, N, K) for M, N, K, _, _ in cases), dtype=torch.uint8, device="cuda:0")

    def run_all(store):
        for i, (M, N, K, packed, x) in enumerate(cases):
            xq, sx = store[i]["xq"], store[i]["sx"]
            B.mnnq_quant_act(x, want_xsum=False, out=(xq, sx, None))
            if M == 1:
                B.mnnq_linear_decode(packed, N, K, xq[0], sx, out=store[i]["y"][0])
                B.mnnq_linear_decode_fused(packed, N, K, x[0], out=store[i]["yf"][0], workspace=ws)
                B.mnnq_linear_decode_o16(packed, N, K, xq[0], sx, out=store[i]["y16"][0])
            else:
                B.mnnq_linear_prefill(packed, N, K, xq, sx, out=store[i]["y"])
                B.mnnq_linear_prefill_fused(packed, N, K, x, out=store[i]["yf"], workspace=ws)
                B.mnnq_linear_prefill_o16(packed, N, K, xq, sx, out=store[i]["y16"])
            B.mnnq_linear_prefill_f16(packed, N, K, x.to(torch.float16), out=store[i]["ya"])

    def buffers():
        return [dict(xq=torch.empty((M, K), dtype=torch.int8, device="cuda:0"),
                     sx=torch.empty((M,), dtype=torch.float32, device="cuda:0"),
                     y=torch.empty((M, N), dtype=torch.float32, device="cuda:0"),
                     yf=torch.empty((M, N), dtype=torch.float32, device="cuda:0"),
                     ya=torch.empty((M, N), dtype=torch.float32, device="cuda:0"),
                     y16=torch.empty((M, N), dtype=torch.float16, device="cuda:0")) for M, N, K, _, _ in cases]

    eager = buffers()
    run_all(eager)
    torch.cuda.synchronize()
    ref = [{k: v.clone() for k, v in b.items()} for b in eager]

    graphed = buffers()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        run_all(graphed)              # warm-up on the capture stream
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        run_all(graphed)
    for rep in range(4):
        for b in graphed:             # poison the outputs, then some eager work and a sync between replays
            for k in ("y", "yf", "ya", "y16", "xq"):
                b[k].fill_(3)
        run_all(eager)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for i, b in enumerate(graphed):
            for k in ("xq", "sx", "y", "yf", "ya", "y16"):
                assert torch.equal(b[k], ref[i][k]), (rep, i, k)
