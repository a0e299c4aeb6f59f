"""The library enqueues kernels only (no allocation, no host copy, no synchronisation), so its calls can be recorded
into a HIP graph.  The graph is replayed several times with eager work and changed inputs in between, and every
replay is checked against the eager result and against the oracle."""
import numpy as np
import pytest

from paper_2604_00529_amd import synth
from test_gpu_parity import assert_same_values, mx, to_gpu, to_host  # noqa: F401  (mx is the module fixture)

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager_and_oracle(mx, oracle):
    import torch
    fa, ft, f6 = mx.make_format("e4m3"), mx.make_format("e2m1"), mx.make_format("e3m2")
    sizes = [(64, 1024), (33, 512), (128, 2048)]
    rng = np.random.default_rng(91)
    host = [(rng.standard_normal(s) * 0.05).astype(np.float32) for s in sizes]
    dense = [to_gpu(h) for h in host]
    anchors = [mx.mx_quantize(d, fa) for d in dense]                       # (codes, scales), written in place below
    t4 = [(torch.empty((c.shape[0], c.shape[1], 16), dtype=torch.uint8, device="cuda"), torch.empty_like(s)) for c, s in anchors]
    t6 = [(torch.empty((c.shape[0], c.shape[1], 24), dtype=torch.uint8, device="cuda"), torch.empty_like(s)) for c, s in anchors]
    nblocks = sum(int(s.numel()) for _, s in anchors)
    ws = torch.empty(mx.binding.lib().mx_slice_and_scale_batched_workspace(len(anchors), nblocks), dtype=torch.uint8, device="cuda")
    fq = [torch.empty_like(d) for d in dense]
    # the fused GEMM too (its tiled kernel: M > 48; one tile and 16 K-steps, so with the workspace that the binding
    # allocates -- from torch's pool of the graph while capturing -- K goes in two slices and a second kernel adds them):
    # activations = tensor 2 (128 x 2048), weight = its first 48 rows
    c_out = torch.empty((128, 48), dtype=torch.float32, device="cuda")
    # and its streaming kernels: 33 x 512 activations (tensor 1) against 32 of its rows, 16 rows of tensor 0 against 64
    c_mid = torch.empty((33, 32), dtype=torch.float32, device="cuda")
    c_dec = torch.empty((16, 64), dtype=torch.float32, device="cuda")
    # and its workspace path (W sliced into a lent workspace, then the 256-row-tile kernel): 768 x 16384 x 128, operands
    # quantized once outside the graph
    big_a = mx.mx_quantize(to_gpu(rng.standard_normal((768, 128)).astype(np.float32)), fa)
    big_w = mx.mx_quantize(to_gpu((rng.standard_normal((16384, 128)) * 0.02).astype(np.float32)), fa)
    big_ws = torch.empty(mx.binding.lib().mx_gemm_ss_fp4_workspace(16384, 128), dtype=torch.uint8, device="cuda")
    c_big = torch.empty((768, 16384), dtype=torch.float32, device="cuda")
    c_big_fly = mx.mx_gemm_ss_fp4(big_a[0], big_a[1], big_w[0], big_w[1], workspace=False)
    batch4 = mx.SsBatch(anchors, fa, ft, t4, ws)
    batch46 = mx.SsBatch(anchors, fa, [f6, ft], [[t6[i], t4[i]] for i in range(len(anchors))], ws)

    def work():
        for d, (ac, asc) in zip(dense, anchors):
            mx.mx_quantize(d, fa, ac, asc)                                 # Eq. (1), (2)
        batch4.run()                                                       # Eq. (6), all tensors in one launch
        batch46.run()                                                      # two targets in one pass (overwrites t4 alike)
        for d, o in zip(dense, fq):
            mx.mx_fake_quant(d, ft, fa, o)                                 # Eq. (7)
        mx.mx_gemm_ss_fp4(anchors[2][0], anchors[2][1], anchors[2][0][:48], anchors[2][1][:48], c_out)
        mx.mx_gemm_ss_fp4(anchors[1][0], anchors[1][1], anchors[1][0][:32], anchors[1][1][:32], c_mid)
        mx.mx_gemm_ss_fp4(anchors[0][0][:16], anchors[0][1][:16], anchors[0][0], anchors[0][1], c_dec)
        mx.mx_gemm_ss_fp4(big_a[0], big_a[1], big_w[0], big_w[1], c_big, workspace=big_ws)

    work()                                                                 # eager once (also sets kernel attributes)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        work()
    for rep in range(3):
        # new inputs, some eager work of the program's own, then the replay
        for i, d in enumerate(dense):
            host[i] = (rng.standard_normal(sizes[i]) * (0.02 * (rep + 1))).astype(np.float32)
            d.copy_(to_gpu(host[i]))
        (dense[0] * 2).sum().item()
        for t in t4 + t6:
            t[0].fill_(0xA5)
            t[1].fill_(0xA5)
        c_out.zero_()
        c_mid.zero_()
        c_dec.zero_()
        c_big.zero_()
        big_ws.fill_(0x5A)
        g.replay()
        torch.cuda.synchronize()
        got = ([(to_host(a), to_host(b)) for a, b in t4], [(to_host(a), to_host(b)) for a, b in t6], [to_host(o) for o in fq], to_host(c_out),
               to_host(c_mid), to_host(c_dec))
        assert torch.equal(c_big.view(torch.int32), c_big_fly.view(torch.int32)), rep   # (bit-identical to the on-the-fly kernels)
        for i, h in enumerate(host):
            wc, wsc = oracle.quantize(h, "e4m3")
            assert np.array_equal(to_host(anchors[i][0]), wc) and np.array_equal(to_host(anchors[i][1]), wsc), (rep, i)
            c4, s4 = oracle.slice_and_scale(wc, wsc, "e4m3", "e2m1")
            c6, s6 = oracle.slice_and_scale(wc, wsc, "e4m3", "e3m2")
            assert np.array_equal(got[0][i][0], c4) and np.array_equal(got[0][i][1], s4), (rep, i)
            assert np.array_equal(got[1][i][0], c6) and np.array_equal(got[1][i][1], s6), (rep, i)
            assert_same_values(got[2][i], oracle.fake_quant(h, "e2m1", anchor="e4m3"))
        # eager run on the same inputs: identical bits, the GEMM included
        work()
        torch.cuda.synchronize()
        assert np.array_equal(to_host(c_out).view(np.uint32), got[3].view(np.uint32)), rep
        assert np.array_equal(to_host(c_mid).view(np.uint32), got[4].view(np.uint32)), rep
        assert np.array_equal(to_host(c_dec).view(np.uint32), got[5].view(np.uint32)), rep
        assert np.abs(got[4]).max() > 0 and np.abs(got[5]).max() > 0
        for i in range(len(anchors)):
            assert np.array_equal(to_host(t4[i][0]), got[0][i][0]) and np.array_equal(to_host(t6[i][0]), got[1][i][0])
