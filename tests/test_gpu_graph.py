"""Every entry point of the library can be captured into a HIP graph and replayed: the calls enqueue
kernels only (no allocation, no host synchronisation, no memset nodes), and the kernels are
deterministic, so each replay must reproduce the eager result bit for bit - also after the inputs
were changed in place between replays, with eager work of the same library in between."""
import numpy as np
import pytest

import gwq_synth as gs
from oracle import gwq_oracle as orc

pytestmark = pytest.mark.gpu


def _layer(seed, N, K, bits):
    rng = np.random.default_rng(seed)
    W = gs.weight(N, K, rng, planted_cols=2)
    S = gs.score_from_weight(W, rng)
    return W, S, rng


@pytest.mark.parametrize("bits", [4, 3])
def test_linear_calls_replay_from_a_graph(bits):
    import torch
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    N, K = 200, 1408
    W, S, rng = _layer(10 + bits, N, K, bits)
    P = orc.pack(W, S, bits, 10000)
    D, D2 = upload_packed(P), upload_packed(P)
    Ms = (1, 8, 16, 40, 300)                              # both decode kernels, GEMM with and without split K
    xs = [to_gpu(gs.activations(M, K, rng)) for M in Ms]
    ys = [torch.empty((M, N), dtype=torch.float16, device="cuda") for M in Ms]
    calls = [gwq.prepare_linear(D, x, y) for x, y in zip(xs, ys)]
    yb = [torch.empty((8, N), dtype=torch.float16, device="cuda") for _ in range(2)]
    calls.append(gwq.prepare_linear_batch([D, D2], [xs[1], xs[1]], yb))
    for c in calls:
        c()                                               # warm up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for c in calls:
            c()
    for trial in range(3):
        for x in xs:                                      # new inputs, in place
            x.copy_(to_gpu(gs.activations(x.shape[0], K, rng)))
        for y in ys + yb:
            y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        replayed = [y.clone() for y in ys + yb]
        for c in calls:                                   # the same work, eagerly
            c()
        torch.cuda.synchronize()
        for got, want in zip(replayed, ys + yb):
            assert torch.equal(got, want), f"replay {trial} differs from the eager result"
    ref = orc.linear_f64(P, xs[3].cpu().numpy())
    assert np.abs(ys[3].cpu().numpy() - ref).max() <= 1e-2 * np.abs(ref).max()


def test_gate_up_bf16_and_small_groups_replay_from_a_graph():
    """gwq_linear_gate_up (fused for M <= 4, two products and an elementwise kernel beyond), gwq_linear_bf16 (decode and
    GEMM) and gwq_linear on a layer with groups of 16, captured together and replayed after the inputs changed."""
    import torch
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    N, K = 176, 1024
    W, S, rng = _layer(31, N, K, 4)
    W2, S2, _ = _layer(32, N, K, 4)
    Dg, Du = upload_packed(orc.pack(W, S, 4, 10000)), upload_packed(orc.pack(W2, S2, 4, 10000))
    P16 = orc.pack(W, S, 4, 10000, 16)
    D16 = upload_packed(P16)
    Ms = (2, 12, 40)
    xs = [to_gpu(gs.activations(M, K, rng)) for M in Ms]
    xb = [x.to(torch.bfloat16) for x in xs]
    hs = [torch.empty((M, N), dtype=torch.float16, device="cuda") for M in Ms[:2]]
    yb = [torch.empty((M, N), dtype=torch.bfloat16, device="cuda") for M in Ms]
    y16 = [torch.empty((M, N), dtype=torch.float16, device="cuda") for M in Ms]
    wsb = [gwq.linear_workspace(Dg, M) for M in Ms]
    calls = [gwq.prepare_linear_gate_up(Dg, Du, xs[i], hs[i]) for i in range(2)]
    calls += [(lambda i=i: gwq.linear_bf16(Dg, xb[i], yb[i], workspace=wsb[i])) for i in range(3)]
    calls += [gwq.prepare_linear(D16, xs[i], y16[i]) for i in range(3)]
    outs = hs + yb + y16
    for c in calls:
        c()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for c in calls:
            c()
    for trial in range(3):
        for x, b in zip(xs, xb):
            x.copy_(to_gpu(gs.activations(x.shape[0], K, rng)))
            b.copy_(x)
        for y in outs:
            y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        replayed = [y.clone() for y in outs]
        for c in calls:
            c()
        torch.cuda.synchronize()
        for got, want in zip(replayed, outs):
            assert torch.equal(got, want), f"replay {trial} differs from the eager result"
    ref = orc.linear_f64(P16, xs[2].cpu().numpy())
    assert np.abs(y16[2].cpu().numpy() - ref).max() <= 1e-2 * np.abs(ref).max()


def test_pack_and_quality_replay_from_a_graph():
    import torch
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, assert_packed_equal
    N, K, bits = 96, 1280, 4
    W, S, rng = _layer(33, N, K, bits)
    Wd, Sd = to_gpu(W), to_gpu(S)
    sz = gwq.layout(N, K, bits, 128, 10000)
    ws = torch.empty(sz["pack_workspace"], dtype=torch.uint8, device="cuda")
    qws = torch.empty(sz["quality_workspace"], dtype=torch.uint8, device="cuda")
    out3 = torch.empty(3, dtype=torch.float64, device="cuda")
    D = gwq.pack(Wd, Sd, bits, 10000, workspace=ws)       # warm up; D's buffers are reused below
    gwq.quality(D, Wd, Sd, out=out3, workspace=qws)
    torch.cuda.synchronize()

    def work():
        cs = D.c_struct()
        import ctypes
        rc = gwq.lib().gwq_pack(Wd.data_ptr(), Sd.data_ptr(), 0, ctypes.byref(cs), ws.data_ptr(), ws.numel(),
                                torch.cuda.current_stream().cuda_stream)
        assert rc == 0
        gwq.quality(D, Wd, Sd, out=out3, workspace=qws)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        work()
    for trial in range(3):
        W2, S2, _ = _layer(100 + trial, N, K, bits)
        Wd.copy_(to_gpu(W2)); Sd.copy_(to_gpu(S2))
        graph.replay()
        torch.cuda.synchronize()
        P = orc.pack(W2, S2, bits, 10000)
        assert_packed_equal(D, P)
        sq, first, mx = orc.quality(P, W2, S2)
        got = out3.cpu().numpy()
        assert abs(got[0] - sq) <= 1e-11 * sq and got[2] == mx


def test_score_replays_from_a_graph():
    """gwq_score, then gwq_pack ranking what it wrote, captured together: the calibration step of one layer."""
    import ctypes
    import torch
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, assert_packed_equal
    M, N, K, bits = 150, 96, 384, 4
    W, _, rng = _layer(44, N, K, bits)
    Wd = to_gpu(W)
    dYd = to_gpu((0.05 * rng.standard_normal((M, N))).astype(np.float16))
    Xd = to_gpu(gs.activations(M, K, rng))
    Sd = torch.empty((N, K), dtype=torch.float32, device="cuda")
    ws = torch.empty(gwq.layout(N, K, bits, 128, 10000)["pack_workspace"], dtype=torch.uint8, device="cuda")
    gwq.score(dYd, Xd, out=Sd)
    D = gwq.pack(Wd, Sd, bits, 10000, workspace=ws)
    torch.cuda.synchronize()

    def work():
        gwq.score(dYd, Xd, out=Sd, alpha=0.5)
        gwq.score(dYd, Xd, out=Sd, alpha=0.5, beta=1.0)
        cs = D.c_struct()
        rc = gwq.lib().gwq_pack(Wd.data_ptr(), Sd.data_ptr(), 0, ctypes.byref(cs), ws.data_ptr(), ws.numel(),
                                torch.cuda.current_stream().cuda_stream)
        assert rc == 0

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        work()
    for trial in range(3):
        dYd.copy_(to_gpu((0.05 * rng.standard_normal((M, N))).astype(np.float16)))
        Xd.copy_(to_gpu(gs.activations(M, K, rng)))
        graph.replay()
        torch.cuda.synchronize()
        got = Sd.cpu().numpy().copy()
        work()                                            # the same work, eager, with the library's other kernels around it
        torch.cuda.synchronize()
        assert np.array_equal(got, Sd.cpu().numpy()), trial
        assert_packed_equal(D, orc.pack(W, got, bits, 10000))
