"""Quantisation groups of 16, 32 and 64 weights (Sec. 3.2, first paragraph: one scale and zero point per group of
beta consecutive weights, beta = 16 in the paper) through gwq_pack, gwq_quality and gwq_linear.

Packing is compared byte for byte with the oracle, gwq_quality to the fp64 summation-order bound of its own test
file.  gwq_linear multiplies these layers with FP16 operands s * (q - z) (a lane's MFMA sums over several groups,
so the scale goes in before it): each operand carries a relative rounding error of at most 2^-11, which adds
2^-11 * sum_k |W_Q[n][k] X[m][k]| to the error of a result next to the 2^-11 |Y| of the FP16 store and the FP32
sums' own rounding (K * 2^-24 of the same sum of magnitudes at most).  The tests check that bound element by element
on top of the two norms every gwq_linear test checks.
"""
import numpy as np
import pytest

import gwq_synth as gs
from oracle import gwq_oracle as orc

pytestmark = pytest.mark.gpu

GROUPS = [16, 32, 64]


def _weights(seed, N, K, planted=2):
    rng = np.random.default_rng(seed)
    W = gs.weight(N, K, rng, planted_cols=min(planted, K // 64))
    return W, gs.score_from_weight(W, rng), rng


def _assert_elementwise(Y_gpu, P, X, what):
    from gpu_helpers import assert_close
    Y_ref = orc.linear_f64(P, X)
    assert_close(Y_gpu, Y_ref, what)
    mag = np.abs(X.astype(np.float64)) @ np.abs(orc.decode(P)).T
    bound = 2.0 ** -10 * np.abs(Y_ref) + (2.0 ** -11 + P.K * 2.0 ** -24) * mag + 1e-7
    excess = np.abs(Y_gpu.astype(np.float64) - Y_ref) - bound
    assert excess.max() <= 0, f"{what}: {np.count_nonzero(excess > 0)} results beyond the rounding bound, worst by {excess.max():.3e}"


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("group", GROUPS)
@pytest.mark.parametrize("N,K,ppm", [(1, 128, 10000), (37, 384, 10000), (200, 1024, 0), (64, 2304, 300000),
                                     (16, 11008, 10000), (9, 256, 1000000)])
def test_pack_small_groups(bits, group, N, K, ppm):
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_packed_equal, to_gpu
    W, S, _ = _weights(N * 5 + K + group + bits, N, K)
    D = gwq.pack(to_gpu(W), to_gpu(S), bits, ppm, group=group)
    P = orc.pack(W, S, bits, ppm, group)
    assert D.group == group and P.scales.size == N * K // group
    assert_packed_equal(D, P)


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("group", GROUPS)
def test_pack_small_groups_special_values(bits, group):
    """FP16 scores with ties, weights at the ends of the FP16 range and non-finite ones: the group's range, scale
    and zero point follow the same rules whatever the group size."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_packed_equal, to_gpu
    N, K = 40, 768
    W, S, rng = _weights(300 + group + bits, N, K)
    S = (np.round(S * 32) / 32).astype(np.float16)
    W = W.copy()
    W[3, :64] = np.float16(65504.0) * rng.choice([-1, 1], 64).astype(np.float16)
    W[5, 100:140] = np.float16(6e-8)
    W[7, 16:32] = np.float16(0.0)
    W[9, 200] = np.float16(np.inf)
    W[9, 300] = np.float16(-np.inf)
    W[11, 17] = np.float16(np.nan)
    assert_packed_equal(gwq.pack(to_gpu(W), to_gpu(S), bits, 20000, group=group), orc.pack(W, S, bits, 20000, group))


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("group", GROUPS)
def test_pack_7b_shape_small_groups(bits, group):
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_packed_equal, to_gpu
    N, K = 1024, 4096                                    # a quarter of a 7B attention projection
    W, S, _ = _weights(group + bits, N, K, planted=8)
    assert_packed_equal(gwq.pack(to_gpu(W), to_gpu(S), bits, 10000, group=group), orc.pack(W, S, bits, 10000, group))


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("group", GROUPS)
@pytest.mark.parametrize("N,K,ppm", [(37, 384, 10000), (200, 1024, 0), (16, 11008, 300000)])
def test_quality_small_groups(bits, group, N, K, ppm):
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    W, S, _ = _weights(N + K + group, N, K)
    P = orc.pack(W, S, bits, ppm, group)
    got = gwq.quality(upload_packed(P), to_gpu(W), to_gpu(S)).cpu().numpy()
    sq, first, mx = orc.quality(P, W, S)
    err = W.astype(np.float64) - orc.decode(P)
    assert abs(got[0] - sq) <= 1e-11 * sq
    assert abs(got[1] - first) <= 1e-11 * float(np.sum(np.abs(S.astype(np.float64) * err)))
    assert got[2] == mx


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("group", GROUPS)
@pytest.mark.parametrize("N,K", [(16, 128), (40, 256), (200, 1024), (72, 11008), (1, 128)])
def test_decode_small_groups_all_M(bits, group, N, K):
    """Every M of the decode path, ragged N, rows of one block of 128 codes up to several phases of K."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    W, S, rng = _weights(N + K + bits + group, N, K)
    P = orc.pack(W, S, bits, 10000, group)
    D = upload_packed(P)
    for M in range(1, 17):
        X = gs.activations(M, K, rng)
        _assert_elementwise(gwq.linear(D, to_gpu(X)).cpu().numpy(), P, X, f"decode group={group} N={N} K={K} M={M} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("group,K", [(16, 32768), (32, 65536), (64, 65536)])
def test_linear_most_groups_per_channel(bits, group, K):
    """The longest rows a group size allows (2048 groups per channel, or K = 65536), decode and GEMM."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    N = 24
    W, S, rng = _weights(7 + group + bits, N, K)
    P = orc.pack(W, S, bits, 10000, group)
    D = upload_packed(P)
    for M in (1, 7, 16, 40):
        X = gs.activations(M, K, rng)
        _assert_elementwise(gwq.linear(D, to_gpu(X)).cpu().numpy(), P, X, f"group={group} K={K} M={M} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("group", GROUPS)
@pytest.mark.parametrize("N,K,M", [(128, 256, 17), (200, 1024, 64), (300, 384, 130), (260, 1408, 300), (72, 11008, 65)])
def test_gemm_small_groups(bits, group, N, K, M):
    """M > 16: whole and partial tiles, every block shape the launcher picks for these M, K split or not."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    W, S, rng = _weights(N + K + M + group, N, K)
    P = orc.pack(W, S, bits, 10000, group)
    X = gs.activations(M, K, rng)
    D = upload_packed(P)
    _assert_elementwise(gwq.linear(D, to_gpu(X)).cpu().numpy(), P, X, f"gemm group={group} N={N} K={K} M={M} bits={bits}")
    index = gwq.linear_index(D)
    Y2 = gwq.linear(D, to_gpu(X), index=index).cpu().numpy()
    _assert_elementwise(Y2, P, X, "indexed")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("rows", [32, 64, 128, 256])
def test_gemm_small_groups_block_shapes(bits, rows):
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    N, K, M = 260, 640, 300
    W, S, rng = _weights(rows + bits, N, K)
    P = orc.pack(W, S, bits, 10000, 16)
    X = gs.activations(M, K, rng)
    gwq.tuning_set("gemm_rows", rows)
    try:
        Y = gwq.linear(upload_packed(P), to_gpu(X)).cpu().numpy()
    finally:
        gwq.tuning_set("gemm_rows", 0)
    _assert_elementwise(Y, P, X, f"rows={rows} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("group", GROUPS)
@pytest.mark.parametrize("pad_byte", [0xFF, 0x7C])
def test_small_groups_padding_is_never_interpreted(bits, group, pad_byte):
    """The bytes behind scales, zeros and the CSR arrays hold NaN and infinity patterns: no result may depend on
    them (the last phase of a ragged K reaches past the last group)."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    N, K = 27, 2688
    W, S, rng = _weights(pad_byte + group, N, K)
    P = orc.pack(W, S, bits, 10000, group)
    D = upload_packed(P, pad_byte)
    for M in (1, 5, 16, 33):
        X = gs.activations(M, K, rng)
        _assert_elementwise(gwq.linear(D, to_gpu(X)).cpu().numpy(), P, X, f"pad={pad_byte:#x} group={group} M={M}")


@pytest.mark.parametrize("bits", [4, 3])
def test_small_groups_extreme_scales(bits):
    """Groups whose range is close to the whole FP16 range: the scale is capped so that the FP16 operands stay
    finite (the header documents the cap), and the results stay finite and within the norms."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close, to_gpu, upload_packed
    N, K = 48, 512
    W, S, rng = _weights(91 + bits, N, K)
    W = W.copy()
    W[:, 32:48] = (rng.choice([-1.0, 1.0], (N, 16)) * 30000.0).astype(np.float16)
    P = orc.pack(W, S, bits, 0, 16)
    D = upload_packed(P)
    for M in (2, 12, 40):
        X = (gs.activations(M, K, rng).astype(np.float32) * 1e-2).astype(np.float16)
        assert_close(gwq.linear(D, to_gpu(X)).cpu().numpy(), orc.linear_f64(P, X), f"extreme M={M} bits={bits}")


@pytest.mark.parametrize("M", [1, 8])
def test_grouped_launch_and_gate_up_with_small_groups(M):
    """gwq_linear_batch over layers of one group size, and the gated pair (two products and the elementwise
    kernel: the fused decode launch is for groups of 128)."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    N, K = 176, 512
    rng = np.random.default_rng(5)
    layers = []
    for i in range(2):
        W, S, _ = _weights(50 + i, N, K)
        layers.append(orc.pack(W, S, 4, 10000, 32))
    X = gs.activations(M, K, rng)
    D = [upload_packed(P) for P in layers]
    Xg = to_gpu(X)
    outs = gwq.linear_batch(D, [Xg, Xg])
    for P, Y in zip(layers, outs):
        _assert_elementwise(Y.cpu().numpy(), P, X, f"batch M={M}")
    from gpu_helpers import assert_close
    H = gwq.linear_gate_up(D[0], D[1], Xg).cpu().numpy()
    assert_close(H, orc.gate_up(orc.linear_f64(layers[0], X), orc.linear_f64(layers[1], X)), f"gate_up M={M}")


@pytest.mark.parametrize("group", GROUPS)
def test_small_groups_7b_shape_full(group):
    """One 7B projection at full size (4096 x 4096, 4 bits) packed on the GPU (byte-exact) and multiplied at M = 1 and 8
    (lean kernel), 16 (wide kernel) and 256 (GEMM, the index carried by the layer): every result compared."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_packed_equal, to_gpu
    W, S = gs.layer_matrix(2, 0, 4096, 4096)
    P = orc.pack(W, S, 4, 10000, group)
    D = gwq.pack(to_gpu(W), to_gpu(S), 4, 10000, group=group)
    assert_packed_equal(D, P)
    rng = np.random.default_rng(group)
    for M in (1, 8, 16, 256):
        X = gs.activations(M, 4096, rng)
        _assert_elementwise(gwq.linear(D, to_gpu(X)).cpu().numpy(), P, X, f"4096x4096 group={group} M={M}")
