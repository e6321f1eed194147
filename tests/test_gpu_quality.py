"""gwq_quality on the GPU against the oracle (Sec. 3.1: Eq. 4 squared error, Eq. 3 and 5 first-order term).

Both sides form every difference W - W_Q exactly in fp64; they differ only in the order of the fp64
sums.  For n terms the order changes a sum by at most about n * 2^-53 times the sum of the terms'
magnitudes (in practice sqrt(n) of that), so the tolerances are 1e-11 relative to sum D^2 and to
sum |score * D| (n < 2^32); the maximum is order-independent and must match exactly.
"""
import numpy as np
import pytest

import gwq_synth as gs
from oracle import gwq_oracle as orc

pytestmark = pytest.mark.gpu

REL = 1e-11


def _check(P, W, S, tag, D=None):
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    D = upload_packed(P) if D is None else D
    got = gwq.quality(D, to_gpu(W), to_gpu(S)).cpu().numpy()
    sq, first, mx = orc.quality(P, W, S)
    err = W.astype(np.float64) - orc.decode(P)
    scale_first = float(np.sum(np.abs(S.astype(np.float64) * err)))
    assert abs(got[0] - sq) <= REL * sq, f"{tag}: squared error {got[0]!r} vs {sq!r}"
    assert abs(got[1] - first) <= REL * scale_first, f"{tag}: first-order term {got[1]!r} vs {first!r}"
    assert got[2] == mx, f"{tag}: max {got[2]!r} vs {mx!r}"
    return got


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K", [(1, 128), (37, 384), (200, 1024), (16, 11008), (5, 65536)])
@pytest.mark.parametrize("ppm", [0, 10000, 300000, 1000000])
def test_quality_small_shapes(bits, N, K, ppm):
    rng = np.random.default_rng(N + K + bits + ppm % 13)
    W = gs.weight(N, K, rng, planted_cols=2)
    S = gs.score_from_weight(W, rng)
    got = _check(orc.pack(W, S, bits, ppm), W, S, f"N={N} K={K} bits={bits} ppm={ppm}")
    if ppm == 1000000:
        assert tuple(got) == (0.0, 0.0, 0.0)


@pytest.mark.parametrize("bits", [4, 3])
def test_quality_fp16_scores_signed_scores_and_foreign_outlier_values(bits):
    """Scores of both signs in FP16 (the first-order term cancels), and a packed layer whose stored
    outlier values are not the weights' copies (another layer's): their differences count too."""
    rng = np.random.default_rng(77 + bits)
    N, K = 48, 1280
    W = gs.weight(N, K, rng, planted_cols=2)
    S = (gs.score_from_weight(W, rng) * rng.choice([-1.0, 1.0], size=(N, K))).astype(np.float16)
    P = orc.pack(W, S, bits, 20000)
    _check(P, W, S, "signed fp16 scores")
    P.out_val = (P.out_val.view(np.float16) * np.float16(0.5)).view(np.uint16)
    got = _check(P, W, S, "halved outlier values")
    assert got[2] > 0


@pytest.mark.parametrize("bits", [4, 3])
def test_quality_is_deterministic_and_takes_gpu_packed_layers(bits):
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu
    rng = np.random.default_rng(5 + bits)
    W = gs.weight(300, 2048, rng, planted_cols=2)
    S = gs.score_from_weight(W, rng)
    Wd, Sd = to_gpu(W), to_gpu(S)
    D = gwq.pack(Wd, Sd, bits, 10000)
    a = gwq.quality(D, Wd, Sd).cpu().numpy()
    b = gwq.quality(D, Wd, Sd).cpu().numpy()
    assert np.array_equal(a, b)
    _check(orc.pack(W, S, bits, 10000), W, S, "gpu-packed", D=D)


@pytest.mark.parametrize("bits", [4, 3])
def test_quality_config1_full(bits):
    W, S, _ = gs.config1()
    _check(orc.pack(W, S, bits, 10000), W, S, f"config 1, {bits} bits")


def test_quality_7b_gate_shape_full():
    name, N, K = gs.SHAPES_7B[4]
    W, S = gs.layer_matrix(2, 4, N, K)
    _check(orc.pack(W, S, 4, 10000), W, S, f"{name} {N}x{K}")
