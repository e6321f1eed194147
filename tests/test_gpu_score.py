"""gwq_score on the GPU against the oracle (Sec. 3.1, Eq. 2: the gradient of the loss with respect to the
weights; for Y = X W^T it is dY^T X by the chain rule).

Every product of two FP16 numbers is exact in FP32; the kernel adds them in FP32 (MFMA) where the oracle
adds in fp64, so an entry differs from the oracle's by at most about M * 2^-24 times the largest partial
sum's magnitude - bounded here by 2^-24 * sum_m |dY[m][n] X[m][k]| times a small factor for the order of
the additions.  The tests check that bound entry by entry (factor 4), which is far tighter than the
library's FP16-output tolerance, and the scaled accumulation on top of it.
"""
import numpy as np
import pytest

import gwq_synth as gs
from oracle import gwq_oracle as orc

pytestmark = pytest.mark.gpu

EPS = 2.0 ** -24


def _inputs(M, N, K, seed, hot=0.0):
    rng = np.random.default_rng(seed)
    X = gs.activations(M, K, rng, hot_frac=hot)
    dY = (0.05 * rng.standard_normal((M, N))).astype(np.float16)
    return dY, X


def _bound(dY, X, alpha=1.0):
    mag = np.abs(dY.astype(np.float64)).T @ np.abs(X.astype(np.float64))
    return 4.0 * EPS * abs(alpha) * mag + 1e-30


def _check(dY, X, tag, alpha=1.0, beta=0.0, prev=None):
    import torch
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu
    out = to_gpu(prev) if prev is not None else torch.full((dY.shape[1], X.shape[1]), float("nan"), device="cuda")
    got = gwq.score(to_gpu(dY), to_gpu(X), out=out, alpha=alpha, beta=beta).cpu().numpy()
    want = orc.score(dY, X, alpha=alpha, beta=beta, prev=prev)
    bound = _bound(dY, X, alpha) + (4.0 * EPS * np.abs(beta * prev.astype(np.float64)) if beta != 0.0 else 0.0)
    bad = np.abs(got.astype(np.float64) - want) > bound
    assert np.isfinite(got).all(), tag
    assert not bad.any(), f"{tag}: {bad.sum()} of {bad.size} entries off, first at {np.argwhere(bad)[:3].tolist()}"
    return got


@pytest.mark.parametrize("M,N,K", [(1, 1, 128), (1, 16, 128), (3, 8, 256), (64, 128, 128), (65, 128, 128),
                                   (70, 200, 256), (127, 136, 384), (128, 264, 128), (129, 40, 1408),
                                   (300, 130, 384), (200, 7, 256), (33, 129, 128), (500, 131, 512), (512, 384, 1024)])
def test_score_small_shapes(M, N, K):
    dY, X = _inputs(M, N, K, seed=M * 7 + N * 3 + K)
    _check(dY, X, f"M={M} N={N} K={K}")


def test_score_picks_rows_and_columns_exactly():
    """dY with a single one at (m0, n0) copies row m0 of X into row n0 of the score, bit for bit, and leaves
    every other row zero: a transposed or shifted operand cannot pass."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu
    M, N, K = 150, 140, 256
    _, X = _inputs(M, N, K, seed=5)
    for m0, n0 in ((0, 0), (63, 127), (64, 128), (149, 139), (77, 5)):
        dY = np.zeros((M, N), np.float16)
        dY[m0, n0] = 1.0
        got = gwq.score(to_gpu(dY), to_gpu(X)).cpu().numpy()
        assert np.array_equal(got[n0], X[m0].astype(np.float32)), (m0, n0)
        got[n0] = 0
        assert not got.any(), (m0, n0)


def test_score_mean_over_samples_and_scaling():
    """Sec. 4.3 (ablation on the number of calibration samples): the mean gradient over calibration samples as calls with alpha = 1 / samples, beta = 0 then 1."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu
    M, N, K = 96, 72, 256
    parts = [_inputs(M, N, K, seed=20 + i, hot=0.01) for i in range(3)]
    out = None
    prev = None
    for i, (dY, X) in enumerate(parts):
        got = _check(dY, X, f"sample {i}", alpha=1.0 / 3, beta=0.0 if i == 0 else 1.0, prev=prev)
        prev = got
    all_dY = np.concatenate([p[0] for p in parts])
    all_X = np.concatenate([p[1] for p in parts])
    mean = orc.score(all_dY, all_X, alpha=1.0 / 3)
    assert np.abs(prev - mean).max() <= 3 * (_bound(all_dY, all_X, 1.0 / 3) + 4 * EPS * np.abs(mean)).max()
    # negative alpha, beta that is neither 0 nor 1
    dY, X = parts[0]
    _check(dY, X, "alpha=-2 beta=0.5", alpha=-2.0, beta=0.5, prev=prev)
    # beta = 0 must not read the old contents (NaN-filled by _check)
    _check(dY, X, "beta=0 over NaN")
    # deterministic
    a = gwq.score(to_gpu(dY), to_gpu(X)).cpu().numpy()
    b = gwq.score(to_gpu(dY), to_gpu(X)).cpu().numpy()
    assert np.array_equal(a, b)


def test_score_feeds_pack():
    """The score made on the device ranks the same outliers as the oracle's score of the same layer wherever the
    two orders can be told apart: pack with the device's score, bit-exact against the oracle packing with
    that same score (the selection is defined on the score it is given)."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, assert_packed_equal
    M, N, K = 256, 96, 512
    rng = np.random.default_rng(31)
    W = gs.weight(N, K, rng, planted_cols=2)
    X = gs.activations(M, K, rng, hot_frac=0.01)
    T = (X.astype(np.float32) @ W.astype(np.float32).T + 0.1 * rng.standard_normal((M, N))).astype(np.float16)
    Y = (X.astype(np.float32) @ W.astype(np.float32).T).astype(np.float16)
    dY = (Y.astype(np.float32) - T.astype(np.float32)).astype(np.float16)        # squared-error loss: dL/dY = Y - T
    S = gwq.score(to_gpu(dY), to_gpu(X))
    D = gwq.pack(to_gpu(W), S, 4, 10000)
    assert_packed_equal(D, orc.pack(W, S.cpu().numpy(), 4, 10000))
    # against the oracle's own score: the kept sets agree except near the threshold
    S_ref = orc.score(dY, X)
    keep_gpu = set(np.argsort(-np.abs(S.cpu().numpy()).ravel(), kind="stable")[:D.n_outliers].tolist())
    keep_ref = set(np.argsort(-np.abs(S_ref).ravel(), kind="stable")[:D.n_outliers].tolist())
    assert len(keep_gpu ^ keep_ref) <= 2


@pytest.mark.parametrize("N,K", [(4096, 4096), (4096, 11008)])
def test_score_7b_shapes_sampled(N, K):
    """Full 7B shapes at M = 2048, as bench.py times them; the oracle computes sampled output rows."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu
    M = 2048
    dY, X = _inputs(M, N, K, seed=N + K, hot=0.001)
    got = gwq.score(to_gpu(dY), to_gpu(X)).cpu().numpy()
    assert np.isfinite(got).all()
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 63, 64, 127, 128, N - 129, N - 128, N - 1],
                                     np.random.default_rng(1).integers(0, N, 13)]))
    sub = np.ascontiguousarray(dY[:, rows])
    want = orc.score(sub, X)
    bad = np.abs(got[rows].astype(np.float64) - want) > _bound(sub, X)
    assert not bad.any(), f"{bad.sum()} entries off, first at {np.argwhere(bad)[:3].tolist()}"
