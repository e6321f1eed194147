"""Seeded synthetic inputs for the GWQ linear-layer path.

Shared by the oracle-side tests, the GPU parity tests, the smoke check and the benchmark.
This module draws random tensors only: it contains none of the method's arithmetic (no
selection, no quantisation, no packing), so the CPU oracle and the HIP path stay independent.

The tensors stand in for the LLaMA-family weights and calibration gradients the paper used
(Sec. 4.1), which are not available here: real layer shapes, heavy-tailed weights, and the
channel-structured outliers the paper reports (Sec. 3, discussion of the outlier figure).
"""
import numpy as np

# (name, N = out features, K = in features)
SHAPES_7B = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
             ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
SHAPES_70B = [("attn", 8192, 8192), ("up", 28672, 8192), ("down", 8192, 28672)]

_CHUNK_ROWS = 1024


def rng_for(*ids):
    """numpy Generator seeded by a tuple of small integers (config id, matrix id, tensor id)."""
    return np.random.default_rng(list(ids))


def weight(N, K, rng, planted_cols=0, planted_gain=20.0):
    """FP16 weight [N, K]: 0.02 * Student-t(df=4); optionally `planted_cols` input columns
    (chosen without replacement) multiplied by `planted_gain` before the FP16 cast."""
    gain = np.ones(K, np.float32)
    if planted_cols:
        cols = rng.choice(K, size=planted_cols, replace=False)
        gain[cols] = planted_gain
    W = np.empty((N, K), np.float16)
    for r0 in range(0, N, _CHUNK_ROWS):
        r1 = min(N, r0 + _CHUNK_ROWS)
        t = rng.standard_t(4, size=(r1 - r0, K)).astype(np.float32)
        W[r0:r1] = (0.02 * t * gain).astype(np.float16)
    return W


def score_from_weight(W, rng, dtype=np.float32):
    """Gradient-score stand-in [N, K]: |N(0,1)| * |W|."""
    N, K = W.shape
    S = np.empty((N, K), dtype)
    for r0 in range(0, N, _CHUNK_ROWS):
        r1 = min(N, r0 + _CHUNK_ROWS)
        g = np.abs(rng.standard_normal(size=(r1 - r0, K), dtype=np.float32))
        S[r0:r1] = (g * np.abs(W[r0:r1].astype(np.float32))).astype(dtype)
    return S


def score_clustered(N, K, n_top, rng, axis="col", frac_hot=0.6, hot_share=0.01):
    """FP32 score [N, K] whose `n_top` largest entries are a known set: a fraction `frac_hot`
    of them lies in `hot_share` of the columns (axis="col") or rows (axis="row").
    Entries of the set get 2 + U(0,1), all others U(0,1).  Returns (S, rows, cols) with the
    positions of the set, so that a caller knows the top-n_top entries without sorting."""
    S = rng.random(size=(N, K), dtype=np.float32)
    if axis == "col":
        n_hot = int(np.ceil(hot_share * K))
        hot = np.sort(rng.choice(K, size=n_hot, replace=False))
        cold = np.setdiff1d(np.arange(K), hot)
        n_in_hot = min(int(round(frac_hot * n_top)), N * n_hot)
        pick = rng.choice(N * n_hot, size=n_in_hot, replace=False)
        rows_h, cols_h = pick // n_hot, hot[pick % n_hot]
        pick = rng.choice(N * cold.size, size=n_top - n_in_hot, replace=False)
        rows_c, cols_c = pick // cold.size, cold[pick % cold.size]
    else:
        n_hot = int(np.ceil(hot_share * N))
        hot = np.sort(rng.choice(N, size=n_hot, replace=False))
        cold = np.setdiff1d(np.arange(N), hot)
        n_in_hot = min(int(round(frac_hot * n_top)), K * n_hot)
        pick = rng.choice(n_hot * K, size=n_in_hot, replace=False)
        rows_h, cols_h = hot[pick // K], pick % K
        pick = rng.choice(cold.size * K, size=n_top - n_in_hot, replace=False)
        rows_c, cols_c = cold[pick // K], pick % K
    rows = np.concatenate([rows_h, rows_c])
    cols = np.concatenate([cols_h, cols_c])
    S[rows, cols] += np.float32(2.0)
    return S, rows, cols


def activations(M, K, rng, hot_frac=0.0, hot_gain=50.0):
    """FP16 activations [M, K] ~ N(0,1); ceil(hot_frac*K) channels multiplied by hot_gain."""
    X = rng.standard_normal(size=(M, K), dtype=np.float32)
    if hot_frac > 0:
        n_hot = int(np.ceil(hot_frac * K))
        cols = rng.choice(K, size=n_hot, replace=False)
        X[:, cols] *= np.float32(hot_gain)
    return X.astype(np.float16)


def config1():
    """Single 4096x4096 layer, seed 0, M = 1."""
    rng = np.random.default_rng(0)
    W = weight(4096, 4096, rng)
    S = score_from_weight(W, rng)
    X = activations(1, 4096, rng)
    return W, S, X


def layer_matrix(config_id, matrix_id, N, K, planted_cols=8):
    """Weight and score of one matrix of the 7B-shaped layer (planted outlier columns)."""
    W = weight(N, K, rng_for(config_id, matrix_id, 0), planted_cols=planted_cols)
    S = score_from_weight(W, rng_for(config_id, matrix_id, 1))
    return W, S
