"""gwq_linear_bf16: bfloat16 activations in, bfloat16 results out, against the oracle's fp64 product of the same
bfloat16 values (widened exactly) with the exact dequantised weights (Sec. 3.2, Eq. 10 plus the FP16 outliers).

Tolerances.  A bfloat16 result has 8 significant bits: the store alone moves it by up to 2^-8 of itself, 2^-8 / sqrt(3) =
2.26e-3 in the root mean square when the errors are spread evenly (the fp64 product rounded to bfloat16 on the CPU
shows 2.1e-3 on the first case below), which is more than the 2e-3 the FP16 path is held to.  So the Frobenius bound
here is 2e-3 for the arithmetic plus 2.26e-3 for the store, the largest error stays <= 1e-2 of the largest result, and
the sharp check is elementwise: 2^-8 |y| for the store plus what the arithmetic can add.  For M <= 16 the MFMA operands
are exact (x and 128 + q); the FP32 sum of a group is a sum of terms (128 + q) x, from which (128 + z) sum x is taken
off afterwards, so its roundings (at most 32 of 2^-24 each: four MFMAs and two multiply-adds) are relative to
s * 143 * sum_k |x| of the group and not to the much smaller sum_k |W_Q x|: 2^-19 of that, next to 2^-10 of
sum_k |W_Q x| for everything else.  For M > 16 the weights are rounded to bfloat16 first: 2^-9 of sum_k |W_Q x|, checked
with a factor of two in hand.
"""
import numpy as np
import pytest

import gwq_synth as gs
from oracle import gwq_oracle as orc

pytestmark = pytest.mark.gpu


def _problem(seed, N, K, bits, ppm=10000):
    rng = np.random.default_rng(seed)
    W = gs.weight(N, K, rng, planted_cols=min(2, K // 64))
    S = gs.score_from_weight(W, rng)
    return orc.pack(W, S, bits, ppm), rng


def _bf16(x32):
    """float32 array -> (torch bfloat16 tensor on the GPU, its values as fp64)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x32, np.float32)).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    return t.cuda(), orc.bf16_bits_to_f64(bits)


def _check(D, P, x32, what):
    import torch
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close
    Xg, Xd = _bf16(x32)
    Y = gwq.linear_bf16(D, Xg)
    assert Y.dtype == torch.bfloat16
    Yg = orc.bf16_bits_to_f64(Y.cpu().view(torch.int16).numpy().view(np.uint16))
    Y_ref = orc.linear_f64_x(P, Xd)
    assert np.isfinite(Yg).all(), what
    rel = np.linalg.norm(Yg - Y_ref) / np.linalg.norm(Y_ref)
    mx = np.abs(Yg - Y_ref).max() / np.abs(Y_ref).max()
    assert rel <= 2e-3 + 2.0 ** -8 / np.sqrt(3.0) and mx <= 1e-2, f"{what}: rel_fro={rel:.3e} max_abs/max={mx:.3e}"
    mag = np.abs(Xd) @ np.abs(orc.decode(P)).T
    M = x32.shape[0]
    group_scale = np.repeat(P.scales.view(np.float16).astype(np.float64).reshape(P.N, -1), P.group, axis=1)
    bound = 2.0 ** -8 * np.abs(Y_ref) + (2.0 ** -10 if M <= 16 else 2.0 ** -8) * mag + 1e-30
    if M <= 16:
        bound += 2.0 ** -19 * (np.abs(Xd) @ (143.0 * group_scale).T)
    excess = np.abs(Yg - Y_ref) - bound
    assert excess.max() <= 0, f"{what}: {np.count_nonzero(excess > 0)} results beyond the rounding bound"
    return rel


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K", [(16, 128), (40, 256), (200, 1024), (72, 11008), (1, 128)])
def test_bf16_decode_all_M(bits, N, K):
    from gpu_helpers import upload_packed
    P, rng = _problem(N + K + bits, N, K, bits)
    D = upload_packed(P)
    for M in range(1, 17):
        _check(D, P, gs.activations(M, K, rng).astype(np.float32), f"bf16 decode N={N} K={K} M={M} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
def test_bf16_longest_rows(bits):
    from gpu_helpers import upload_packed
    N, K = 24, 65536
    P, rng = _problem(31 + bits, N, K, bits)
    D = upload_packed(P)
    for M in (1, 9, 16, 40):
        _check(D, P, gs.activations(M, K, rng).astype(np.float32), f"bf16 K={K} M={M} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K,M", [(128, 256, 17), (200, 1024, 64), (300, 384, 130), (260, 1408, 300), (72, 11008, 65),
                                   (128, 4096, 17), (1500, 1024, 300)])
def test_bf16_gemm(bits, N, K, M):
    """M > 16: whole and partial tiles, launches that split K (FP32 partial sums, bfloat16 store in the reduction)."""
    from gpu_helpers import upload_packed
    P, rng = _problem(N + K + M + bits, N, K, bits)
    rel = _check(upload_packed(P), P, gs.activations(M, K, rng).astype(np.float32), f"bf16 gemm N={N} K={K} M={M} bits={bits}")
    assert rel > 1e-4                                  # bfloat16 operands and results: no better than that, or the check is vacuous


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("rows", [32, 64, 128, 256])
def test_bf16_gemm_block_shapes(bits, rows):
    import paper_2411_00850_amd as gwq
    from gpu_helpers import upload_packed
    N, K, M = 260, 640, 300
    P, rng = _problem(rows + bits, N, K, bits)
    gwq.tuning_set("gemm_rows", rows)
    try:
        _check(upload_packed(P), P, gs.activations(M, K, rng).astype(np.float32), f"bf16 rows={rows} bits={bits}")
    finally:
        gwq.tuning_set("gemm_rows", 0)


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("M", [1, 12, 48])
def test_bf16_activations_beyond_the_fp16_range(bits, M):
    """Activations up to 1e8 and down to 1e-12 (FP16 ends at 65504 and 6e-8): finite, accurate results."""
    from gpu_helpers import upload_packed
    N, K = 96, 768
    P, rng = _problem(200 + bits + M, N, K, bits)
    x = gs.activations(M, K, rng).astype(np.float32)
    x[:, 5] *= 1e8
    x[:, 300:320] *= 1e5
    x[:, 600:] *= 1e-12
    _check(upload_packed(P), P, x, f"bf16 wide range M={M} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("pad_byte", [0xFF, 0x7C])
def test_bf16_padding_is_never_interpreted(bits, pad_byte):
    from gpu_helpers import upload_packed
    N, K = 27, 2688
    P, rng = _problem(pad_byte + bits, N, K, bits)
    D = upload_packed(P, pad_byte)
    for M in (1, 5, 16, 33):
        _check(D, P, gs.activations(M, K, rng).astype(np.float32), f"bf16 pad={pad_byte:#x} M={M}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("ppm", [0, 1000000])
def test_bf16_outlier_extremes(bits, ppm):
    """No outliers at all, and every weight an outlier (then the product is X W^T with the FP16 weights themselves;
    for M > 16 they are rounded to bfloat16 operands)."""
    from gpu_helpers import upload_packed
    N, K = 48, 512
    P, rng = _problem(ppm % 7 + bits, N, K, bits, ppm)
    D = upload_packed(P)
    for M in (3, 16, 40):
        _check(D, P, gs.activations(M, K, rng).astype(np.float32), f"bf16 ppm={ppm} M={M}")


def test_bf16_7b_shape_full():
    """One 7B projection at full size (4096 x 4096, 4 bits): M = 1 and 16 through the decode kernel and M = 256
    through the GEMM, every result compared."""
    from gpu_helpers import upload_packed
    W, S = gs.layer_matrix(2, 0, 4096, 4096)
    P = orc.pack(W, S, 4, 10000)
    D = upload_packed(P)
    rng = np.random.default_rng(4)
    for M in (1, 16, 256):
        _check(D, P, gs.activations(M, 4096, rng).astype(np.float32), f"bf16 4096x4096 M={M}")
