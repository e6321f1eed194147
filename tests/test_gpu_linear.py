"""gwq_linear on the GPU against the oracle's fp64 product (Sec. 3.2, Eq. 10 plus the FP16 outliers).

Tolerances (written in gpu_helpers): relative Frobenius error <= 2e-3 and
max|Y_gpu - Y_ref| <= 1e-2 * max|Y_ref|.  The packed inputs of these tests come from the oracle,
so the linear kernels are checked independently of the GPU packer.
"""
import functools

import numpy as np
import pytest

import gwq_synth as gs
from oracle import gwq_oracle as orc

pytestmark = pytest.mark.gpu


def _problem(seed, N, K, bits, ppm=10000, planted=2):
    rng = np.random.default_rng(seed)
    W = gs.weight(N, K, rng, planted_cols=planted)
    S = gs.score_from_weight(W, rng)
    return orc.pack(W, S, bits, ppm), rng


def _run(P, X):
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    D = upload_packed(P)
    return gwq.linear(D, to_gpu(X)).cpu().numpy()


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K", [(16, 128), (40, 256), (200, 1024), (72, 11008), (1, 128)])
def test_decode_small_all_M(bits, N, K):
    """Every M of the decode kernel (1..16), ragged N (not a multiple of 16), several K splits."""
    from gpu_helpers import assert_close
    P, rng = _problem(N + K + bits, N, K, bits)
    for M in range(1, 17):
        X = gs.activations(M, K, rng)
        assert_close(_run(P, X), orc.linear_f64(P, X), f"decode N={N} K={K} M={M} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
def test_decode_longest_rows(bits):
    """K = 65536, the largest the format allows (16-bit column indices): 512 groups per channel, more
    than one block's waves can hold at once, so every M goes through several chunks of K."""
    from gpu_helpers import assert_close
    N, K = 24, 65536
    P, rng = _problem(900 + bits, N, K, bits)
    for M in (1, 3, 9, 16):
        X = gs.activations(M, K, rng)
        assert_close(_run(P, X), orc.linear_f64(P, X), f"decode N={N} K={K} M={M} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("waves", [1, 2, 3, 6, 12, 16])
@pytest.mark.parametrize("M", [1, 3, 5])
def test_decode_launch_shapes(bits, waves, M):
    """Every split of K over the waves of a block that the tuning knob can ask for (4, 8 or 16 groups
    per wave in the kernel for M <= 4; the kernel for larger M picks its own) gives the same answer
    within tolerance."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close
    P, rng = _problem(77, 150, 1536, bits)
    X = gs.activations(M, 1536, rng)
    ref = orc.linear_f64(P, X)
    gwq.tuning_set("decode_waves", waves)
    try:
        assert_close(_run(P, X), ref, f"waves={waves} M={M}")
    finally:
        gwq.tuning_set("decode_waves", 0)


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K,ppm", [(16, 128, 10000), (150, 1536, 10000), (333, 4096, 10000), (100, 640, 300000),
                                     (40, 512, 1000000), (97, 2048, 0)])
@pytest.mark.parametrize("tiles", [0, 1, 2, 3, 4, 7])
def test_decode_streaming_kernel(bits, N, K, ppm, tiles):
    """The streaming decode kernel (X operands in registers, transposed X in LDS, tiles requested three ahead)
    for every M it takes, forced on for M <= 4 as well, with every number of tiles per block from one
    (nothing to pipeline) through the three register sets and beyond, ragged N, short rows (one wave),
    and rows with more outliers than the staged window holds (ppm = 30 % and 100 %)."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close
    P, rng = _problem(N + K + bits + ppm % 7, N, K, bits, ppm=ppm)
    gwq.tuning_set("decode_stream", 2)
    gwq.tuning_set("decode_tiles", tiles)
    try:
        for M in (1, 2, 3, 4, 5, 7, 8, 9, 12, 16):
            X = gs.activations(M, K, rng)
            assert_close(_run(P, X), orc.linear_f64(P, X), f"stream N={N} K={K} M={M} bits={bits} ppm={ppm} tiles={tiles}")
    finally:
        gwq.tuning_set("decode_stream", 0)
        gwq.tuning_set("decode_tiles", 0)


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K,ppm", [(1, 128, 10000), (17, 256, 10000), (33, 1536, 10000), (47, 640, 300000), (150, 2048, 10000),
                                     (333, 4096, 10000), (96, 512, 1000000), (100, 3968, 0)])
def test_decode_two_tiles_per_block(bits, N, K, ppm):
    """The kernel for M <= 8 in its paired form (two neighbouring tiles per block, one copy of X between two sets of
    waves, each staging every second row; half the staged CSR window), forced on for every M it takes: odd tile counts
    (the second set of the last block has no tile), ragged N, one to eight waves per set, rows with more outliers
    than the window holds."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close, to_gpu, upload_packed
    P, rng = _problem(N * 3 + K + bits + ppm % 11, N, K, bits, ppm=ppm)
    D = upload_packed(P)
    gwq.tuning_set("decode_pairs", 2)
    try:
        for M in (5, 6, 7, 8):
            assert ",true> grid %dx1" % ((N + 31) // 32) in gwq.linear_plan(D, M)
            X = gs.activations(M, K, rng)
            assert_close(gwq.linear(D, to_gpu(X)).cpu().numpy(), orc.linear_f64(P, X), f"pairs N={N} K={K} M={M} bits={bits} ppm={ppm}")
    finally:
        gwq.tuning_set("decode_pairs", 0)


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("ppm", [0, 1000000, 200000])
def test_decode_outlier_extremes(bits, ppm):
    """No outliers, only outliers (a dense FP16 layer in CSR form), and a heavy 20 %."""
    from gpu_helpers import assert_close
    P, rng = _problem(5, 48, 512, bits, ppm=ppm)
    for M in (1, 7, 16):
        X = gs.activations(M, 512, rng)
        assert_close(_run(P, X), orc.linear_f64(P, X), f"ppm={ppm} M={M}")


def test_decode_row_clustered_outliers():
    """Outliers piled into 1 % of the output channels (the row-clustered pattern)."""
    from gpu_helpers import assert_close
    rng = np.random.default_rng(12)
    N, K = 400, 1024
    W = gs.weight(N, K, rng)
    S, _, _ = gs.score_clustered(N, K, orc.outlier_count(N, K, 10000), rng, axis="row")
    P = orc.pack(W, S, 4, 10000)
    assert np.diff(P.row_ptr).max() > 200
    X = gs.activations(3, K, rng)
    assert_close(_run(P, X), orc.linear_f64(P, X))


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("M", [1, 3, 8, 16])
def test_decode_grouped_launch(bits, M):
    """gwq_linear_batch over layers of different N and K (short and long rows, shared activations)
    matches the oracle layer by layer, and agrees with gwq_linear on each layer alone up to the
    rounding of a different split of K over the waves."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close, to_gpu, upload_packed
    shapes = [(200, 1024), (72, 2304), (48, 1024), (16, 128), (130, 11008)]
    rng = np.random.default_rng(bits * 100 + M)
    Xh = {K: gs.activations(M, K, rng) for K in {k for _, k in shapes}}
    Xd = {K: to_gpu(x) for K, x in Xh.items()}
    Ps = [_problem(i + bits, N, K, bits)[0] for i, (N, K) in enumerate(shapes)]
    Ds = [upload_packed(P) for P in Ps]
    outs = gwq.linear_batch(Ds, [Xd[P.K] for P in Ps])
    for P, D, Y in zip(Ps, Ds, outs):
        alone = gwq.linear(D, Xd[P.K]).cpu().numpy().astype(np.float64)
        assert_close(Y.cpu().numpy(), orc.linear_f64(P, Xh[P.K]), f"grouped N={P.N} K={P.K} M={M}")
        assert_close(Y.cpu().numpy(), alone, f"grouped vs alone N={P.N} K={P.K} M={M}")


def test_linear_is_deterministic():
    P, rng = _problem(1, 256, 2048, 4)
    for M in (4, 100):
        X = gs.activations(M, 2048, rng)
        assert np.array_equal(_run(P, X), _run(P, X))


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K", [(128, 256), (200, 1024), (300, 384)])
@pytest.mark.parametrize("M", [17, 64, 65, 130, 300])
def test_gemm_small(bits, N, K, M):
    """The MFMA path: every tile height (64 / 128 / 256 rows), ragged M and N."""
    from gpu_helpers import assert_close
    P, rng = _problem(N + K + M + bits, N, K, bits)
    X = gs.activations(M, K, rng, hot_frac=0.01)
    assert_close(_run(P, X), orc.linear_f64(P, X), f"gemm N={N} K={K} M={M} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K,M", [(256, 256, 512), (260, 384, 300), (384, 128, 256), (130, 256, 256), (128, 512, 128)])
def test_gemm_whole_and_partial_tiles(bits, N, K, M):
    """Launches whose tiles all lie wholly inside Y, and launches with a ragged last m- or n-tile or
    rows of Y that are not a multiple of four long; every element is checked."""
    from gpu_helpers import assert_close
    P, rng = _problem(3 * N + K + M + bits, N, K, bits)
    X = gs.activations(M, K, rng, hot_frac=0.01)
    assert_close(_run(P, X), orc.linear_f64(P, X), f"gemm tiles N={N} K={K} M={M} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("rows", [32, 64, 128, 256])
def test_gemm_block_shapes(bits, rows):
    """Each of the GEMM's four block shapes (rows of Y per block; the library picks by M) forced on
    the same problems, so that every shape also sees several tiles along m, a ragged last tile and
    a K split."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close
    try:
        gwq.tuning_set("gemm_rows", rows)
        for N, K, M in ((200, 1408, 100), (130, 512, 300), (72, 2048, 17)):
            P, rng = _problem(rows + N + M + bits, N, K, bits)
            X = gs.activations(M, K, rng, hot_frac=0.01)
            assert_close(_run(P, X), orc.linear_f64(P, X), f"gemm rows={rows} N={N} K={K} M={M} bits={bits}")
    finally:
        gwq.tuning_set("gemm_rows", 0)


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,M", [(16, 17), (130, 40), (257, 129)])
def test_gemm_shortest_rows(bits, N, M):
    """The GEMM at K = 128: one group, two steps, the shortest loop every role of the kernel can run."""
    from gpu_helpers import assert_close
    P, rng = _problem(700 + N + bits, N, 128, bits)
    X = gs.activations(M, 128, rng)
    assert_close(_run(P, X), orc.linear_f64(P, X), f"gemm N={N} K=128 M={M} bits={bits}")


@pytest.mark.parametrize("bits", [4, 3])
def test_gemm_longest_rows(bits):
    """The GEMM at K = 65536 (512 groups: the most its per-group outlier counts are laid out for)."""
    from gpu_helpers import assert_close
    N, K, M = 40, 65536, 33
    P, rng = _problem(950 + bits, N, K, bits)
    X = gs.activations(M, K, rng)
    assert_close(_run(P, X), orc.linear_f64(P, X), f"gemm N={N} K={K} M={M} bits={bits}")


@pytest.mark.parametrize("ppm", [0, 1000000])
def test_gemm_outlier_extremes(ppm):
    from gpu_helpers import assert_close
    P, rng = _problem(9, 160, 512, 4, ppm=ppm)
    X = gs.activations(70, 512, rng)
    assert_close(_run(P, X), orc.linear_f64(P, X), f"gemm ppm={ppm}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K,ppm", [(200, 1024, 10000), (72, 11008, 10000), (160, 512, 1000000), (50, 384, 0)])
def test_linear_index_contents(bits, N, K, ppm):
    """gwq_linear_index: one 8-byte record per channel and group (plus one that closes the row) holding
    where the group's CSR entries start, its scale and its zero point -- recomputed here from the
    packed arrays with a sorted search."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import upload_packed
    P, _ = _problem(77 + bits, N, K, bits, ppm=ppm)
    gpr = K // 128
    rec = gwq.linear_index(upload_packed(P)).cpu().numpy().view(np.uint32)[:N * (gpr + 1) * 2].reshape(N, gpr + 1, 2)
    for n in range(N):
        lo, hi = int(P.row_ptr[n]), int(P.row_ptr[n + 1])
        want = lo + np.searchsorted(P.col_idx[lo:hi].astype(np.int64), 128 * np.arange(gpr + 1))
        assert np.array_equal(rec[n, :, 0], want), f"first-entry indices of channel {n}"
        sz = P.scales.reshape(N, gpr)[n].view(np.uint16).astype(np.uint32) | P.zeros.reshape(N, gpr)[n].astype(np.uint32) << 16
        assert np.array_equal(rec[n, :gpr, 1], sz), f"scale / zero point of channel {n}"


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K,M", [(200, 1024, 130), (300, 384, 17), (72, 11008, 300), (128, 256, 5)])
def test_linear_indexed_equals_linear(bits, N, K, M):
    """gwq_linear_indexed with a prebuilt index gives gwq_linear's result bit for bit (M <= 16 ignores it),
    also when one index serves several calls."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, upload_packed
    P, rng = _problem(31 + N + bits, N, K, bits)
    D = upload_packed(P)
    index = gwq.linear_index(D)
    for _ in range(2):
        X = to_gpu(gs.activations(M, K, rng))
        assert np.array_equal(gwq.linear(D, X, index=index).cpu().numpy(), gwq.linear(D, X).cpu().numpy())


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K,M", [(200, 1408, 40), (128, 4096, 17), (300, 2048, 200), (1500, 1024, 300), (72, 11008, 64)])
def test_gemm_split_k(bits, N, K, M):
    """Few tiles: the launch also splits K (here 2 to 8 ways, also unevenly: 11 groups in 3 + 3 + 3 + 2) and
    a second kernel adds the FP32 partial sums in a fixed order.  Checked against the oracle, against
    itself (deterministic) and against the same call without scratch, which does not split."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close, to_gpu, upload_packed
    P, rng = _problem(500 + N + bits, N, K, bits)
    X = gs.activations(M, K, rng, hot_frac=0.01)
    D, Xd = upload_packed(P), to_gpu(X)
    index = gwq.linear_index(D)
    split = gwq.linear(D, Xd, index=index).cpu().numpy()
    whole = gwq.linear(D, Xd, index=index, scratch=None).cpu().numpy()
    ref = orc.linear_f64(P, X)
    assert_close(split, ref, f"split-K N={N} K={K} M={M} bits={bits}")
    assert_close(whole, ref, f"no split N={N} K={K} M={M} bits={bits}")
    assert np.array_equal(split, gwq.linear(D, Xd, index=index).cpu().numpy())
    assert np.array_equal(split, gwq.linear(D, Xd).cpu().numpy())          # gwq_linear splits the same way


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("pad_byte", [0xFF, 0xC5, 0x7C])
@pytest.mark.parametrize("N,K", [(396, 640), (27, 384), (45, 2688), (16, 640)])
def test_padding_and_neighbours_are_never_interpreted(bits, pad_byte, N, K):
    """The decode kernels run whole waves of 4, 8 or 16 groups, so with K / 128 not a multiple of that
    the last wave of a channel also multiplies groups that do not exist (against zeros of X).  What
    such a group finds as its scale and zero point must not matter: for the last channel it is the
    padding of the caller's buffers (here bytes 0xFF and 0x7C: NaN scales with zero points 255 and 124;
    and 0xC5: a zero point that carries the 3-bit magic-number decode into a NaN), for channel 15 of a
    tile the bytes of another array.  N * K / 128 is not a multiple of 8 in the first three shapes, so the last 16-byte vector
    of scales and zeros ends in padding."""
    from gpu_helpers import assert_close, to_gpu, upload_packed
    import paper_2411_00850_amd as gwq
    P, rng = _problem(N + K + bits + pad_byte, N, K, bits, ppm=200000)
    D = upload_packed(P, pad_byte=pad_byte)
    for M in (1, 2, 4, 5, 16, 40):
        X = gs.activations(M, K, rng)
        Y = gwq.linear(D, to_gpu(X)).cpu().numpy()
        assert np.isfinite(Y).all(), f"N={N} K={K} bits={bits} M={M} pad={pad_byte:#x}"
        assert_close(Y, orc.linear_f64(P, X), f"padding N={N} K={K} M={M} bits={bits} pad={pad_byte:#x}")


@pytest.mark.parametrize("bits", [4, 3])
def test_linear_extreme_weight_ranges(bits):
    """Groups that span the whole FP16 range (scale 4368: s * 15 would round to infinity as an FP16 product),
    subnormal groups, one-sided and empty ones, through the decode kernels (FP32 scale) and the GEMM (FP16
    operands s * (q - z), scale capped so that they stay finite: the cap moves such a weight by < 0.1 %).
    Activations are small so that the FP16 outputs stay finite; every channel is checked on its own."""
    from gpu_helpers import assert_close, to_gpu, upload_packed
    import paper_2411_00850_amd as gwq
    rng = np.random.default_rng(8)
    N, K = 32, 512
    W = gs.weight(N, K, rng)
    W[0] = (rng.integers(-40, 40, K) * 2.0 ** -24).astype(np.float16)      # subnormals
    W[1] = (rng.standard_normal(K) * 9000).astype(np.float16)               # near the FP16 maximum
    W[2] = np.abs(W[2])
    W[3] = -np.abs(W[3])
    W[4] = 0
    W[6, :128] = np.float16(65504.0)
    W[6, 128:256] = np.float16(-65504.0)
    W[7, :128] = (rng.random(128) * 65504).astype(np.float16)               # 0 .. max: scale 4368 (4-bit)
    W[7, 5] = np.float16(65504.0)
    W[7, 9] = 0
    S = gs.score_from_weight(W, rng)
    S[6:8] = 0                                                              # keep those rows quantised
    P = orc.pack(W, S, bits, 10000)
    assert orc.half_to_double(int(P.scales[7, 0])) * ((1 << bits) - 1) >= 65504
    D = upload_packed(P)
    wnorm = np.linalg.norm(orc.decode(P), axis=1)
    live = np.flatnonzero(wnorm > 1e-3)                                    # not the subnormal and the empty channel
    for M in (1, 5, 16, 17, 40, 300):
        X = (gs.activations(M, K, rng).astype(np.float32) * 1e-3).astype(np.float16)
        Y = gwq.linear(D, to_gpu(X)).cpu().numpy().astype(np.float64)
        ref = orc.linear_f64(P, X)
        assert np.isfinite(Y).all(), f"M={M}"
        # channels equalised by the norm of their weights, so the huge ones do not hide the others
        assert_close(Y[:, live] / wnorm[live], ref[:, live] / wnorm[live], f"extreme ranges bits={bits} M={M}")
        assert not Y[:, 4].any()
        assert np.abs(Y[:, 0] - ref[:, 0]).max() <= 2.0 ** -24             # subnormal weights: FP16 output underflows


def _sweep_cases():
    """40 seeded cases: ragged N, K in whole groups, both bit widths, outlier fractions from none to
    half, outliers spread by weight-scaled scores or clustered in a few columns or a few rows (many
    entries per group: the kernels' long-run paths), and M from 1 to 300 (decode, GEMM, split-K)."""
    rng = np.random.default_rng(20241127)
    cases = []
    for i in range(40):
        N = int(rng.integers(1, 400))
        K = 128 * int(rng.integers(1, 17))
        bits = (4, 3)[i % 2]
        ppm = int(rng.choice([0, 1000, 10000, 10000, 50000, 200000, 500000]))
        kind = ("spread", "cols", "rows")[int(rng.integers(0, 3))]
        M = int(rng.choice([1, 2, 3, 4, 5, 8, 13, 16, 17, 31, 64, 100, 129, 300]))
        cases.append((i, N, K, bits, ppm, kind, M))
    return cases


@pytest.mark.parametrize("case,N,K,bits,ppm,kind,M", _sweep_cases())
def test_linear_random_sweep(case, N, K, bits, ppm, kind, M):
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close, to_gpu, upload_packed
    rng = np.random.default_rng(1000 + case)
    W = gs.weight(N, K, rng, planted_cols=2)
    k_out = orc.outlier_count(N, K, ppm)
    if kind == "spread" or k_out == 0:
        S = gs.score_from_weight(W, rng)
    else:
        S, _, _ = gs.score_clustered(N, K, k_out, rng, axis="col" if kind == "cols" else "row", frac_hot=0.6,
                                     hot_share=0.02)
    P = orc.pack(W, S, bits, ppm)
    X = gs.activations(M, K, rng, hot_frac=0.01)
    D, Xd = upload_packed(P), to_gpu(X)
    ref = orc.linear_f64(P, X)
    tag = f"sweep {case}: N={N} K={K} bits={bits} ppm={ppm} {kind} M={M}"
    assert_close(gwq.linear(D, Xd).cpu().numpy(), ref, tag)
    if M > 16:
        assert_close(gwq.linear(D, Xd, index=gwq.linear_index(D), scratch=None).cpu().numpy(), ref, tag + " (no split)")


# ----------------------------------------------------------------------------- full-size configurations

def test_config1_decode_full():
    from gpu_helpers import assert_close
    W, S, X = gs.config1()
    P = orc.pack(W, S, 4, 10000)
    assert_close(_run(P, X), orc.linear_f64(P, X), "config 1")


@functools.lru_cache(maxsize=2)
def _layer7b(mid, N, K):
    W, S = gs.layer_matrix(2, mid, N, K)
    return W, orc.select(S, 10000)


SHAPES_7B = [(0, 4096, 4096), (4, 11008, 4096), (6, 4096, 11008)]


@pytest.mark.parametrize("mid,N,K", SHAPES_7B)
def test_config2_and_3_decode_7b_shapes(mid, N, K):
    """7B-shaped matrices with planted outlier columns: 4-bit at M in {1, 4, 16}, 3-bit at M in {1, 8}."""
    from gpu_helpers import assert_close
    W, mask = _layer7b(mid, N, K)
    for bits, Ms in ((4, (1, 4, 16)), (3, (1, 8))):
        P = orc.encode(W, mask, bits, 10000)
        for M in Ms:
            X = gs.activations(M, K, gs.rng_for(2, mid, 10 + M))
            assert_close(_run(P, X), orc.linear_f64(P, X), f"7B N={N} K={K} bits={bits} M={M}")


@pytest.mark.parametrize("mid,N,K", SHAPES_7B)
def test_config4_prefill_7b_shapes_full(mid, N, K):
    """Prefill M = 2048 with hot activation channels: every one of the 2048 x N outputs against the
    oracle's fp64 product (the full product, so every tile of the GEMM's grid, its ragged last
    n-tile at N = 11008 and the tile order over the XCDs are all compared)."""
    from gpu_helpers import assert_close
    W, mask = _layer7b(mid, N, K)
    P = orc.encode(W, mask, 4, 10000)
    X = gs.activations(2048, K, gs.rng_for(4, mid, 2), hot_frac=0.001)
    Y = _run(P, X)
    assert np.isfinite(Y.astype(np.float32)).all()
    ref = orc.linear_f64(P, X)
    assert_close(Y, ref, f"prefill N={N} K={K}")
    # no tile may hide behind the matrix-wide norms: every 256 x 128 tile of Y meets the tolerance on its own
    for m0 in range(0, 2048, 256):
        for n0 in range(0, N, 128):
            assert_close(Y[m0:m0 + 256, n0:n0 + 128], ref[m0:m0 + 256, n0:n0 + 128], f"prefill N={N} K={K} tile {m0},{n0}")


# ----------------------------------------------------------------------------- 70B-shaped layers (config 5)

@functools.lru_cache(maxsize=1)
def _layer70b(mid, N, K):
    """Weights plus a score whose top 1 % is a known set (60 % of it in 1 % of the columns), so the
    oracle needs no sort at this size: the generator returns the positions and the test checks that
    they really are the largest scores."""
    n_top = orc.outlier_count(N, K, 10000)
    W = gs.weight(N, K, gs.rng_for(5, mid, 0))
    S, rows, cols = gs.score_clustered(N, K, n_top, gs.rng_for(5, mid, 1), axis="col")
    mask = np.zeros((N, K), np.uint8)
    mask[rows, cols] = 1
    assert int(mask.sum()) == n_top
    assert S[mask.astype(bool)].min() >= 2.0 > S[~mask.astype(bool)].max()     # the set is the top-k, no ties
    return W, S, mask


def _stratified_channels(N, rng):
    """One channel out of every band of 16 (the decode kernels' tile; eight per 128-wide GEMM tile), plus
    the first and the last channel."""
    starts = np.arange(0, N, 16)
    picks = starts + rng.integers(0, 16, starts.size)
    picks = np.minimum(picks, N - 1)
    return np.unique(np.concatenate([[0, N - 1], picks])).astype(np.int32)


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("mid,N,K", [(0, 8192, 8192), (1, 28672, 8192), (2, 8192, 28672)])
def test_config5_70b_shapes(mid, N, K, bits):
    """Full-size 70B-shaped matrices with column-clustered outliers: gwq_pack byte-exact against the
    oracle's encoding of the known outlier set; gwq_linear at M in {1, 4, 8, 16, 64} on EVERY output
    against the oracle's full product, and at M = 2048 on a stratified sample that has a channel in
    every 16-channel band (so in every tile of both kernels), all 2048 rows of each (K = 28672 takes
    several chunks of K in the kernel for 5 <= M <= 16)."""
    import torch
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close, assert_packed_equal, to_gpu
    W, S, mask = _layer70b(mid, N, K)
    P = orc.encode(W, mask, bits, 10000)
    D = gwq.pack(to_gpu(W), to_gpu(S), bits, 10000)
    assert_packed_equal(D, P)
    for M in (1, 4, 8, 16, 64):
        X = gs.activations(M, K, gs.rng_for(5, mid, 10 + M))
        Y = gwq.linear(D, to_gpu(X)).cpu().numpy()
        assert np.isfinite(Y.astype(np.float32)).all()
        ref = orc.linear_f64(P, X)
        assert_close(Y, ref, f"70B N={N} K={K} bits={bits} M={M}")
        for n0 in range(0, N, 1024):                      # and band by band, so no part hides behind the whole
            assert_close(Y[:, n0:n0 + 1024], ref[:, n0:n0 + 1024], f"70B N={N} K={K} bits={bits} M={M} band {n0}")
    rows = _stratified_channels(N, gs.rng_for(5, mid, 3))
    X = gs.activations(2048, K, gs.rng_for(5, mid, 10 + 2048))
    Y = gwq.linear(D, to_gpu(X)).cpu().numpy()
    assert np.isfinite(Y.astype(np.float32)).all()
    assert_close(Y[:, rows], orc.linear_f64(P, X, rows), f"70B N={N} K={K} bits={bits} M=2048")
    del D
    torch.cuda.empty_cache()


@pytest.mark.parametrize("bits", [4, 3])
def test_pack_time_index_is_the_index_and_gwq_linear_reads_it(bits):
    """gwq_pack fills the layer's optional index; it must equal what gwq_linear_index builds, and gwq_linear must give
    the same bits with it, without it (index built per call) and through gwq_linear_indexed."""
    import dataclasses
    import torch
    import paper_2411_00850_amd as gwq
    from gpu_helpers import to_gpu, assert_close
    N, K = 200, 1408
    rng = np.random.default_rng(90 + bits)
    W = gs.weight(N, K, rng, planted_cols=2)
    S = gs.score_from_weight(W, rng)
    D = gwq.pack(to_gpu(W), to_gpu(S), bits, 10000)
    assert D.index is not None
    built = gwq.linear_index(D)
    assert torch.equal(D.index[:built.numel()], built)
    bare = dataclasses.replace(D, index=None)
    assert gwq.pack(to_gpu(W), to_gpu(S), bits, 10000, with_index=False).index is None
    P = orc.pack(W, S, bits, 10000)
    for M in (17, 64, 300):
        X = gs.activations(M, K, rng)
        Xd = to_gpu(X)
        y_own = gwq.linear(D, Xd)
        y_bare = gwq.linear(bare, Xd)
        y_idx = gwq.linear(bare, Xd, index=built)
        assert torch.equal(y_own, y_bare) and torch.equal(y_own, y_idx), M
        assert_close(y_own.cpu().numpy(), orc.linear_f64(P, X), f"bits={bits} M={M}")


# ----------------------------------------------------------------------------- gated pair: silu(gate) * up in one launch

@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K", [(16, 128), (200, 1024), (333, 4096), (72, 11008), (40, 24576)])
def test_gate_up_fused_decode(bits, N, K):
    """gwq_linear_gate_up against the oracle: silu(X Wg^T) * (X Wu^T) from the oracle's fp64 products.  M <= 4 is
    one launch (both products in the same block), larger M two products and a combining kernel; K = 24576
    is past what the one-launch kernel stages, so it takes the workspace path at every M."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close, to_gpu, upload_packed
    Pg, rng = _problem(500 + N + bits, N, K, bits)
    Pu, _ = _problem(900 + N + bits, N, K, bits)
    Dg, Du = upload_packed(Pg), upload_packed(Pu)
    for M in (1, 2, 3, 4, 5, 9, 16):
        X = gs.activations(M, K, rng)
        H = gwq.linear_gate_up(Dg, Du, to_gpu(X)).cpu().numpy()
        ref = orc.gate_up(orc.linear_f64(Pg, X), orc.linear_f64(Pu, X))
        assert_close(H, ref, f"gate_up N={N} K={K} M={M} bits={bits}")
    if K <= 4096:
        assert gwq.linear_plan([Dg, Du], 1).startswith("decode_small_kernel")     # the plain batch, for comparison


def test_gate_up_7b_shape_full():
    """The 7B gate/up pair (11008 x 4096) at M = 1 and 4, every output."""
    import paper_2411_00850_amd as gwq
    from gpu_helpers import assert_close, to_gpu, upload_packed
    Wg, mg = _layer7b(4, 11008, 4096)
    Pg = orc.encode(Wg, mg, 4, 10000)
    Wu, Su = gs.layer_matrix(2, 5, 11008, 4096)
    Pu = orc.pack(Wu, Su, 4, 10000)
    Dg, Du = upload_packed(Pg), upload_packed(Pu)
    for M in (1, 4):
        X = gs.activations(M, 4096, gs.rng_for(2, 5, 20 + M))
        H = gwq.linear_gate_up(Dg, Du, to_gpu(X)).cpu().numpy()
        assert_close(H, orc.gate_up(orc.linear_f64(Pg, X), orc.linear_f64(Pu, X)), f"gate/up 7B M={M}")
