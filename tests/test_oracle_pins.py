"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test names the passage of the GWQ paper the checked function follows (Sec. 3.2, Eq. 6-10)
and pins it to brute force, exact-rational arithmetic, a library routine or a hand-worked case.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import gwq_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers

def half_fraction(bits):
    """Exact rational value of a finite FP16 pattern, from the format definition."""
    sign = -1 if bits >> 15 else 1
    e, f = (bits >> 10) & 31, bits & 1023
    assert e != 31
    if e == 0:
        return sign * Fraction(f, 1 << 24)
    return sign * Fraction(f | 1024) * Fraction(2) ** (e - 25)


def round_half_even(x: Fraction) -> int:
    return round(x)  # Python rounds Fractions half to even


def clamp(v, lo, hi):
    return max(lo, min(hi, v))


ALL_POS_HALF = np.arange(1, 0x7C00, dtype=np.uint16)            # every positive finite FP16
ALL_POS_HALF_VAL = ALL_POS_HALF.view(np.float16).astype(np.float64)


def brute_scale(R: Fraction, maxq: int) -> int:
    """Smallest FP16 pattern s with s*maxq >= R, by scanning every positive finite FP16 value."""
    ok = ALL_POS_HALF_VAL * maxq >= float(R)     # exact: R is a multiple of 2^-24 below 2^17
    return int(ALL_POS_HALF[np.argmax(ok)])


def exact_group(w_bits, mask, bits):
    """Group quantiser (Eq. 6, 7, 9) in exact rational arithmetic."""
    maxq = (1 << bits) - 1
    vals = [half_fraction(int(b)) for b in w_bits]
    keep = [v for v, m in zip(vals, mask) if not m]
    mn = min([Fraction(0)] + keep)
    mx = max([Fraction(0)] + keep)
    R = mx - mn
    if R == 0:
        s_bits, z = 0x3C00, 0
    else:
        s_bits = brute_scale(R, maxq)
        z = clamp(round_half_even(-mn / half_fraction(s_bits)), 0, maxq)
    s = half_fraction(s_bits)
    q = [z if m else clamp(round_half_even(v / s) + z, 0, maxq) for v, m in zip(vals, mask)]
    return s_bits, z, q


def py_positions(bits):
    """(word, shift) of every k_local in a 128-group, written from the layout statement."""
    pos = []
    for kl in range(128):
        b, r = divmod(kl, 32)
        if bits == 4:
            j, t = divmod(r, 8)
            pos.append((4 * b + j, 16 * (t & 1) + 4 * (t >> 1)))
        elif r < 30:
            i, t = divmod(r, 10)
            pos.append((3 * b + i, 16 * (t & 1) + 3 * (t >> 1)))
        else:
            pos.append((12, 16 * (r - 30) + 3 * b))
    return pos


def py_unpack(qweight, N, K, bits):
    pos = py_positions(bits)
    qw = qweight.reshape(N, K // 128, -1)
    out = np.empty((N, K // 128, 128), np.uint8)
    for kl, (w, sh) in enumerate(pos):
        out[:, :, kl] = (qw[:, :, w] >> np.uint32(sh)) & np.uint32((1 << bits) - 1)
    return out.reshape(N, K)


def numpy_select(score, k_out):
    """Full sort by (|score| bits descending, flat index ascending); first k_out."""
    s32 = score.astype(np.float32)
    key = (s32.view(np.uint32) & np.uint32(0x7FFFFFFF)).ravel().astype(np.int64)
    idx = np.arange(key.size)
    order = np.lexsort((idx, -key))
    mask = np.zeros(key.size, np.uint8)
    mask[order[:k_out]] = 1
    return mask.reshape(score.shape)


def random_w(rng, shape, scale=0.02):
    return (scale * rng.standard_t(4, size=shape)).astype(np.float16)


# ----------------------------------------------------------------------------- FP16 decode

def test_half_to_double_all_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([orc.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ----------------------------------------------------------------------------- Eq. 8: selection

def test_outlier_count_is_ceil_of_fraction():
    assert orc.outlier_count(4096, 4096, 10000) == 167773          # 1 % of 2^24 = 167772.16
    assert orc.outlier_count(11008, 4096, 10000) == 450888
    assert orc.outlier_count(100, 100, 10000) == 100               # exact, no rounding up
    assert orc.outlier_count(7, 128, 0) == 0
    assert orc.outlier_count(7, 128, 1000000) == 7 * 128
    assert orc.outlier_count(3, 128, 1) == 1                        # any positive fraction keeps one


@pytest.mark.parametrize("case", ["random", "all_equal", "two_valued", "fp16", "signed_zero",
                                  "nan_inf", "negatives"])
@pytest.mark.parametrize("ppm", [0, 1, 10000, 250000, 1000000])
def test_select_matches_full_sort(case, ppm):
    rng = np.random.default_rng(hash(case) % 1000 + ppm)
    N, K = 8, 128
    if case == "random":
        S = rng.standard_normal((N, K)).astype(np.float32)
    elif case == "all_equal":
        S = np.full((N, K), 0.5, np.float32)
    elif case == "two_valued":
        S = rng.choice(np.array([0.25, -0.75], np.float32), size=(N, K))
    elif case == "fp16":
        S = (rng.standard_normal((N, K)) * 0.01).astype(np.float16)   # few distinct values: ties
        S = (S.astype(np.float32) * 0 + np.round(S.astype(np.float32) * 200) / 200).astype(np.float16)
    elif case == "signed_zero":
        S = rng.choice(np.array([0.0, -0.0, 1e-30, -1e-30], np.float32), size=(N, K))
    elif case == "nan_inf":
        S = rng.standard_normal((N, K)).astype(np.float32)
        S.ravel()[rng.choice(N * K, 6, replace=False)] = [np.nan, np.inf, -np.inf, np.nan, 3e38, -3e38]
    else:
        S = -np.abs(rng.standard_normal((N, K))).astype(np.float32)
    k_out = orc.outlier_count(N, K, ppm)
    got = orc.select(S, ppm)
    want = numpy_select(S, k_out)
    assert int(got.sum()) == k_out
    assert np.array_equal(got, want)


def test_select_invariants_and_tie_rule():
    rng = np.random.default_rng(5)
    N, K = 16, 256
    S = (np.round(rng.standard_normal((N, K)) * 4) / 4).astype(np.float32)   # heavy ties
    ppm = 100000
    k_out = orc.outlier_count(N, K, ppm)
    mask = orc.select(S, ppm).ravel().astype(bool)
    a = np.abs(S).ravel()
    assert mask.sum() == k_out
    thr = a[mask].min()
    assert a[~mask].max() <= thr
    tie = a == thr
    sel_tie = np.flatnonzero(tie & mask)
    unsel_tie = np.flatnonzero(tie & ~mask)
    assert unsel_tie.size > 0 and sel_tie.size > 0       # the case really has a tie at the cut
    assert sel_tie.max() < unsel_tie.min()               # ties go to the lowest flat index


@pytest.mark.parametrize("ppm", [1, 10000, 31000, 500000])
def test_select_fp16_scores_every_pattern_incl_nan_payloads(ppm):
    """FP16 scores are ranked by the binary32 pattern of their exact widening; a NaN keeps sign and
    payload (shifted into the binary32 fraction) and so ranks above +inf, larger payloads first.  Pinned
    to numpy's binary16 -> binary32 conversion on all 65 536 patterns, shuffled: 2046 NaNs, both
    infinities, both zeros, every subnormal.  31 000 ppm cuts inside the NaN block."""
    rng = np.random.default_rng(ppm)
    bits = rng.permutation(np.arange(65536, dtype=np.uint16))
    S = bits.view(np.float16).reshape(512, 128)
    wide = S.astype(np.float32).view(np.uint32).ravel()
    nan = ((bits >> 10) & 31 == 31) & (bits & 1023 != 0)
    assert nan.sum() == 2046
    assert np.array_equal(wide[nan] & 0x7FFFFFFF, 0x7F800000 | ((bits[nan].astype(np.uint32) & 1023) << 13))
    k_out = orc.outlier_count(512, 128, ppm)
    got = orc.select(S, ppm)
    assert int(got.sum()) == k_out
    assert np.array_equal(got, numpy_select(S, k_out))
    if k_out >= 2046:
        assert got.ravel()[nan].all()                      # every NaN outranks every number
    else:
        assert not got.ravel()[~nan].any()                 # and the cut inside the NaNs takes NaNs only


def test_select_rejects_bad_ppm():
    with pytest.raises(RuntimeError):
        orc.select(np.zeros((2, 128), np.float32), 1000001)


# ----------------------------------------------------------------------------- CSR

def test_csr_invariants():
    rng = np.random.default_rng(11)
    N, K = 24, 384
    W = random_w(rng, (N, K))
    W[3, 7] = np.float16(-0.0)
    S = rng.random((N, K)).astype(np.float32)
    S[3, 7] = 9.0
    mask = orc.select(S, 20000)
    row_ptr, col, val = orc.csr(W, mask)
    assert row_ptr[0] == 0 and row_ptr[-1] == mask.sum() and np.all(np.diff(row_ptr) >= 0)
    rebuilt = np.zeros_like(mask)
    for n in range(N):
        c = col[row_ptr[n]:row_ptr[n + 1]].astype(np.int64)
        assert np.all(np.diff(c) > 0)
        rebuilt[n, c] = 1
        assert np.array_equal(val[row_ptr[n]:row_ptr[n + 1]], W.view(np.uint16)[n, c])
    assert np.array_equal(rebuilt, mask)
    assert val[np.flatnonzero(col[row_ptr[3]:row_ptr[4]] == 7)[0] + row_ptr[3]] == 0x8000  # -0 kept


# ----------------------------------------------------------------------------- Eq. 6, 7, 9: one group

def _golden_groups():
    rows = []
    with open(os.path.join(GOLDEN, "quant_group_examples.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            b, w, m, s, z, q = [x.strip() for x in line.split(";")]
            rows.append((int(b), [float(x) for x in w.split()], [int(x) for x in m.split()],
                         int(s, 16), int(z), [int(x) for x in q.split()]))
    return rows


@pytest.mark.parametrize("row", _golden_groups())
def test_quant_group_hand_examples(row):
    bits, w, mask, s_want, z_want, q_want = row
    w16 = np.array(w, np.float16)
    assert np.array_equal(w16.astype(np.float64), np.array(w))      # fixture values are exact FP16
    s, z, q = orc.quant_group(w16, np.array(mask, np.uint8), bits)
    assert (s, z, list(q)) == (s_want, z_want, q_want)
    # the hand-worked line itself agrees with exact-rational arithmetic
    assert exact_group(w16.view(np.uint16), mask, bits) == (s_want, z_want, q_want)


@pytest.mark.parametrize("bits", [3, 4])
def test_quant_group_matches_exact_rationals(bits):
    rng = np.random.default_rng(100 + bits)
    for trial in range(150):
        n = int(rng.choice([2, 8, 32, 128]))
        kind = trial % 5
        if kind == 0:
            w = random_w(rng, n)
        elif kind == 1:
            w = random_w(rng, n, scale=30.0)                            # large magnitudes
        elif kind == 2:
            w = (rng.integers(-40, 40, n) * 2.0 ** -24).astype(np.float16)  # subnormals
        elif kind == 3:
            w = np.abs(random_w(rng, n)) * (1 if trial % 2 else -1)    # one-sided groups
        else:
            w = (rng.integers(-15, 16, n) / 64.0).astype(np.float16)   # many exact half-step ties
        mask = (rng.random(n) < (0.0, 0.05, 0.5)[trial % 3]).astype(np.uint8)
        s, z, q = orc.quant_group(w, mask, bits)
        assert (s, z, list(q)) == exact_group(w.view(np.uint16), mask, bits), (trial, w, mask)


@pytest.mark.parametrize("bits", [3, 4])
def test_scale_is_minimal_and_error_within_half_step(bits):
    """Invariants: s*maxq >= R > prev(s)*maxq; |s*(q-z) - w| <= s/2 for every non-outlier."""
    rng = np.random.default_rng(7 + bits)
    maxq = (1 << bits) - 1
    worst = Fraction(0)
    for trial in range(100):
        w = random_w(rng, 128, scale=(0.02, 1.0, 200.0)[trial % 3])
        mask = (rng.random(128) < 0.02).astype(np.uint8)
        s_bits, z, q = orc.quant_group(w, mask, bits)
        vals = [half_fraction(int(b)) for b in w.view(np.uint16)]
        keep = [v for v, m in zip(vals, mask) if not m]
        R = max([Fraction(0)] + keep) - min([Fraction(0)] + keep)
        s = half_fraction(s_bits)
        assert s * maxq >= R and half_fraction(s_bits - 1) * maxq < R
        assert 0 <= z <= maxq
        for v, m, c in zip(vals, mask, q):
            if m:
                assert c == z
            else:
                err = abs(s * (int(c) - z) - v)
                assert err <= s / 2
                worst = max(worst, err / s)
        if min(keep) < 0:
            assert q[int(np.argmin(np.where(mask, np.inf, w.astype(np.float64))))] == 0
        assert q[int(np.argmax(np.where(mask, -np.inf, w.astype(np.float64))))] >= maxq - 1
    assert worst > Fraction(2, 5)          # the bound is nearly attained, i.e. the test has teeth


# ----------------------------------------------------------------------------- word layout

def _golden_words():
    rows = []
    with open(os.path.join(GOLDEN, "word_layout_examples.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            b, kind, c, w = [x.strip() for x in line.split(";")]
            rows.append((int(b), kind, [int(x) for x in c.split()], int(w, 16)))
    return rows


@pytest.mark.parametrize("row", _golden_words())
def test_word_layout_hand_examples(row):
    bits, kind, codes, word = row
    full = np.zeros((1, 128), np.uint8)
    if kind == "word":
        per = 8 if bits == 4 else 10
        # put the example into word 5 of the group: slot 1, second word of that slot
        slot, j = 1, 1
        widx = (4 if bits == 4 else 3) * slot + j
        base = 32 * slot + per * j
        full[0, base:base + per] = codes
    else:
        widx = 12
        for b in range(4):
            full[0, 32 * b + 30] = codes[2 * b]
            full[0, 32 * b + 31] = codes[2 * b + 1]
    qw = orc.pack_codes(full, bits)
    assert qw.shape == (1, 1, 16 if bits == 4 else 13)
    assert int(qw[0, 0, widx]) == word
    others = np.delete(qw[0, 0], widx)
    assert not others.any()


@pytest.mark.parametrize("bits", [3, 4])
def test_pack_unpack_roundtrip_and_padding(bits):
    rng = np.random.default_rng(bits)
    N, K = 5, 384
    codes = rng.integers(0, 1 << bits, (N, K)).astype(np.uint8)
    qw = orc.pack_codes(codes, bits)
    assert np.array_equal(orc.unpack_codes(qw, N, K, bits), codes)
    assert np.array_equal(py_unpack(qw, N, K, bits), codes)      # independent index map
    if bits == 3:
        assert not (qw[:, :, :12] & np.uint32(0x80008000)).any()  # bits 15 and 31 unused
        assert not (qw[:, :, 12] & np.uint32(0xF000F000)).any()   # tail uses 12 bits per half
    all_ones = orc.pack_codes(np.full((1, 128), (1 << bits) - 1, np.uint8), bits)
    want = [0xFFFFFFFF] * 16 if bits == 4 else [0x7FFF7FFF] * 12 + [0x0FFF0FFF]
    assert [int(x) for x in all_ones[0, 0]] == want


# ----------------------------------------------------------------------------- whole encoding

def _small_problem(seed, N=12, K=384, planted=True):
    rng = np.random.default_rng(seed)
    W = random_w(rng, (N, K))
    if planted:
        W[:, 5] = (W[:, 5].astype(np.float32) * 20).astype(np.float16)
    S = (np.abs(rng.standard_normal((N, K))) * np.abs(W.astype(np.float32))).astype(np.float32)
    return W, S


@pytest.mark.parametrize("group", [128, 64, 32, 16])
@pytest.mark.parametrize("bits", [3, 4])
@pytest.mark.parametrize("ppm", [0, 10000, 300000])
def test_pack_is_composition_of_pinned_steps(bits, ppm, group):
    """Every group size of Sec. 3.2 (beta: the paper's 16, and 32, 64, 128): scale, zero point and codes of every
    group equal the exact-rational quantiser on that group's `group` weights; the word layout (128-code blocks)
    and the CSR do not depend on the group size."""
    W, S = _small_problem(bits * 10 + ppm % 7)
    N, K = W.shape
    P = orc.pack(W, S, bits, ppm, group)
    assert P.scales.shape == P.zeros.shape == (N, K // group)
    k_out = orc.outlier_count(N, K, ppm)
    mask = numpy_select(S, k_out)
    assert np.array_equal(P.mask, mask)
    assert P.row_ptr[-1] == k_out
    codes = py_unpack(P.qweight, N, K, bits)
    Wb = W.view(np.uint16)
    for n in range(N):
        for g in range(K // group):
            sl = slice(group * g, group * g + group)
            s, z, q = exact_group(Wb[n, sl], mask[n, sl], bits)
            assert (int(P.scales[n, g]), int(P.zeros[n, g])) == (s, z)
            assert list(codes[n, sl]) == q
    # outlier positions reproduced exactly, values bit-exact
    for n in range(N):
        c = P.col_idx[P.row_ptr[n]:P.row_ptr[n + 1]].astype(np.int64)
        assert np.array_equal(np.flatnonzero(mask[n]), c)
        assert np.array_equal(P.out_val[P.row_ptr[n]:P.row_ptr[n + 1]], Wb[n, c])


@pytest.mark.parametrize("group", [128, 64, 32, 16])
@pytest.mark.parametrize("bits", [3, 4])
def test_no_outliers_is_plain_group_rtn(bits, group):
    """ppm = 0 reduces to group-wise min-max round-to-nearest (the quantiser the paper's first
    table names), written here with numpy: s from the minimal-FP16 rule, codes by np.rint."""
    W, S = _small_problem(77)
    N, K = W.shape
    maxq = (1 << bits) - 1
    P = orc.pack(W, S, bits, 0, group)
    assert P.row_ptr[-1] == 0 and not P.mask.any()
    Wd = W.astype(np.float64).reshape(N, K // group, group)
    mn = np.minimum(Wd.min(-1), 0.0)
    mx = np.maximum(Wd.max(-1), 0.0)
    s = P.scales.view(np.float16).astype(np.float64)
    assert np.all(s * maxq >= mx - mn)
    z = np.clip(np.rint(-mn / s), 0, maxq)
    q = np.clip(np.rint(Wd / s[..., None]) + z[..., None], 0, maxq)
    assert np.array_equal(P.zeros, z.astype(np.uint8))
    assert np.array_equal(py_unpack(P.qweight, N, K, bits), q.reshape(N, K).astype(np.uint8))
    deq = orc.decode(P)
    assert np.all(np.abs(deq.reshape(Wd.shape) - Wd) <= s[..., None] / 2)


@pytest.mark.parametrize("bits", [3, 4])
def test_all_outliers_is_dense_fp16_matmul(bits):
    """ppm = 1e6 keeps every weight in FP16: decode gives W itself and the layer is X W^T."""
    W, S = _small_problem(3, N=10, K=256)
    rng = np.random.default_rng(4)
    X = rng.standard_normal((3, 256)).astype(np.float16)
    P = orc.pack(W, S, bits, 1000000)
    assert np.array_equal(orc.decode(P), W.astype(np.float64))
    want = X.astype(np.float64) @ W.astype(np.float64).T
    got = orc.linear_f64(P, X)
    assert got.shape == (3, 10)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("bits", [3, 4])
def test_non_finite_weights_stay_local_and_keep_the_invariants(bits):
    """Weights that are inf or NaN: their values are unspecified, but (a) the selection does not look at
    W, so the count and the positions are those of the finite matrix; (b) a non-finite weight that is an
    outlier is only copied, bit for bit, so the rest of the encoding equals that of the matrix with the
    weight replaced by 0; (c) a non-finite weight that is quantised can only change its own group; (d)
    every stored field stays in range (zero points, the unused bits of 3-bit words, CSR structure)."""
    rng = np.random.default_rng(400 + bits)
    N, K = 12, 512
    W = random_w(rng, (N, K))
    S = rng.random((N, K)).astype(np.float32)
    ppm = 20000
    specials = np.array([0x7C00, 0xFC00, 0x7E00, 0xFE01, 0x7C01, 0x7FFF], np.uint16)   # +-inf, quiet and signalling NaNs
    flat = rng.choice(N * K, 24, replace=False)
    kept, quantised = flat[:12], flat[12:]
    S.ravel()[kept] = 5.0 + np.arange(12)                  # these are certainly selected
    S.ravel()[quantised] = 0.0                             # these certainly are not
    Wb = W.view(np.uint16).copy()
    Wb.ravel()[kept] = np.tile(specials, 2)
    clean = Wb.copy()
    clean.ravel()[kept] = 0
    # (a), (b): non-finite outliers
    P, C = orc.pack(Wb.view(np.float16), S, bits, ppm), orc.pack(clean.view(np.float16), S, bits, ppm)
    assert np.array_equal(P.mask, C.mask) and P.mask.ravel()[kept].all()
    for name in ("qweight", "scales", "zeros", "row_ptr", "col_idx"):
        assert np.array_equal(getattr(P, name), getattr(C, name)), name
    pos = {int(f): j for j, f in enumerate(np.flatnonzero(P.mask.ravel()))}
    for f, pat in zip(kept, np.tile(specials, 2)):
        assert P.out_val[pos[int(f)]] == pat               # NaN payloads and signs survive
    # (c), (d): non-finite weights inside the quantised part
    Wq = clean.copy()
    Wq.ravel()[quantised] = np.tile(specials, 2)
    Q = orc.pack(Wq.view(np.float16), S, bits, ppm)
    assert np.array_equal(Q.mask, C.mask) and np.array_equal(Q.row_ptr, C.row_ptr) and np.array_equal(Q.col_idx, C.col_idx)
    assert np.array_equal(Q.out_val, C.out_val)
    touched = np.zeros((N, K // 128), bool)
    touched[quantised // K, (quantised % K) // 128] = True
    assert np.array_equal(Q.qweight[~touched], C.qweight[~touched])
    assert np.array_equal(Q.scales[~touched], C.scales[~touched]) and np.array_equal(Q.zeros[~touched], C.zeros[~touched])
    assert Q.zeros.max() <= (1 << bits) - 1
    if bits == 3:
        assert not (Q.qweight[:, :, :12] & np.uint32(0x80008000)).any()
        assert not (Q.qweight[:, :, 12] & np.uint32(0xF000F000)).any()
    assert np.array_equal(py_unpack(Q.qweight, N, K, bits) <= (1 << bits) - 1, np.ones((N, K), bool))
    assert np.array_equal(orc.unpack_codes(Q.qweight, N, K, bits)[Q.mask.astype(bool)],
                          np.repeat(Q.zeros, 128).reshape(N, K)[Q.mask.astype(bool)])   # outliers still carry z


# ----------------------------------------------------------------------------- Eq. 10 + the layer

@pytest.mark.parametrize("group", [128, 64, 32, 16])
@pytest.mark.parametrize("bits", [3, 4])
def test_decode_and_linear_match_numpy(bits, group):
    W, S = _small_problem(21 + bits, N=20, K=512)
    N, K = W.shape
    rng = np.random.default_rng(9)
    X = rng.standard_normal((5, K)).astype(np.float16)
    P = orc.pack(W, S, bits, 10000, group)
    # independent decode: Python index map, s*(q-z), outliers from the CSR arrays
    q = py_unpack(P.qweight, N, K, bits).astype(np.float64).reshape(N, K // group, group)
    s = P.scales.view(np.float16).astype(np.float64)[..., None]
    z = P.zeros.astype(np.float64)[..., None]
    What = (s * (q - z)).reshape(N, K)
    for n in range(N):
        for j in range(P.row_ptr[n], P.row_ptr[n + 1]):
            assert What[n, P.col_idx[j]] == 0.0                    # code under an outlier decodes to 0
            What[n, P.col_idx[j]] = float(P.out_val[j:j + 1].view(np.float16)[0])
    assert np.array_equal(orc.decode(P), What)
    want = X.astype(np.float64) @ What.T
    got = orc.linear_f64(P, X)
    assert got.shape == (5, N)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    rows = np.array([19, 0, 7], np.int32)
    assert np.allclose(orc.linear_f64(P, X, rows), want[:, rows], rtol=1e-12, atol=1e-12)
    # activations handed over as fp64 values: the same sums bit for bit when they are FP16 values, and the numpy
    # product for bfloat16 values (widened exactly from their bit patterns: 1.0, -2.5, 2^-20, 3 * 2^100)
    assert np.array_equal(orc.linear_f64_x(P, X.astype(np.float64)), got)
    assert np.array_equal(orc.bf16_bits_to_f64(np.array([0x3F80, 0xC020, 0x3580, 0x7240, 0x0000, 0x8000], np.uint16)),
                          np.array([1.0, -2.5, 2.0 ** -20, 3 * 2.0 ** 100, 0.0, -0.0]))
    Xb = (rng.standard_normal((3, K)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    Xb[0, :4] = [0x7240, 0x0A00, 0x3F80, 0xC020]          # far outside the FP16 range on both ends
    Xd = orc.bf16_bits_to_f64(Xb)
    assert np.allclose(orc.linear_f64_x(P, Xd), Xd @ What.T, rtol=1e-12, atol=0)
    assert np.allclose(orc.linear_f64_x(P, Xd, rows), (Xd @ What.T)[:, rows], rtol=1e-12, atol=0)
    # sanity, not parity: the quantised layer is close to the FP16 layer, closer at 4 bits than at 3
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert rel < (0.25 if bits == 3 else 0.12)


@pytest.mark.parametrize("bits", [3, 4])
def test_smaller_groups_quantise_no_worse(bits):
    """A group's range can only shrink when the group is cut in two, so the squared error (Eq. 4) of the paper's
    group size 16 is at most that of 32, 64, 128 up to the scale's FP16 rounding - here clearly below; and
    the figures of merit follow the group size (max |W - W_Q| <= s / 2 of the group the weight lies in)."""
    W, S = _small_problem(123, N=16, K=512)
    sq = {}
    for group in (128, 64, 32, 16):
        P = orc.pack(W, S, bits, 10000, group)
        sq[group], _, mx = orc.quality(P, W, S)
        s = P.scales.view(np.float16).astype(np.float64)
        assert mx <= s.max() / 2
        D = np.abs(W.astype(np.float64) - orc.decode(P))
        assert np.all(D <= np.repeat(s, group, axis=1) / 2)
        assert np.isclose(sq[group], (D ** 2).sum(), rtol=1e-12)
    assert sq[16] < sq[32] < sq[64] < sq[128]


def test_four_bits_beat_three_bits():
    W, S = _small_problem(50, N=16, K=512)
    X = np.random.default_rng(1).standard_normal((4, 512)).astype(np.float16)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    err = {}
    for bits in (3, 4):
        err[bits] = np.linalg.norm(orc.linear_f64(orc.pack(W, S, bits, 10000), X) - ref)
    assert err[4] < err[3]


# ----------------------------------------------------------------------------- Sec. 3.1, Eq. 3-5: figures of merit

@pytest.mark.parametrize("row", [r for r in _golden_groups() if 128 % len(r[1]) == 0 and len(r[1]) >= 2])
def test_quality_on_hand_worked_groups(row):
    """|| W - W_Q ||^2 (Eq. 4), g^T (W - W_Q) (Eq. 3, 5) and max |W - W_Q| of a one-channel layer made
    of one hand-worked group repeated to 128 columns, against exact rationals computed from the
    fixture's own scale, zero point and codes (not from the oracle's decoder).  The scores ascend
    with the column and are negative in the second half, so a swapped sign, a dropped outlier or a
    shifted index all change the expected numbers."""
    bits, w, mask, s_bits, z, codes = row
    reps = 128 // len(w)
    W = np.array(w * reps, np.float16).reshape(1, 128)
    M = np.array(mask * reps, np.uint8).reshape(1, 128)
    g = np.where(np.arange(128) < 64, np.arange(128) + 1, -(np.arange(128) + 1)).astype(np.float32).reshape(1, 128)
    P = orc.encode(W, M, bits)
    assert int(P.scales[0, 0]) == s_bits and int(P.zeros[0, 0]) == z           # the tiling keeps the group's range
    s = half_fraction(s_bits)
    sq = first = mx = Fraction(0)
    for k in range(128):
        i = k % len(w)
        w_q = Fraction(w[i]) if mask[i] else s * (codes[i] - z)
        d = Fraction(w[i]) - w_q
        sq += d * d
        first += Fraction(int(g[0, k])) * d
        mx = max(mx, abs(d))
    got = orc.quality(P, W, g)
    for have, want in zip(got, (sq, first, mx)):
        assert abs(Fraction(have) - want) <= abs(want) * Fraction(1, 10 ** 13)
    if any(mask) and not all(mask):
        # the same layer without its outliers kept: a different (larger) error, so the CSR part matters
        assert orc.quality(orc.encode(W, np.zeros_like(M), bits), W, g)[0] != got[0]


@pytest.mark.parametrize("bits", [3, 4])
def test_quality_special_cases_and_invariants(bits):
    W, S = _small_problem(60 + bits, N=24, K=384)
    # everything kept in FP16: no error at all
    assert orc.quality(orc.pack(W, S, bits, 1000000), W, S) == (0.0, 0.0, 0.0)
    P = orc.pack(W, S, bits, 10000)
    D = W.astype(np.float64) - orc.decode(P)
    sq, first, mx = orc.quality(P, W, S)
    # definitions through numpy's own reductions
    assert np.isclose(sq, np.sum(D * D), rtol=1e-12)
    assert np.isclose(first, np.sum(S.astype(np.float64) * D), rtol=1e-9, atol=1e-12 * np.sum(np.abs(S * D)))
    assert mx == np.max(np.abs(D))
    # with the error itself as the score the two sums coincide (D is exact in FP32 here: few bits)
    Dg = D.astype(np.float32)
    assert np.array_equal(Dg.astype(np.float64), D)
    sq2, first2, _ = orc.quality(P, W, Dg)
    assert np.isclose(first2, sq2, rtol=1e-12)
    # half a step bounds the error of every kept weight (the scale never clips), outliers have none
    s_max = float(P.scales.view(np.float16).astype(np.float64).max())
    assert mx <= s_max / 2 * (1 + 1e-12)
    assert mx * mx <= sq <= W.size * mx * mx
    # FP16 scores give the same numbers as their FP32 widening
    S16 = S.astype(np.float16)
    assert orc.quality(P, W, S16) == orc.quality(P, W, S16.astype(np.float32))


# ----------------------------------------------------------------------------- gated pair (silu(gate) * up)

def test_gate_up_closed_forms_and_identities():
    """silu(x) = x * sigmoid(x): exact values where the sigmoid is rational (sigmoid(ln 3) = 3/4, sigmoid(ln 7) = 7/8,
    sigmoid(0) = 1/2), the identity silu(x) - silu(-x) = x, the limits silu(x) -> x and silu(-x) -> 0 for large x,
    the slope 1/2 at 0 - and the second factor entering linearly."""
    ln3, ln7 = np.log(3.0), np.log(7.0)
    G = np.array([0.0, ln3, -ln3, ln7, -ln7, 40.0, -40.0, 745.0, -745.0, 1e-9])
    one = np.ones_like(G)
    H = orc.gate_up(G, one)
    want = [0.0, 0.75 * ln3, -0.25 * ln3, 0.875 * ln7, -0.125 * ln7, 40.0, 0.0, 745.0, 0.0, 0.5e-9]
    assert np.allclose(H, want, rtol=1e-14, atol=1e-15)
    assert np.isfinite(H).all() and H[8] <= 0.0 and abs(H[8]) < 1e-300        # no overflow of exp on the way
    rng = np.random.default_rng(3)
    x = rng.standard_normal(1000) * 5
    assert np.allclose(orc.gate_up(x, np.ones_like(x)) - orc.gate_up(-x, np.ones_like(x)), x, rtol=1e-13, atol=1e-15)
    u = rng.standard_normal(1000)
    assert np.allclose(orc.gate_up(x, 3.0 * u), 3.0 * orc.gate_up(x, u), rtol=1e-15)
    assert np.array_equal(orc.gate_up(x, np.zeros_like(x)), np.zeros_like(x) * x)
    # a transposed pair of arguments would fail this: silu acts on the first factor only
    assert not np.allclose(orc.gate_up(x, u), orc.gate_up(u, x))
    # shape is kept, elementwise
    Hm = orc.gate_up(x.reshape(10, 100), u.reshape(10, 100))
    assert Hm.shape == (10, 100) and np.array_equal(Hm.ravel(), orc.gate_up(x, u))


# ----------------------------------------------------------------------------- score of one layer (Eq. 2)

def test_score_hand_worked_case():
    """Eq. 2 with the chain rule for Y = X W^T, on a case worked by hand (tests/golden/score_hand_worked.txt)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "score_hand_worked.txt")) if l.strip() and l[0] != "#"]
    M, N, K = map(int, rows[0])
    num = lambda rs: np.array([[float(v) for v in r] for r in rs])
    dY, X, want = num(rows[1:1 + M]), num(rows[1 + M:1 + 2 * M]), num(rows[1 + 2 * M:1 + 2 * M + N])
    assert dY.shape == (M, N) and X.shape == (M, K) and want.shape == (N, K)
    got = orc.score(dY.astype(np.float16), X.astype(np.float16))
    assert np.array_equal(got, want)
    # asymmetric on purpose: the transposed product, or rows taken for columns, gives other numbers
    assert not np.array_equal(got, (X.T @ dY).T[:, ::-1])


def test_score_is_the_derivative_of_a_loss():
    """The score is the gradient of the loss with respect to W (Eq. 2).  For the squared-error loss
    L(W) = 1/2 sum (X W^T - T)^2 the gradient with respect to Y is Y - T, and L is quadratic in each
    weight, so a central difference of L is its exact derivative: the oracle must agree with it entry by
    entry.  Values are small dyadic rationals, so every quantity is exact in fp64."""
    rng = np.random.default_rng(11)
    M, N, K = 5, 4, 6
    X = rng.integers(-8, 9, (M, K)) / 4.0
    W = rng.integers(-8, 9, (N, K)) / 8.0
    T = rng.integers(-8, 9, (M, N)) / 2.0
    loss = lambda w: 0.5 * ((X @ w.T - T) ** 2).sum()
    dY = X @ W.T - T
    assert np.array_equal(dY.astype(np.float16).astype(np.float64), dY)
    got = orc.score(dY.astype(np.float16), X.astype(np.float16))
    for n in range(N):
        for k in range(K):
            up, dn = W.copy(), W.copy()
            up[n, k] += 1.0
            dn[n, k] -= 1.0
            assert got[n, k] == (loss(up) - loss(dn)) / 2.0, (n, k)


def test_score_special_cases_and_linearity():
    rng = np.random.default_rng(12)
    M, N, K = 7, 5, 9
    dY = rng.standard_normal((M, N)).astype(np.float16)
    X = rng.standard_normal((M, K)).astype(np.float16)
    # one sample: the outer product, each entry one exact product of two FP16 numbers
    one = orc.score(dY[:1], X[:1])
    for n in range(N):
        for k in range(K):
            assert Fraction(float(one[n, k])) == Fraction(float(dY[0, n])) * Fraction(float(X[0, k]))
    # a sum over samples, in the order of m: exact rationals, rounded by fp64 additions
    full = orc.score(dY, X)
    for n, k in ((0, 0), (4, 8), (2, 3)):
        acc = 0.0
        for m in range(M):
            acc += float(dY[m, n]) * float(X[m, k])
        assert full[n, k] == acc
        exact = sum(Fraction(float(dY[m, n])) * Fraction(float(X[m, k])) for m in range(M))
        assert abs(Fraction(full[n, k]) - exact) <= Fraction(1, 2 ** 45)
    # a unit dY picks a row of X: dY[m][n] = 1 only at (m0, n0) -> g[n0] = X[m0], all other rows 0
    unit = np.zeros((M, N), np.float16)
    unit[3, 2] = 1.0
    g = orc.score(unit, X)
    assert np.array_equal(g[2], X[3].astype(np.float64)) and not g[[0, 1, 3, 4]].any()
    # mean over samples (Sec. 4.3) as a scaled accumulation: two halves with alpha = 1/2
    prev = orc.score(dY[:4], X[:4], alpha=0.5).astype(np.float32)
    both = orc.score(dY[4:], X[4:], alpha=0.5, beta=1.0, prev=prev)
    want = prev.astype(np.float64) + 0.5 * orc.score(dY[4:], X[4:])
    assert np.array_equal(both, want)
    assert np.allclose(both, 0.5 * full, rtol=0, atol=1e-6)
    # beta = 0 ignores prev altogether, NaN included
    nan_prev = np.full((N, K), np.nan, np.float32)
    assert np.array_equal(orc.score(dY, X, alpha=2.0, beta=0.0, prev=nan_prev), 2.0 * full)
