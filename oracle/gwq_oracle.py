"""ctypes front end of the C oracle (oracle/gwq_oracle.c).  TEST INFRASTRUCTURE ONLY.

Every function takes and returns numpy arrays in host memory.  Nothing here is imported by
the GPU package; only tests, the smoke check and the benchmark's CPU-baseline leg use it.
The arithmetic lives in the C file; this module only marshals arguments.
"""
import ctypes
import os
from dataclasses import dataclass

import numpy as np

from . import build_oracle

GROUP = 128


def _load():
    lib = ctypes.CDLL(build_oracle.build(force=False))
    i64, u32, i32, vp = ctypes.c_int64, ctypes.c_uint32, ctypes.c_int, ctypes.c_void_p
    lib.gwq_oracle_half_to_double.restype = ctypes.c_double
    lib.gwq_oracle_half_to_double.argtypes = [ctypes.c_uint16]
    lib.gwq_oracle_outlier_count.restype = i64
    lib.gwq_oracle_outlier_count.argtypes = [i64, i64, u32]
    lib.gwq_oracle_select.argtypes = [vp, i32, i64, i64, u32, vp]
    lib.gwq_oracle_csr.argtypes = [vp, vp, i64, i64, vp, vp, vp]
    lib.gwq_oracle_quant_group.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    lib.gwq_oracle_pack_codes.argtypes = [vp, i64, i64, i32, vp]
    lib.gwq_oracle_unpack_codes.argtypes = [vp, i64, i64, i32, vp]
    lib.gwq_oracle_encode.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.gwq_oracle_pack.argtypes = [vp, vp, i32, i64, i64, i32, i32, u32, vp, vp, vp, vp, vp, vp, vp]
    lib.gwq_oracle_decode.argtypes = [i64, i64, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.gwq_oracle_linear_f64.argtypes = [i64, i64, i32, i32, vp, vp, vp, vp, vp, vp, vp, i64, vp, i64, vp]
    lib.gwq_oracle_linear_f64_x.argtypes = [i64, i64, i32, i32, vp, vp, vp, vp, vp, vp, vp, i64, vp, i64, vp]
    lib.gwq_oracle_quality.argtypes = [i64, i64, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
    lib.gwq_oracle_gate_up.argtypes = [vp, vp, i64, vp]
    lib.gwq_oracle_score.argtypes = [vp, vp, i64, i64, i64, ctypes.c_double, ctypes.c_double, vp, vp]
    return lib


_lib = _load()


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _chk(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed with oracle status {rc}")


def _f16_bits(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    if a.dtype == np.uint16:
        return a
    raise TypeError("expected float16 (or its uint16 bit patterns)")


def _score(score):
    score = np.ascontiguousarray(score)
    if score.dtype == np.float32:
        return score, 0
    if score.dtype == np.float16:
        return score, 1
    raise TypeError("score must be float32 or float16")


def words_per_group(bits):
    return {4: 16, 3: 13}[bits]


def outlier_count(N, K, ppm):
    return int(_lib.gwq_oracle_outlier_count(N, K, ppm))


def half_to_double(bits):
    return float(_lib.gwq_oracle_half_to_double(int(bits)))


def select(score, ppm):
    score, is16 = _score(score)
    N, K = score.shape
    mask = np.empty((N, K), np.uint8)
    _chk(_lib.gwq_oracle_select(_p(score), is16, N, K, ppm, _p(mask)), "select")
    return mask


def csr(W, mask):
    Wb = _f16_bits(W)
    N, K = Wb.shape
    mask = np.ascontiguousarray(mask, np.uint8)
    nnz = int(mask.sum())
    row_ptr = np.empty(N + 1, np.int32)
    col_idx = np.empty(nnz, np.uint16)
    val = np.empty(nnz, np.uint16)
    _chk(_lib.gwq_oracle_csr(_p(Wb), _p(mask), N, K, _p(row_ptr), _p(col_idx), _p(val)), "csr")
    return row_ptr, col_idx, val


def quant_group(w, mask, bits):
    wb = _f16_bits(w)
    mask = np.ascontiguousarray(mask, np.uint8)
    s = np.zeros(1, np.uint16)
    z = np.zeros(1, np.uint8)
    q = np.empty(wb.size, np.uint8)
    _chk(_lib.gwq_oracle_quant_group(_p(wb), _p(mask), wb.size, bits, _p(s), _p(z), _p(q)), "quant_group")
    return int(s[0]), int(z[0]), q


def pack_codes(codes, bits):
    codes = np.ascontiguousarray(codes, np.uint8)
    N, K = codes.shape
    out = np.empty((N, K // GROUP, words_per_group(bits)), np.uint32)
    _chk(_lib.gwq_oracle_pack_codes(_p(codes), N, K, bits, _p(out)), "pack_codes")
    return out


def unpack_codes(qweight, N, K, bits):
    qweight = np.ascontiguousarray(qweight, np.uint32)
    out = np.empty((N, K), np.uint8)
    _chk(_lib.gwq_oracle_unpack_codes(_p(qweight), N, K, bits, _p(out)), "unpack_codes")
    return out


@dataclass
class Packed:
    N: int
    K: int
    bits: int
    ppm: int
    qweight: np.ndarray   # uint32 [N, K/128, words_per_group]
    scales: np.ndarray    # uint16 (FP16 bits) [N, K/group]
    zeros: np.ndarray     # uint8 [N, K/group]
    row_ptr: np.ndarray   # int32 [N+1]
    col_idx: np.ndarray   # uint16 [k_out]
    out_val: np.ndarray   # uint16 (FP16 bits) [k_out]
    mask: np.ndarray      # uint8 [N, K] outlier indicator (not part of the stored format)
    group: int = GROUP    # weights per scale and zero point: 16, 32, 64 or 128


def pack(W, score, bits, ppm=10000, group=GROUP):
    Wb = _f16_bits(W)
    score, is16 = _score(score)
    N, K = Wb.shape
    assert score.shape == (N, K)
    k_out = outlier_count(N, K, ppm)
    P = Packed(N, K, bits, ppm,
               np.empty((N, K // GROUP, words_per_group(bits)), np.uint32),
               np.empty((N, K // group), np.uint16), np.empty((N, K // group), np.uint8),
               np.empty(N + 1, np.int32), np.empty(k_out, np.uint16), np.empty(k_out, np.uint16),
               np.empty((N, K), np.uint8), group)
    _chk(_lib.gwq_oracle_pack(_p(Wb), _p(score), is16, N, K, bits, group, ppm, _p(P.qweight), _p(P.scales),
                              _p(P.zeros), _p(P.row_ptr), _p(P.col_idx), _p(P.out_val), _p(P.mask)),
         "pack")
    return P


def encode(W, mask, bits, ppm=-1, group=GROUP):
    """Everything after the selection, for a given outlier indicator `mask` [N, K]."""
    Wb = _f16_bits(W)
    N, K = Wb.shape
    mask = np.ascontiguousarray(mask, np.uint8)
    nnz = int(mask.sum())
    P = Packed(N, K, bits, ppm,
               np.empty((N, K // GROUP, words_per_group(bits)), np.uint32),
               np.empty((N, K // group), np.uint16), np.empty((N, K // group), np.uint8),
               np.empty(N + 1, np.int32), np.empty(nnz, np.uint16), np.empty(nnz, np.uint16), mask, group)
    _chk(_lib.gwq_oracle_encode(_p(Wb), _p(mask), N, K, bits, group, _p(P.qweight), _p(P.scales), _p(P.zeros),
                                _p(P.row_ptr), _p(P.col_idx), _p(P.out_val)), "encode")
    return P


def decode(P):
    out = np.empty((P.N, P.K), np.float64)
    _chk(_lib.gwq_oracle_decode(P.N, P.K, P.bits, P.group, _p(P.qweight), _p(P.scales), _p(P.zeros),
                                _p(P.row_ptr), _p(P.col_idx), _p(P.out_val), _p(out)), "decode")
    return out


def linear_f64(P, X, rows=None):
    """Y[M, n_rows] in fp64; rows=None gives all N output channels."""
    Xb = _f16_bits(X)
    M, K = Xb.shape
    assert K == P.K
    if rows is None:
        rows_arr, n_rows = None, P.N
    else:
        rows_arr = np.ascontiguousarray(rows, np.int32)
        n_rows = rows_arr.size
    Y = np.empty((M, n_rows), np.float64)
    _chk(_lib.gwq_oracle_linear_f64(P.N, P.K, P.bits, P.group, _p(P.qweight), _p(P.scales), _p(P.zeros),
                                    _p(P.row_ptr), _p(P.col_idx), _p(P.out_val), _p(Xb), M,
                                    _p(rows_arr), n_rows, _p(Y)), "linear_f64")
    return Y


def bf16_bits_to_f64(bits):
    """The values of bfloat16 bit patterns (uint16: the upper half of a binary32) as fp64: an exact widening."""
    return (np.ascontiguousarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def linear_f64_x(P, Xd, rows=None):
    """linear_f64 for activations given as an fp64 array [M, K] (bfloat16 inputs widened by bf16_bits_to_f64)."""
    Xd = np.ascontiguousarray(Xd, np.float64)
    M, K = Xd.shape
    assert K == P.K
    if rows is None:
        rows_arr, n_rows = None, P.N
    else:
        rows_arr = np.ascontiguousarray(rows, np.int32)
        n_rows = rows_arr.size
    Y = np.empty((M, n_rows), np.float64)
    _chk(_lib.gwq_oracle_linear_f64_x(P.N, P.K, P.bits, P.group, _p(P.qweight), _p(P.scales), _p(P.zeros),
                                      _p(P.row_ptr), _p(P.col_idx), _p(P.out_val), _p(Xd), M,
                                      _p(rows_arr), n_rows, _p(Y)), "linear_f64_x")
    return Y


def quality(P, W, score):
    """(sum (W - W_Q)^2, sum score * (W - W_Q), max |W - W_Q|) in fp64 (Sec. 3.1, Eq. 3-5)."""
    Wb = _f16_bits(W)
    score, is16 = _score(score)
    assert Wb.shape == (P.N, P.K) and score.shape == (P.N, P.K)
    out = np.empty(3, np.float64)
    _chk(_lib.gwq_oracle_quality(P.N, P.K, P.bits, P.group, _p(P.qweight), _p(P.scales), _p(P.zeros), _p(P.row_ptr),
                                 _p(P.col_idx), _p(P.out_val), _p(Wb), _p(score), is16, _p(out)), "quality")
    return float(out[0]), float(out[1]), float(out[2])


def gate_up(G, U):
    """silu(G) * U element by element in fp64 (the gated pair of a decoder MLP) for two products of linear_f64."""
    G = np.ascontiguousarray(G, np.float64)
    U = np.ascontiguousarray(U, np.float64)
    assert G.shape == U.shape
    H = np.empty_like(G)
    _chk(_lib.gwq_oracle_gate_up(_p(G), _p(U), G.size, _p(H)), "gate_up")
    return H


def score(dY, X, alpha=1.0, beta=0.0, prev=None):
    """out[n][k] = beta * prev[n][k] + alpha * sum_m dY[m][n] X[m][k] in fp64: the weight gradient of a
    linear layer Y = X W^T from the gradient dY of the loss with respect to Y (Eq. 2, chain rule)."""
    dYb, Xb = _f16_bits(dY), _f16_bits(X)
    M, N = dYb.shape
    K = Xb.shape[1]
    assert Xb.shape[0] == M
    if prev is not None:
        prev = np.ascontiguousarray(prev, np.float32)
        assert prev.shape == (N, K)
    out = np.empty((N, K), np.float64)
    _chk(_lib.gwq_oracle_score(_p(dYb), _p(Xb), M, N, K, ctypes.c_double(alpha), ctypes.c_double(beta),
                               _p(prev) if prev is not None else None, _p(out)), "score")
    return out
