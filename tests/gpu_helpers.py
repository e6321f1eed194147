"""Helpers for the GPU parity tests: host<->device copies of packed layers and error measures."""
import numpy as np

import paper_2411_00850_amd as gwq
from paper_2411_00850_amd.binding import PackedLayer

REL_FRO_TOL = 2e-3      # ||Y_gpu - Y_ref||_F / ||Y_ref||_F
MAX_ABS_TOL = 1e-2      # max|Y_gpu - Y_ref| / max|Y_ref|


def to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def upload_packed(P, pad_byte=0x5A):
    """Oracle-packed host arrays -> device PackedLayer (so gwq_linear is tested on its own).
    The padding that gwq_layout prescribes behind scales, zeros, col_idx and out_val is filled with
    `pad_byte`: the library promises never to interpret it."""
    import torch

    n_out = int(P.row_ptr[-1])
    group = getattr(P, "group", 128)
    sizes = gwq.layout(P.N, P.K, P.bits, group, 0)     # scales / zeros sizes do not depend on ppm

    def dev(a, dt, nbytes=None):
        a = np.ascontiguousarray(a).ravel()
        if nbytes is not None:                       # pad to the size gwq_layout prescribes
            buf = np.full(nbytes // a.itemsize, (pad_byte * 0x0101) & (2 ** (8 * a.itemsize) - 1), a.dtype)
            buf[:a.size] = a
            a = buf
        return torch.from_numpy(a.view(dt)).cuda()

    csr_bytes = (2 * n_out + 15) // 16 * 16 + 16
    D = PackedLayer(P.N, P.K, P.bits, P.ppm, n_out,
                    dev(P.qweight, np.int32).view(P.N, P.K // 128, -1),
                    dev(P.scales, np.int16, sizes["scales"]), dev(P.zeros, np.uint8, sizes["zeros"]),
                    dev(P.row_ptr, np.int32), dev(P.col_idx, np.int16, csr_bytes),
                    dev(P.out_val, np.int16, csr_bytes), None, group)
    return D


def download_packed(D):
    """Device PackedLayer -> dict of numpy arrays with the unsigned dtypes of the format."""
    k = D.n_outliers
    g = D.N * (D.K // D.group)
    return dict(qweight=D.qweight.cpu().numpy().view(np.uint32),
                scales=D.scales.cpu().numpy().view(np.uint16).ravel()[:g],
                zeros=D.zeros.cpu().numpy().ravel()[:g],
                row_ptr=D.row_ptr.cpu().numpy(),
                col_idx=D.col_idx.cpu().numpy().view(np.uint16)[:k],
                out_val=D.out_val.cpu().numpy().view(np.uint16)[:k])


def assert_packed_equal(D, P):
    """Byte-for-byte comparison of a device-packed layer with the oracle's."""
    got = download_packed(D)
    assert D.n_outliers == int(P.row_ptr[-1])
    for name in ("row_ptr", "col_idx", "out_val", "scales", "zeros", "qweight"):
        want = getattr(P, name)
        g = got[name].reshape(want.shape)
        if not np.array_equal(g, want):
            bad = np.flatnonzero(g.ravel() != want.ravel())
            raise AssertionError(f"{name}: {bad.size} of {want.size} entries differ, first at {bad[:5]}: "
                                 f"gpu {g.ravel()[bad[:5]]} oracle {want.ravel()[bad[:5]]}")


def errors(Y_gpu, Y_ref):
    Yg = Y_gpu.astype(np.float64)
    rel = np.linalg.norm(Yg - Y_ref) / max(np.linalg.norm(Y_ref), 1e-300)
    mx = np.abs(Yg - Y_ref).max() / max(np.abs(Y_ref).max(), 1e-300)
    return rel, mx


def assert_close(Y_gpu, Y_ref, what=""):
    assert np.isfinite(Y_gpu.astype(np.float64)).all(), what
    rel, mx = errors(Y_gpu, Y_ref)
    assert rel <= REL_FRO_TOL and mx <= MAX_ABS_TOL, f"{what}: rel_fro={rel:.3e} max_abs/max={mx:.3e}"
    return rel, mx
