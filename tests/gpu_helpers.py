"""Helpers for the GPU parity tests: host<->device copies of packed layers and error measures."""
import numpy as np

import paper_2411_00850_amd as gwq
from paper_2411_00850_amd.binding import PackedLayer

REL_FRO_TOL = 2e-3      # ||Y_gpu - Y_ref||_F / ||Y_ref||_F
MAX_ABS_TOL = 1e-2      # max|Y_gpu - Y_ref| / max|Y_ref|


def to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def upload_packed(P):
    """Oracle-packed host arrays -> device PackedLayer (so gwq_linear is tested on its own)."""
    import torch

    def dev(a, dt):
        a = np.ascontiguousarray(a)
        if a.size == 0:
            a = np.zeros(8, a.dtype)
        return torch.from_numpy(a.view(dt)).cuda()

    return PackedLayer(P.N, P.K, P.bits, P.ppm, int(P.row_ptr[-1]),
                       dev(P.qweight, np.int32), dev(P.scales, np.int16), dev(P.zeros, np.uint8),
                       dev(P.row_ptr, np.int32), dev(P.col_idx, np.int16), dev(P.out_val, np.int16))


def download_packed(D):
    """Device PackedLayer -> dict of numpy arrays with the unsigned dtypes of the format."""
    k = D.n_outliers
    return dict(qweight=D.qweight.cpu().numpy().view(np.uint32),
                scales=D.scales.cpu().numpy().view(np.uint16),
                zeros=D.zeros.cpu().numpy(),
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
