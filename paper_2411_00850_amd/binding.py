"""ctypes binding of libgwq.so: the same calls as include/gwq.h, argument marshalling only.

The library is loaded from this directory.  It is built by `__graft_entry__.build()` (or
`python -m paper_2411_00850_amd.build`); if it is missing, it is built here once - but only while this
process has not touched the GPU yet (a compiler run started from a process that holds the GPU, or from
under a profiler's preload, is not safe), otherwise loading raises.  A library older than its sources
is loaded with a warning.  There is no fallback path: without the library every call raises.
"""
import ctypes
import os
from dataclasses import dataclass

HERE = os.path.dirname(os.path.abspath(__file__))
# GWQ_SANITIZE_HOST=1: the checking build of the library (host code under the sanitizers; see build.py), CPU-side tests only
_LIB_PATH = os.path.join(HERE, "libgwq_san.so" if os.environ.get("GWQ_SANITIZE_HOST", "") == "1" else "libgwq.so")

GWQ_OK = 0
SCORE_F32, SCORE_F16 = 0, 1


class GwqError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {lib().gwq_status_string(status).decode()} (status {status})")


class _Packed(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("K", ctypes.c_int32), ("bits", ctypes.c_int32),
                ("group", ctypes.c_int32), ("outlier_ppm", ctypes.c_uint32),
                ("n_outliers", ctypes.c_int64),
                ("qweight", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("zeros", ctypes.c_void_p),
                ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p), ("out_val", ctypes.c_void_p),
                ("index", ctypes.c_void_p)]


class _Sizes(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in ("qweight", "scales", "zeros", "row_ptr", "col_idx",
                                                "out_val", "pack_workspace", "linear_workspace", "linear_index",
                                                "linear_scratch")]
    _fields_.append(("n_outliers", ctypes.c_int64))
    _fields_.append(("quality_workspace", ctypes.c_size_t))


_lib = None


def library_path():
    return _LIB_PATH


def lib():
    """The loaded C library (built on first use if the shared object is not there)."""
    global _lib
    if _lib is None:
        from . import build as _build
        if not os.path.exists(_LIB_PATH):
            import sys
            torch = sys.modules.get("torch")
            if torch is not None and torch.cuda.is_initialized():
                raise RuntimeError("libgwq.so is not built and this process already uses the GPU: run "
                                   "__graft_entry__.build() (or python -m paper_2411_00850_amd.build) first")
            _build.build(sanitize_host=_LIB_PATH.endswith("libgwq_san.so"))
        elif _build.stale():
            import warnings
            warnings.warn("libgwq.so is older than its sources: rebuild with __graft_entry__.build()")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, u32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint32
        L.gwq_layout.restype = ctypes.c_int
        L.gwq_layout.argtypes = [i32, i32, i32, i32, u32, i32, ctypes.POINTER(_Sizes)]
        L.gwq_pack.restype = ctypes.c_int
        L.gwq_pack.argtypes = [vp, vp, ctypes.c_int, ctypes.POINTER(_Packed), vp, ctypes.c_size_t, vp]
        L.gwq_quality.restype = ctypes.c_int
        L.gwq_quality.argtypes = [ctypes.POINTER(_Packed), vp, vp, ctypes.c_int, vp, vp, ctypes.c_size_t, vp]
        L.gwq_score.restype = ctypes.c_int
        L.gwq_score.argtypes = [vp, vp, i32, i32, i32, ctypes.c_float, ctypes.c_float, vp, vp]
        L.gwq_linear.restype = ctypes.c_int
        L.gwq_linear.argtypes = [ctypes.POINTER(_Packed), vp, i32, vp, vp, ctypes.c_size_t, vp]
        L.gwq_linear_bf16.restype = ctypes.c_int
        L.gwq_linear_bf16.argtypes = [ctypes.POINTER(_Packed), vp, i32, vp, vp, ctypes.c_size_t, vp]
        L.gwq_linear_index.restype = ctypes.c_int
        L.gwq_linear_index.argtypes = [ctypes.POINTER(_Packed), vp, ctypes.c_size_t, vp]
        L.gwq_linear_indexed.restype = ctypes.c_int
        L.gwq_linear_indexed.argtypes = [ctypes.POINTER(_Packed), vp, i32, vp, vp, ctypes.c_size_t, vp,
                                         ctypes.c_size_t, vp]
        L.gwq_linear_static.restype = ctypes.c_int
        L.gwq_linear_static.argtypes = [ctypes.POINTER(_Packed), vp, i32, vp, vp]
        L.gwq_linear_batch.restype = ctypes.c_int
        L.gwq_linear_batch.argtypes = [i32, ctypes.POINTER(ctypes.POINTER(_Packed)), ctypes.POINTER(vp), i32,
                                       ctypes.POINTER(vp), vp]
        L.gwq_linear_gate_up.restype = ctypes.c_int
        L.gwq_linear_gate_up.argtypes = [ctypes.POINTER(_Packed), ctypes.POINTER(_Packed), vp, i32, vp, vp, ctypes.c_size_t, vp]
        L.gwq_linear_plan.restype = ctypes.c_int
        L.gwq_linear_plan.argtypes = [i32, ctypes.POINTER(ctypes.POINTER(_Packed)), i32, i32, ctypes.c_char_p, ctypes.c_size_t]
        L.gwq_probe_stream.restype = ctypes.c_int
        L.gwq_probe_stream.argtypes = [vp, ctypes.c_size_t, vp, vp]
        L.gwq_probe_mfma.restype = ctypes.c_int
        L.gwq_probe_mfma.argtypes = [i32, i32, vp, vp]
        L.gwq_tuning_set.restype = ctypes.c_int
        L.gwq_tuning_set.argtypes = [ctypes.c_char_p, i32]
        L.gwq_status_string.restype = ctypes.c_char_p
        L.gwq_status_string.argtypes = [ctypes.c_int]
        L.gwq_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def version():
    return lib().gwq_version().decode()


def layout(N, K, bits, group=128, ppm=10000, M_max=0):
    """Buffer sizes in bytes for one layer, as a dict (pure host call)."""
    s = _Sizes()
    rc = lib().gwq_layout(N, K, bits, group, ppm, M_max, ctypes.byref(s))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_layout")
    return {n: getattr(s, n) for n, _ in _Sizes._fields_}


def tuning_set(key, value):
    rc = lib().gwq_tuning_set(key.encode(), int(value))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_tuning_set")


def prepare_linear_gate_up(Pg, Pu, X, out):
    """Pre-marshalled gwq_linear_gate_up call: out = silu(X Wg^T) * (X Wu^T) (FP16 [M, N]); returns a zero-argument
    callable that enqueues it on the current torch stream.  The workspace (needed beyond M = 4) is allocated here."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and X.shape[1] == Pg.K == Pu.K
    M = X.shape[0]
    assert out.is_cuda and out.dtype == torch.float16 and out.is_contiguous() and tuple(out.shape) == (M, Pg.N) and Pg.N == Pu.N
    ws = torch.empty(4 * M * Pg.N, dtype=torch.uint8, device=X.device) if (M > 4 or Pg.K > 16384 or Pg.group != 128) else None
    cg, cu = Pg.c_struct(), Pu.c_struct()
    rg, ru = ctypes.byref(cg), ctypes.byref(cu)
    xp, hp = ctypes.c_void_p(X.data_ptr()), ctypes.c_void_p(out.data_ptr())
    wp, wl = (ctypes.c_void_p(ws.data_ptr()), ws.numel()) if ws is not None else (None, 0)
    fn = lib().gwq_linear_gate_up
    current_stream = torch.cuda.current_stream

    def call(_keep=(cg, cu, Pg, Pu, X, out, ws)):
        rc = fn(rg, ru, xp, M, hp, wp, wl, ctypes.c_void_p(current_stream().cuda_stream))
        if rc != GWQ_OK:
            raise GwqError(rc, "gwq_linear_gate_up")
    return call


def linear_gate_up(Pg, Pu, X, out=None):
    """gwq_linear_gate_up: silu(X Wg^T) * (X Wu^T) as FP16 [M, N]."""
    import torch
    if out is None:
        out = torch.empty((X.shape[0], Pg.N), dtype=torch.float16, device=X.device)
    prepare_linear_gate_up(Pg, Pu, X, out)()
    return out


def linear_plan(layers, M, with_scratch=True):
    """gwq_linear_plan: the kernel (name, template arguments, launch shape) that gwq_linear / gwq_linear_batch
    would launch for these layers (one PackedLayer or a list of layers of one K) and M, as text."""
    if not isinstance(layers, (list, tuple)):
        layers = [layers]
    structs = [P.c_struct() for P in layers]
    parr = (ctypes.POINTER(_Packed) * len(structs))(*[ctypes.pointer(c) for c in structs])
    buf = ctypes.create_string_buffer(256)
    rc = lib().gwq_linear_plan(len(structs), parr, int(M), int(bool(with_scratch)), buf, 256)
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_linear_plan")
    return buf.value.decode()


def probe_stream(src, sink, stream=None):
    """gwq_probe_stream over the bytes of the tensor `src` (a multiple of 16)."""
    rc = lib().gwq_probe_stream(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream_ptr(stream))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_probe_stream")


def probe_mfma(blocks, iters, sink, stream=None):
    """gwq_probe_mfma; returns the floating-point operations the launch performs."""
    rc = lib().gwq_probe_mfma(int(blocks), int(iters), sink.data_ptr(), _stream_ptr(stream))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_probe_mfma")
    return 2.0 * 32 * 32 * 16 * 8 * iters * 4 * blocks


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


@dataclass
class PackedLayer:
    """Device buffers of one packed layer (torch tensors own the memory)."""
    N: int
    K: int
    bits: int
    ppm: int
    n_outliers: int
    qweight: "torch.Tensor"   # int32 view of the uint32 words [N, K/128, wpg]
    scales: "torch.Tensor"    # int16 view of the FP16 bits [N * K/group], padded to 16 bytes
    zeros: "torch.Tensor"     # uint8 [N * K/group], padded to 16 bytes
    row_ptr: "torch.Tensor"   # int32 [N+1]
    col_idx: "torch.Tensor"   # int16 view of uint16 [n_outliers + padding]
    out_val: "torch.Tensor"   # int16 view of FP16 bits [n_outliers + padding]
    index: "torch.Tensor" = None   # optional uint8 [linear_index bytes]: filled by gwq_pack, read by gwq_linear for M > 16
    group: int = 128               # weights per scale and zero point: 16, 32, 64 or 128 (scales, zeros: [N * K/group])

    def c_struct(self):
        return _Packed(self.N, self.K, self.bits, self.group, self.ppm, self.n_outliers,
                       self.qweight.data_ptr(), self.scales.data_ptr(), self.zeros.data_ptr(),
                       self.row_ptr.data_ptr(), self.col_idx.data_ptr(), self.out_val.data_ptr(),
                       self.index.data_ptr() if self.index is not None else None)

    def nbytes(self):
        return sum(t.numel() * t.element_size() for t in
                   (self.qweight, self.scales, self.zeros, self.row_ptr, self.col_idx, self.out_val))


def alloc_packed(N, K, bits, ppm=10000, device="cuda", with_index=True, group=128):
    import torch
    sz = layout(N, K, bits, group, ppm)
    gpr = K // 128
    wpg = 16 if bits == 4 else 13
    n_slots = sz["col_idx"] // 2
    return PackedLayer(N, K, bits, ppm, sz["n_outliers"],
                       torch.empty((N, gpr, wpg), dtype=torch.int32, device=device),
                       torch.empty(sz["scales"] // 2, dtype=torch.int16, device=device),
                       torch.empty(sz["zeros"], dtype=torch.uint8, device=device),
                       torch.empty(N + 1, dtype=torch.int32, device=device),
                       torch.empty(n_slots, dtype=torch.int16, device=device),
                       torch.empty(n_slots, dtype=torch.int16, device=device),
                       torch.empty(sz["linear_index"], dtype=torch.uint8, device=device) if with_index else None,
                       group), sz


def pack(W, score, bits, ppm=10000, stream=None, workspace=None, with_index=True, group=128):
    """gwq_pack: W FP16 [N, K] and score FP32/FP16 [N, K] on the GPU -> PackedLayer.  with_index: also fill the
    layer's index (8 bytes per group, +12 % memory), which gwq_linear then reads for M > 16 instead of building one
    on every call."""
    import torch
    assert W.is_cuda and score.is_cuda and W.dtype == torch.float16 and W.is_contiguous()
    assert score.shape == W.shape and score.is_contiguous()
    if score.dtype == torch.float32:
        st = SCORE_F32
    elif score.dtype == torch.float16:
        st = SCORE_F16
    else:
        raise TypeError("score must be float32 or float16")
    N, K = W.shape
    P, sz = alloc_packed(N, K, bits, ppm, W.device, with_index, group)
    if workspace is None:
        workspace = torch.empty(sz["pack_workspace"], dtype=torch.uint8, device=W.device)
    cs = P.c_struct()
    rc = lib().gwq_pack(W.data_ptr(), score.data_ptr(), st, ctypes.byref(cs), workspace.data_ptr(),
                        workspace.numel(), _stream_ptr(stream))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_pack")
    return P


def quality(P, W, score, out=None, stream=None, workspace=None):
    """gwq_quality: float64 tensor [sum (W - W_Q)^2, sum score * (W - W_Q), max |W - W_Q|] on the GPU for the
    packed layer P against the weights W (FP16 [N, K]) and scores (FP32/FP16 [N, K]) it was packed from."""
    import torch
    assert W.is_cuda and score.is_cuda and W.dtype == torch.float16 and W.is_contiguous()
    assert tuple(W.shape) == (P.N, P.K) and score.shape == W.shape and score.is_contiguous()
    if score.dtype == torch.float32:
        st = SCORE_F32
    elif score.dtype == torch.float16:
        st = SCORE_F16
    else:
        raise TypeError("score must be float32 or float16")
    if out is None:
        out = torch.empty(3, dtype=torch.float64, device=W.device)
    if workspace is None:
        nbytes = layout(P.N, P.K, P.bits, P.group, P.ppm, 0)["quality_workspace"]
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    cs = P.c_struct()
    rc = lib().gwq_quality(ctypes.byref(cs), W.data_ptr(), score.data_ptr(), st, out.data_ptr(), workspace.data_ptr(),
                           workspace.numel(), _stream_ptr(stream))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_quality")
    return out


def score(dY, X, out=None, alpha=1.0, beta=0.0, stream=None):
    """gwq_score: out = beta * out + alpha * dY^T X, the weight gradient of a linear layer Y = X W^T from the gradient
    dY (FP16 [M, N]) of the loss with respect to Y and the layer's input X (FP16 [M, K]); out is FP32 [N, K]."""
    import torch
    assert dY.is_cuda and X.is_cuda and dY.dtype == torch.float16 and X.dtype == torch.float16
    assert dY.is_contiguous() and X.is_contiguous() and dY.dim() == 2 and X.dim() == 2 and dY.shape[0] == X.shape[0]
    M, N = dY.shape
    K = X.shape[1]
    if out is None:
        assert beta == 0.0, "beta != 0 accumulates into `out`"
        out = torch.empty((N, K), dtype=torch.float32, device=X.device)
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == (N, K)
    rc = lib().gwq_score(dY.data_ptr(), X.data_ptr(), M, N, K, alpha, beta, out.data_ptr(), _stream_ptr(stream))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_score")
    return out


def linear_workspace(P, M, device="cuda"):
    """Scratch tensor gwq_linear needs for this layer at M rows (None for the decode path)."""
    import torch
    nbytes = layout(P.N, P.K, P.bits, P.group, P.ppm, M)["linear_workspace"]
    return torch.empty(nbytes, dtype=torch.uint8, device=device) if nbytes else None


def linear_scratch(P, M, device="cuda"):
    """Scratch tensor gwq_linear_indexed may use for this layer at M rows (None for the decode path)."""
    import torch
    nbytes = layout(P.N, P.K, P.bits, P.group, P.ppm, M)["linear_scratch"]
    return torch.empty(nbytes, dtype=torch.uint8, device=device) if nbytes else None


def linear_index(P, stream=None):
    """gwq_linear_index: the per-layer index gwq_linear_indexed reads for M > 16 (a uint8 tensor).  Build it
    once per packed layer; it stays valid until the layer's buffers change."""
    import torch
    nbytes = layout(P.N, P.K, P.bits, P.group, P.ppm, 0)["linear_index"]
    index = torch.empty(nbytes, dtype=torch.uint8, device=P.qweight.device)
    cs = P.c_struct()
    rc = lib().gwq_linear_index(ctypes.byref(cs), index.data_ptr(), index.numel(), _stream_ptr(stream))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_linear_index")
    return index


def linear(P, X, out=None, stream=None, workspace=None, index=None, scratch="auto"):
    """gwq_linear: X FP16 [M, K] on the GPU -> Y FP16 [M, N].  With `index` (from linear_index) the call
    is gwq_linear_indexed; its scratch is allocated here unless one (or None) is passed."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and X.shape[1] == P.K
    M = X.shape[0]
    if out is None:
        out = torch.empty((M, P.N), dtype=torch.float16, device=X.device)
    if index is not None:
        cs = P.c_struct()
        if isinstance(scratch, str):
            scratch = linear_scratch(P, M, X.device)
        rc = lib().gwq_linear_indexed(ctypes.byref(cs), X.data_ptr(), M, out.data_ptr(), index.data_ptr(),
                                      index.numel(), scratch.data_ptr() if scratch is not None else None,
                                      scratch.numel() if scratch is not None else 0, _stream_ptr(stream))
        if rc != GWQ_OK:
            raise GwqError(rc, "gwq_linear_indexed")
        return out
    if workspace is None:
        workspace = linear_workspace(P, M, X.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() if workspace is not None else 0
    cs = P.c_struct()
    rc = lib().gwq_linear(ctypes.byref(cs), X.data_ptr(), M, out.data_ptr(), ws_ptr, ws_len, _stream_ptr(stream))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_linear")
    return out


def linear_bf16(P, X, out=None, stream=None, workspace=None):
    """gwq_linear_bf16: X bfloat16 [M, K] on the GPU -> Y bfloat16 [M, N] (layers with groups of 128)."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous() and X.shape[1] == P.K
    M = X.shape[0]
    if out is None:
        out = torch.empty((M, P.N), dtype=torch.bfloat16, device=X.device)
    assert out.is_cuda and out.dtype == torch.bfloat16 and out.is_contiguous() and tuple(out.shape) == (M, P.N)
    if workspace is None:
        workspace = linear_workspace(P, M, X.device)
    cs = P.c_struct()
    rc = lib().gwq_linear_bf16(ctypes.byref(cs), X.data_ptr(), M, out.data_ptr(),
                               workspace.data_ptr() if workspace is not None else None,
                               workspace.numel() if workspace is not None else 0, _stream_ptr(stream))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_linear_bf16")
    return out


STATIC_SCRATCH_BYTES = 48 << 20


def linear_static(P, X, out, stream=None):
    """gwq_linear_static: gwq_linear with the library's own static scratch instead of a workspace; the call
    allocates nothing, so `out` (FP16 [M, N]) is the caller's."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and X.shape[1] == P.K
    assert out.is_cuda and out.dtype == torch.float16 and out.is_contiguous() and tuple(out.shape) == (X.shape[0], P.N)
    cs = P.c_struct()
    rc = lib().gwq_linear_static(ctypes.byref(cs), X.data_ptr(), X.shape[0], out.data_ptr(), _stream_ptr(stream))
    if rc != GWQ_OK:
        raise GwqError(rc, "gwq_linear_static")
    return out


def prepare_linear(P, X, out, index=None):
    """Pre-marshalled gwq_linear call for launch-bound loops: returns a zero-argument callable that
    enqueues the same call on whatever torch stream is current when it is invoked (so it can be
    captured into a HIP graph).  P, X and out must stay alive while the callable is used.  With
    `index` (from linear_index) the call is gwq_linear_indexed."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and X.shape[1] == P.K
    assert out.shape == (X.shape[0], P.N) and out.dtype == torch.float16 and out.is_contiguous()
    cs = P.c_struct()
    ref = ctypes.byref(cs)
    xp, yp, M = ctypes.c_void_p(X.data_ptr()), ctypes.c_void_p(out.data_ptr()), X.shape[0]
    current_stream = torch.cuda.current_stream

    def ptr_len(t):
        return (ctypes.c_void_p(t.data_ptr()), t.numel()) if t is not None else (None, 0)

    if index is None:
        fn = lib().gwq_linear
        ws = linear_workspace(P, M, X.device)
        wp, wl = ptr_len(ws)

        def call(_keep=(cs, P, X, out, ws)):
            rc = fn(ref, xp, M, yp, wp, wl, ctypes.c_void_p(current_stream().cuda_stream))
            if rc != GWQ_OK:
                raise GwqError(rc, "gwq_linear")
        return call
    fn = lib().gwq_linear_indexed
    sc = linear_scratch(P, M, X.device)
    (ip, il), (sp, sl) = ptr_len(index), ptr_len(sc)

    def call_indexed(_keep=(cs, P, X, out, index, sc)):
        rc = fn(ref, xp, M, yp, ip, il, sp, sl, ctypes.c_void_p(current_stream().cuda_stream))
        if rc != GWQ_OK:
            raise GwqError(rc, "gwq_linear_indexed")
    return call_indexed


def prepare_linear_batch(layers, Xs, outs):
    """Pre-marshalled gwq_linear_batch call (one decode launch over several layers, M <= 16): returns a
    zero-argument callable that enqueues it on the current torch stream.  `layers`, `Xs`, `outs` are
    equally long sequences; entries of Xs may repeat (shared activations)."""
    import torch
    n = len(layers)
    assert n == len(Xs) == len(outs) and 1 <= n
    M = Xs[0].shape[0]
    for P, X, Y in zip(layers, Xs, outs):
        assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and X.shape == (M, P.K)
        assert Y.shape == (M, P.N) and Y.dtype == torch.float16 and Y.is_contiguous()
    structs = [P.c_struct() for P in layers]
    parr = (ctypes.POINTER(_Packed) * n)(*[ctypes.pointer(c) for c in structs])
    xarr = (ctypes.c_void_p * n)(*[X.data_ptr() for X in Xs])
    yarr = (ctypes.c_void_p * n)(*[Y.data_ptr() for Y in outs])
    fn = lib().gwq_linear_batch
    current_stream = torch.cuda.current_stream

    def call(_keep=(structs, layers, Xs, outs)):
        rc = fn(n, parr, xarr, M, yarr, ctypes.c_void_p(current_stream().cuda_stream))
        if rc != GWQ_OK:
            raise GwqError(rc, "gwq_linear_batch")
    return call


def linear_batch(layers, Xs, outs=None):
    """gwq_linear_batch: returns the list of outputs."""
    import torch
    if outs is None:
        outs = [torch.empty((X.shape[0], P.N), dtype=torch.float16, device=X.device) for P, X in zip(layers, Xs)]
    prepare_linear_batch(layers, Xs, outs)()
    return outs
