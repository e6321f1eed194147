"""C-ABI checks that need no GPU: exported symbols, layout arithmetic, argument validation."""
import ctypes
import os
import re

import pytest

import paper_2411_00850_amd as gwq
from paper_2411_00850_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gwq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gwq_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_calls():
    assert declared_functions() == ["gwq_layout", "gwq_linear", "gwq_linear_batch", "gwq_linear_bf16", "gwq_linear_gate_up",
                                    "gwq_linear_index", "gwq_linear_indexed", "gwq_linear_plan", "gwq_linear_static", "gwq_pack",
                                    "gwq_probe_mfma", "gwq_probe_stream", "gwq_quality", "gwq_score",
                                    "gwq_status_string", "gwq_tuning_set", "gwq_version"]


@pytest.mark.parametrize("name", declared_functions())
def test_library_exports_every_declared_symbol(name):
    lib = ctypes.CDLL(gwq.library_path())
    assert hasattr(lib, name)


def test_layout_sizes_7b_shapes():
    s = gwq.layout(4096, 4096, 4)
    assert s["qweight"] == 4096 * 32 * 16 * 4 and s["scales"] == 4096 * 32 * 2 + 16 and s["zeros"] == 4096 * 32 + 16
    assert s["row_ptr"] == 4097 * 4 and s["n_outliers"] == 167773
    assert s["col_idx"] == s["out_val"] == (167773 * 2 + 15) // 16 * 16 + 16     # whole vectors + one spare
    s3 = gwq.layout(11008, 4096, 3)
    assert s3["qweight"] == 11008 * 32 * 13 * 4 and s3["n_outliers"] == 450888
    # bytes per weight of the packed layer: 4.5 bits and 3.77 bits
    total = sum(s[k] for k in ("qweight", "scales", "zeros", "row_ptr", "col_idx", "out_val"))
    assert abs(total / 4096 ** 2 - 0.5644) < 1e-3
    assert gwq.layout(8, 128, 4, ppm=0)["col_idx"] == 16          # never a zero-size buffer
    assert s["linear_workspace"] == 0 and gwq.layout(4096, 4096, 4)["linear_index"] == 4096 * 33 * 8     # one 8-byte record per channel and group, plus one
    big = gwq.layout(4096, 4096, 4, M_max=2048)
    assert big["linear_scratch"] == 256 * 256 * 128 * 4 and big["linear_workspace"] == big["linear_index"] + big["linear_scratch"]
    assert gwq.layout(4096, 4096, 4, M_max=64)["linear_scratch"] == 8 * 64 * 4096 * 4      # eight FP32 copies of Y at most
    small = gwq.layout(3, 128, 4)                                  # 3 groups: padded to one vector
    assert small["scales"] == 32 and small["zeros"] == 32


@pytest.mark.parametrize("args, status", [
    ((0, 128, 4, 128, 10000, 1), -2), ((4, 100, 4, 128, 10000, 1), -2), ((4, 0, 4, 128, 10000, 1), -2),
    ((4, 65536 + 128, 4, 128, 10000, 1), -2), ((70000, 65536, 4, 128, 10000, 1), -2),
    ((4, 128, 5, 128, 10000, 1), -3), ((4, 128, 2, 128, 10000, 1), -3), ((4, 128, 4, 48, 10000, 1), -3),
    ((4, 128, 4, 8, 10000, 1), -3), ((4, 128, 4, 256, 10000, 1), -3), ((4, 128, 4, 0, 10000, 1), -3),
    ((4, 65536, 4, 16, 10000, 1), -2), ((4, 32768 + 128, 4, 16, 10000, 1), -2),        # more than 2048 groups per channel
    ((4, 128, 4, 128, 1000001, 1), -2), ((4, 128, 4, 128, 10000, -1), -2),
])
def test_layout_rejects_bad_arguments(args, status):
    s = binding._Sizes()
    assert binding.lib().gwq_layout(*args, ctypes.byref(s)) == status


def test_layout_sizes_of_small_groups():
    """Group sizes 16, 32 and 64 (Sec. 3.2 sets 16): the code words do not change, scales and zero points
    are one per group, and the index for M > 16 grows by one 4-byte pair per 16 columns."""
    base = gwq.layout(4096, 4096, 4)
    for group in (16, 32, 64):
        s = gwq.layout(4096, 4096, 4, group)
        per_row = 4096 // group
        assert s["qweight"] == base["qweight"] and s["col_idx"] == base["col_idx"] and s["n_outliers"] == base["n_outliers"]
        assert s["scales"] == 4096 * per_row * 2 + 16 and s["zeros"] == 4096 * per_row + 16
        assert s["linear_index"] == base["linear_index"] + 4096 * (4096 // 16) * 4
    assert gwq.layout(4, 32768, 3, 16)["scales"] == 4 * 2048 * 2 + 16          # the most groups per channel
    assert gwq.layout(4, 65536, 3, 32)["zeros"] == 4 * 2048 + 16


def test_layout_null_out():
    assert binding.lib().gwq_layout(4, 128, 4, 128, 10000, 1, None) == -1


def _packed(N=4, K=128, bits=4, ppm=10000, fake=0x1000, **kw):
    n_out = (ppm * N * K + 999999) // 1000000
    p = binding._Packed(N, K, bits, 128, ppm, n_out, fake, fake, fake, fake, fake, fake)
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_pack_and_linear_validate_before_touching_the_device():
    """All of these return an error code on a machine with no GPU: nothing is launched."""
    L = binding.lib()
    fake = ctypes.c_void_p(0x1000)
    ok = _packed()
    assert ok.index is None                              # the optional index defaults to NULL
    assert L.gwq_pack(fake, fake, 0, ctypes.byref(_packed(index=0x1008)), fake, 1 << 20, None) == -2   # present: 16-byte aligned
    assert L.gwq_linear(ctypes.byref(_packed(index=0x1004)), fake, 1, fake, None, 0, None) == -2
    assert L.gwq_pack(None, fake, 0, ctypes.byref(ok), fake, 1 << 20, None) == -1
    assert L.gwq_pack(fake, None, 0, ctypes.byref(ok), fake, 1 << 20, None) == -1
    assert L.gwq_pack(fake, fake, 0, None, fake, 1 << 20, None) == -1
    assert L.gwq_pack(fake, fake, 7, ctypes.byref(ok), fake, 1 << 20, None) == -3
    assert L.gwq_pack(fake, fake, 0, ctypes.byref(ok), None, 1 << 20, None) == -4
    assert L.gwq_pack(fake, fake, 0, ctypes.byref(ok), fake, 16, None) == -4
    assert L.gwq_pack(fake, fake, 0, ctypes.byref(_packed(bits=5)), fake, 1 << 20, None) == -3
    assert L.gwq_pack(fake, fake, 0, ctypes.byref(_packed(K=100)), fake, 1 << 20, None) == -2
    assert L.gwq_pack(fake, fake, 0, ctypes.byref(_packed(n_outliers=3)), fake, 1 << 20, None) == -2
    assert L.gwq_pack(fake, fake, 0, ctypes.byref(_packed(zeros=None)), fake, 1 << 20, None) == -1
    assert L.gwq_linear(None, fake, 1, fake, None, 0, None) == -1
    assert L.gwq_linear(ctypes.byref(ok), None, 1, fake, None, 0, None) == -1
    assert L.gwq_linear(ctypes.byref(ok), fake, 1, None, None, 0, None) == -1
    assert L.gwq_linear(ctypes.byref(ok), fake, 0, fake, None, 0, None) == -2
    assert L.gwq_linear(ctypes.byref(_packed(group=48)), fake, 1, fake, None, 0, None) == -3
    assert L.gwq_linear(ctypes.byref(ok), ctypes.c_void_p(0x1002), 1, fake, None, 0, None) == -2
    assert L.gwq_linear(ctypes.byref(ok), fake, 17, fake, None, 0, None) == -4       # M > 16 needs scratch
    assert L.gwq_linear_bf16(None, fake, 1, fake, None, 0, None) == -1
    assert L.gwq_linear_bf16(ctypes.byref(ok), None, 1, fake, None, 0, None) == -1
    assert L.gwq_linear_bf16(ctypes.byref(ok), fake, 0, fake, None, 0, None) == -2
    assert L.gwq_linear_bf16(ctypes.byref(ok), ctypes.c_void_p(0x1002), 1, fake, None, 0, None) == -2
    assert L.gwq_linear_bf16(ctypes.byref(ok), fake, 17, fake, None, 0, None) == -4
    assert L.gwq_linear_bf16(ctypes.byref(_packed(group=32)), fake, 1, fake, None, 0, None) == -3   # groups of 128 only
    assert L.gwq_linear(ctypes.byref(ok), fake, 17, fake, fake, 8, None) == -4


def test_linear_index_validates_before_touching_the_device():
    L = binding.lib()
    fake = ctypes.c_void_p(0x1000)
    ok = _packed()
    need = gwq.layout(4, 128, 4, M_max=17)["linear_index"]
    assert need == 256                                                          # 4 * 2 records of 8 bytes, in 256-byte units
    assert L.gwq_linear_index(None, fake, need, None) == -1
    assert L.gwq_linear_index(ctypes.byref(ok), None, need, None) == -4
    assert L.gwq_linear_index(ctypes.byref(ok), fake, need - 1, None) == -4
    assert L.gwq_linear_index(ctypes.byref(ok), ctypes.c_void_p(0x1008), need, None) == -2
    assert L.gwq_linear_index(ctypes.byref(_packed(bits=5)), fake, need, None) == -3
    assert L.gwq_linear_indexed(None, fake, 17, fake, fake, need, None, 0, None) == -1
    assert L.gwq_linear_indexed(ctypes.byref(ok), None, 17, fake, fake, need, None, 0, None) == -1
    assert L.gwq_linear_indexed(ctypes.byref(ok), fake, 0, fake, fake, need, None, 0, None) == -2
    assert L.gwq_linear_indexed(ctypes.byref(ok), fake, 17, fake, None, 0, None, 0, None) == -4      # M > 16 needs the index
    assert L.gwq_linear_indexed(ctypes.byref(ok), fake, 17, fake, fake, need - 1, None, 0, None) == -4
    assert L.gwq_linear_indexed(ctypes.byref(ok), fake, 17, fake, ctypes.c_void_p(0x1004), need, None, 0, None) == -2
    assert L.gwq_linear_indexed(ctypes.byref(ok), fake, 17, fake, fake, need, ctypes.c_void_p(0x1004), 64, None) == -2


def test_linear_static_validates_before_touching_the_device():
    L = binding.lib()
    fake = ctypes.c_void_p(0x1000)
    ok = _packed()
    assert L.gwq_linear_static(None, fake, 17, fake, None) == -1
    assert L.gwq_linear_static(ctypes.byref(ok), None, 17, fake, None) == -1
    assert L.gwq_linear_static(ctypes.byref(ok), fake, 17, None, None) == -1
    assert L.gwq_linear_static(ctypes.byref(ok), fake, 0, fake, None) == -2
    assert L.gwq_linear_static(ctypes.byref(ok), ctypes.c_void_p(0x1002), 17, fake, None) == -2
    assert L.gwq_linear_static(ctypes.byref(_packed(bits=5)), fake, 17, fake, None) == -3
    # index + partial sums beyond the static array: refused, nothing launched
    big = _packed(N=60000, K=65536)
    assert L.gwq_linear_static(ctypes.byref(big), fake, 2048, fake, None) == -4
    assert gwq.STATIC_SCRATCH_BYTES == 48 << 20


def test_linear_plan_names_the_kernel_without_a_device():
    """gwq_linear_plan is pure host arithmetic: it names the kernel the dispatcher picks for a shape and M."""
    L = binding.lib()
    buf = ctypes.create_string_buffer(256)

    def plan(layers, M, scratch=1):
        arr = (ctypes.POINTER(binding._Packed) * len(layers))(*[ctypes.pointer(p) for p in layers])
        assert L.gwq_linear_plan(len(layers), arr, M, scratch, buf, 256) == 0
        return buf.value.decode()

    q = _packed(N=4096, K=4096)
    gate = _packed(N=11008, K=4096)
    down = _packed(N=4096, K=11008)
    assert plan([q], 1).startswith("decode_small_kernel<4,8,1> grid 256x1 block 256")
    assert plan([q, q, q], 1).startswith("decode_small_kernel<4,8,1> grid 256x3")
    assert plan([down], 1).startswith("decode_small_kernel<4,8,1> grid 256x1 block 704")
    assert plan([gate, gate], 16).startswith("decode_stream_kernel<4,16>")          # several tiles per block
    assert plan([q], 16).startswith("decode_wide_kernel<4,4,16,false,false,1>")                # one tile per block
    assert plan([_packed(N=4096, K=4096, bits=3)], 8).startswith("decode_small_kernel<3,8,8> grid 256x1 block 256 lds 78000")   # two blocks per CU
    assert plan([_packed(N=4096, K=4096, bits=3)], 9).startswith("decode_wide_kernel<3,")
    assert plan([down], 8).startswith("decode_wide_kernel<4,4,8,false,false,2>")    # several phases at M <= 8: two copies of X
    assert plan([gate, gate], 8).startswith("decode_small_kernel<4,8,8,false,false,true> grid 344x2 block 512 lds 81120")   # two tiles per block
    assert plan([q, q, q], 8).startswith("decode_small_kernel<4,8,8> grid 256x3")              # fewer than four tiles per CU: one
    assert plan([q], 2048).startswith("gemm_kernel<4,2,2,4,false,false> tile 256x128 grid 256 ")
    q16 = _packed(N=4096, K=4096, group=16)               # groups of 16: the wide decode kernel and the GEMM in their small-group forms
    assert plan([q16], 1).startswith("decode_small_kernel<4,8,1,true>") and plan([q16], 2048).startswith("gemm_kernel<4,2,2,4,true,false>")
    assert plan([q16], 16).startswith("decode_wide_kernel<4,4,16,true,false,1>")
    assert "k_splits 1" in plan([q], 64, scratch=0) and "k_splits 1" not in plan([q], 64, scratch=1)
    arr = (ctypes.POINTER(binding._Packed) * 2)(ctypes.pointer(q), ctypes.pointer(down))
    assert L.gwq_linear_plan(2, arr, 1, 1, buf, 256) == -2                          # one K per launch
    assert L.gwq_linear_plan(1, arr, 1, 1, None, 256) == -1
    assert L.gwq_probe_stream(None, 1024, ctypes.c_void_p(0x1000), None) == -1
    assert L.gwq_probe_stream(ctypes.c_void_p(0x1000), 1000, ctypes.c_void_p(0x1000), None) == -2
    assert L.gwq_probe_mfma(0, 10, ctypes.c_void_p(0x1000), None) == -2


def test_launch_plans_stay_within_the_machine():
    """Every launch the dispatcher plans - seeded sweep over shapes, M, bit widths, group sizes, layers per launch and
    the tuning keys - names a kernel and stays within what a gfx950 CU takes: at most 160 KB of LDS and 1024
    threads per block (512 for the kernels built for that), a grid of at least one block and at most the layers asked
    for along y.  Host arithmetic only: this is the check that a shape the library accepts has a launch that fits."""
    import numpy as np
    L = binding.lib()
    buf = ctypes.create_string_buffer(256)
    rng = np.random.default_rng(2024)
    keys = ["decode_waves", "decode_stream", "decode_tiles", "decode_lean_rows", "decode_pairs", "gemm_rows"]
    seen = set()
    try:
        for case in range(1500):
            bits = int(rng.choice([3, 4]))
            group = int(rng.choice([16, 32, 64, 128, 128]))
            K = 128 * int(rng.choice([1, 2, 3, 5, 8, 16, 31, 32, 33, 64, 86, 128, 224, 256, 511, 512]))
            if K // group > 2048:
                group = 128
            count = int(rng.choice([1, 1, 1, 2, 3, 8]))
            Ns = [int(rng.choice([1, 15, 16, 17, 100, 1000, 4096, 11008, 28672, 50000])) for _ in range(count)]
            M = int(rng.choice([1, 2, 4, 5, 8, 9, 16, 17, 33, 64, 200, 2048])) if count == 1 else int(rng.integers(1, 17))
            for k in keys:
                L.gwq_tuning_set(k.encode(), 0)
            if case % 3 == 1:
                L.gwq_tuning_set(b"decode_waves", int(rng.choice([1, 2, 3, 6, 12, 16])))
                L.gwq_tuning_set(b"decode_stream", int(rng.choice([0, 1, 2])))
                L.gwq_tuning_set(b"decode_tiles", int(rng.choice([0, 1, 3, 7])))
                L.gwq_tuning_set(b"decode_lean_rows", int(rng.choice([0, 1, 4, 8])))
                L.gwq_tuning_set(b"decode_pairs", int(rng.choice([0, 1, 2])))
            if case % 3 == 2:
                L.gwq_tuning_set(b"gemm_rows", int(rng.choice([0, 32, 64, 128, 256])))
            layers = [_packed(N=n, K=K, bits=bits, group=group) for n in Ns]
            arr = (ctypes.POINTER(binding._Packed) * count)(*[ctypes.pointer(p) for p in layers])
            what = f"bits={bits} group={group} K={K} Ns={Ns} M={M} case={case}"
            assert L.gwq_linear_plan(count, arr, M, int(rng.integers(0, 2)), buf, 256) == 0, what
            text = buf.value.decode()
            seen.add(text.split("<")[0])
            lds = int(re.search(r" lds (\d+)", text).group(1))
            block = int(re.search(r" block (\d+)", text).group(1))
            assert 0 < lds <= 160 * 1024, (what, text)
            assert block % 64 == 0 and 64 <= block <= (1024 if text.startswith(("decode_small", "gemm_kernel")) else 512), (what, text)
            grid = re.search(r" grid (\d+)(?:x(\d+))?", text)
            assert int(grid.group(1)) >= 1, (what, text)
            if grid.group(2):
                assert 1 <= int(grid.group(2)) <= count, (what, text)
    finally:
        for k in keys:
            L.gwq_tuning_set(k.encode(), 0)
    assert {"decode_small_kernel", "decode_stream_kernel", "decode_wide_kernel", "gemm_kernel"} <= seen


def test_linear_gate_up_validates_before_touching_the_device():
    L = binding.lib()
    fake = ctypes.c_void_p(0x1000)
    ok = _packed()
    assert L.gwq_linear_gate_up(None, ctypes.byref(ok), fake, 1, fake, None, 0, None) == -1
    assert L.gwq_linear_gate_up(ctypes.byref(ok), None, fake, 1, fake, None, 0, None) == -1
    assert L.gwq_linear_gate_up(ctypes.byref(ok), ctypes.byref(ok), None, 1, fake, None, 0, None) == -1
    assert L.gwq_linear_gate_up(ctypes.byref(ok), ctypes.byref(ok), fake, 17, fake, None, 0, None) == -2     # decode sizes only
    assert L.gwq_linear_gate_up(ctypes.byref(ok), ctypes.byref(_packed(N=8)), fake, 1, fake, None, 0, None) == -2
    assert L.gwq_linear_gate_up(ctypes.byref(ok), ctypes.byref(_packed(bits=3)), fake, 1, fake, None, 0, None) == -3
    assert L.gwq_linear_gate_up(ctypes.byref(ok), ctypes.byref(ok), fake, 8, fake, None, 0, None) == -4      # M > 4 needs the workspace
    assert L.gwq_linear_gate_up(ctypes.byref(ok), ctypes.byref(ok), fake, 8, fake, fake, 4 * 8 * 4 - 1, None) == -4
    assert L.gwq_linear_gate_up(ctypes.byref(ok), ctypes.byref(ok), fake, 8, fake, ctypes.c_void_p(0x1008), 1 << 20, None) == -2


def test_quality_validates_before_touching_the_device():
    L = binding.lib()
    fake = ctypes.c_void_p(0x1000)
    ok = _packed()
    need = gwq.layout(4, 128, 4)["quality_workspace"]
    assert need == 4 * 24                                                       # three doubles per channel
    assert L.gwq_quality(None, fake, fake, 0, fake, fake, need, None) == -1
    assert L.gwq_quality(ctypes.byref(ok), None, fake, 0, fake, fake, need, None) == -1
    assert L.gwq_quality(ctypes.byref(ok), fake, None, 0, fake, fake, need, None) == -1
    assert L.gwq_quality(ctypes.byref(ok), fake, fake, 0, None, fake, need, None) == -1
    assert L.gwq_quality(ctypes.byref(ok), fake, fake, 2, fake, fake, need, None) == -3
    assert L.gwq_quality(ctypes.byref(ok), fake, fake, 0, fake, None, need, None) == -4
    assert L.gwq_quality(ctypes.byref(ok), fake, fake, 0, fake, fake, need - 1, None) == -4
    assert L.gwq_quality(ctypes.byref(ok), ctypes.c_void_p(0x1008), fake, 0, fake, fake, need, None) == -2
    assert L.gwq_quality(ctypes.byref(ok), fake, fake, 0, ctypes.c_void_p(0x1004), fake, need, None) == -2
    assert L.gwq_quality(ctypes.byref(_packed(bits=5)), fake, fake, 0, fake, fake, need, None) == -3


def test_linear_batch_validates_before_touching_the_device():
    L = binding.lib()
    fake = ctypes.c_void_p(0x1000)
    ok, other = _packed(), _packed(bits=3)
    P = (ctypes.POINTER(binding._Packed) * 2)(ctypes.pointer(ok), ctypes.pointer(ok))
    Pmixed = (ctypes.POINTER(binding._Packed) * 2)(ctypes.pointer(ok), ctypes.pointer(other))
    ptrs = (ctypes.c_void_p * 2)(0x1000, 0x1000)
    holes = (ctypes.c_void_p * 2)(0x1000, None)
    assert L.gwq_linear_batch(2, None, ptrs, 1, ptrs, None) == -1
    assert L.gwq_linear_batch(2, P, None, 1, ptrs, None) == -1
    assert L.gwq_linear_batch(2, P, ptrs, 1, holes, None) == -1
    assert L.gwq_linear_batch(0, P, ptrs, 1, ptrs, None) == -2
    assert L.gwq_linear_batch(9, P, ptrs, 1, ptrs, None) == -2
    assert L.gwq_linear_batch(2, P, ptrs, 17, ptrs, None) == -2         # the grouped launch is decode only
    assert L.gwq_linear_batch(2, Pmixed, ptrs, 1, ptrs, None) == -3     # mixed bit widths


def test_tuning_and_strings():
    L = binding.lib()
    assert L.gwq_tuning_set(b"decode_waves", 17) == -3
    assert L.gwq_tuning_set(b"decode_waves", -1) == -3
    assert L.gwq_tuning_set(b"nonsense", 1) == -3
    assert L.gwq_tuning_set(None, 1) == -1
    assert L.gwq_tuning_set(b"decode_waves", 2) == 0 and L.gwq_tuning_set(b"decode_waves", 0) == 0
    assert L.gwq_tuning_set(b"decode_pairs", 3) == -3 and L.gwq_tuning_set(b"decode_pairs", 2) == 0 and L.gwq_tuning_set(b"decode_pairs", 0) == 0
    assert L.gwq_tuning_set(b"gemm_rows", 48) == -3 and L.gwq_tuning_set(b"gemm_rows", 512) == -3
    for rows in (32, 64, 128, 256, 0):
        assert L.gwq_tuning_set(b"gemm_rows", rows) == 0
    assert L.gwq_status_string(0) == b"ok"
    assert b"workspace" in L.gwq_status_string(-4)
    assert gwq.version().startswith("gwq-gfx950")
    with pytest.raises(gwq.GwqError):
        gwq.layout(4, 100, 4)


def test_score_validates_before_touching_the_device():
    L = gwq.binding.lib()
    fake = ctypes.c_void_p(0x1000)
    f = ctypes.c_float
    assert L.gwq_score(None, fake, 4, 8, 128, f(1), f(0), fake, None) == -1
    assert L.gwq_score(fake, None, 4, 8, 128, f(1), f(0), fake, None) == -1
    assert L.gwq_score(fake, fake, 4, 8, 128, f(1), f(0), None, None) == -1
    for M, N, K in ((0, 8, 128), (4, 0, 128), (4, 8, 0), (4, 8, 64), (4, 8, 192), (4, 8, 65536 + 128), (4, (1 << 24) + 8, 128)):
        assert L.gwq_score(fake, fake, M, N, K, f(1), f(0), fake, None) == -2, (M, N, K)
    assert L.gwq_score(ctypes.c_void_p(0x1008), fake, 4, 8, 128, f(1), f(0), fake, None) == -2   # N % 8 == 0: 16 bytes
    assert L.gwq_score(ctypes.c_void_p(0x1001), fake, 4, 7, 128, f(1), f(0), fake, None) == -2
    assert L.gwq_score(fake, ctypes.c_void_p(0x1008), 4, 8, 128, f(1), f(0), fake, None) == -2
    assert L.gwq_score(fake, fake, 4, 8, 128, f(1), f(0), ctypes.c_void_p(0x1002), None) == -2
