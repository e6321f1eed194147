"""Where the time of one decode launch goes: shader-clock stamps of the kernels' milestones.

    python -m paper_2411_00850_amd.stamps N K M bits [key=value ...]

A measurement tool, not part of the product path.  It loads the separate library libgwq_stamp.so (the same sources
built with -DGWQ_STAMP: `python -m paper_2411_00850_amd.build --stamps`), in which wave 0 of every block (the lean
kernel: its first and its last wave) records the shader clock at the kernel's milestones, packs a seeded random
N x K layer (1 % outliers), warms up over four copies of it, runs one launch at M rows and prints, per milestone,
the median and the maximum over the blocks of the clocks since the block's first stamp.  key=value pairs go to
gwq_tuning_set first (decode_tiles=6, decode_stream=2, ...).  Which table is printed follows from the kernel that
gwq_linear_plan names for the call.
"""
import ctypes
import os
import sys


def main(argv):
    if len(argv) < 4:
        print(__doc__)
        return 2
    import numpy as np
    import torch
    from . import binding, build
    if not os.path.exists(build.STAMP_LIB):
        build.build(stamps=True)
    binding._LIB_PATH = build.STAMP_LIB
    N, K, M, bits = (int(a) for a in argv[:4])
    for kv in argv[4:]:
        k, _, v = kv.partition("=")
        binding.tuning_set(k, int(v))
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    layers = []
    for _ in range(4):
        W = (torch.randn((N, K), device=dev, generator=gen) * 0.02).half()
        S = torch.rand((N, K), device=dev, generator=gen)
        layers.append(binding.pack(W, S, bits, 10000, with_index=False))
    x = torch.randn((M, K), device=dev, generator=gen).half()
    y = torch.empty((M, N), dtype=torch.float16, device=dev)
    plan = binding.linear_plan(layers[0], M)
    print(plan)
    L = binding.lib()
    L.gwq_debug_read_stamps.argtypes = [ctypes.c_void_p, ctypes.c_int]
    for _ in range(3):
        for P in layers:
            binding.linear(P, x, out=y)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    binding.linear(layers[0], x, out=y)
    e1.record()
    torch.cuda.synchronize()
    buf = np.zeros(2048 * 16, np.uint64)
    if L.gwq_debug_read_stamps(buf.ctypes.data, buf.size) < 0:
        raise RuntimeError("gwq_debug_read_stamps failed")
    grid = int(plan.split(" grid ")[1].split("x")[0])
    st = buf.reshape(2048, 16)[:min(2048, grid)].astype(np.int64)
    print(f"N={N} K={K} M={M} bits={bits}: one launch, {e0.elapsed_time(e1) * 1e3:.1f} us between HIP events (stamps included); "
          f"shader clocks, median / max over {st.shape[0]} blocks")

    def table(names, rel):
        for i, nm in enumerate(names):
            if nm:
                print(f"  {nm:30s} {np.median(rel[:, i]):9.0f} {rel[:, i].max():9.0f}")

    if plan.startswith("decode_small"):
        names = ["descriptor has arrived", "staging and first codes requested", "X, scales, zero points in LDS",
                 "all codes multiplied", "outliers added", "partial sums in LDS", "stored"]
        print("  first wave of the block:")
        table(names, st[:, 1:8] - st[:, 1:2])
        print("  last wave of the block (clocks since the first wave's first stamp):")
        table(names, st[:, 8:15] - st[:, 1:2])
    elif plan.startswith("decode_stream"):
        tiles = int(plan.split("tiles_per_block ")[1])
        st = st[st[:, 12] > 0]
        rel = st[:, 2:13] - st[:, 1:2]
        table(["everything requested", "X operands in registers", "XT written, first barrier passed",
               "tile 0: codes have arrived", "tile 0: multiplied", "tile 0: CSR segment in LDS", "tile 0: through the barrier",
               "tile 0: outliers added", "all tiles done", "last barrier", "stored"], rel)
        if tiles > 1:
            print(f"  {'per tile after the first':30s} {np.median((rel[:, 8] - rel[:, 7]) / (tiles - 1)):9.0f}")
    else:
        st = st[st[:, 12] > 0]
        rel = st[:, 2:13] - st[:, 1:2]
        phases = int(plan.split(" phases ")[1])
        names = []
        for ph in range(3):
            names += [f"phase {ph}: X in LDS", f"phase {ph}: multiplied", f"phase {ph}: outliers added"] if ph < phases else ["", "", ""]
        table(names + ["", "first tile stored"], rel)
    wall = st[:, 0] - st[:, 0].min()
    print(f"  block start spread: median {np.median(wall) / 100:.2f} us, max {wall.max() / 100:.2f} us (100 MHz wall clock)")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
