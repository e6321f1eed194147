#!/usr/bin/env python3
"""Benchmark of the GWQ linear-layer path on one MI355X.

Workload (benchmark configs[1]): one LLaMA-2-7B-shaped decoder layer, 7 matrices, 4-bit codes,
group 128, 1 % FP16 outliers, synthetic weights with planted outlier columns.  A step is one decode
pass (M = 1) over the 7 matrices, launched the way the layer's data flow allows: q, k and v in one
grouped launch (gwq_linear_batch), o alone, gate and up in one, down alone - 4 launches.  The packed
layer exists in several copies and the steps rotate over them, so every step streams its weights
from HBM rather than from the 256 MB last-level cache, as a decode pass over a whole model does.

One JSON line is printed.  `value` is the algorithmic GB/s of the K timed steps (packed bytes + X + Y
per step over wall time, inputs resident in HBM).  `roofline` is the decode kernel alone: algorithmic
bytes per launch over the launch duration, from HIP events on the launch stream around each of at least
200 further steps (median over the replays, whatever --steps says: 20 steps are 0.7 ms, too short to
settle).  `roofline.kernel` is what the library's dispatcher reports for the launches that ran
(gwq_linear_plan), `roofline.achievable` a plain streaming read of the same bytes launched the same way
(gwq_probe_stream: the ceiling a kernel with no arithmetic reaches on this machine), and
`roofline.traffic` the counter-measured HBM bytes, taken from profiles/ only when that summary was made
from the decode sources as they are now.  Further objects report the same pass at M = 4 and 16, the
prefill GEMM (M = 2048) in TFLOP/s against the MFMA peak and against MFMAs issued from registers
(gwq_probe_mfma), the 3-bit layer, the 70B shapes, gwq_pack / gwq_quality / gwq_score, one row per
(configuration, shape, bits, M) with the oracle timed beside the kernel (`extras.rows`), a 512-step
decoder-layer loop against FP16 weights, and the CPU oracle on a bounded sample (`cpu_baseline`).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(P, M):
    """Bytes the method must move for one gwq_linear call: packed layer + X + Y."""
    gpr = P.K // 128
    wpg = 16 if P.bits == 4 else 13
    packed = P.N * gpr * wpg * 4 + P.N * (P.K // P.group) * (2 + 1) + (P.N + 1) * 4 + P.n_outliers * 4
    return packed + 2 * M * P.K + 2 * M * P.N


def flops(P, M):
    return 2.0 * M * P.N * P.K + 2.0 * M * P.n_outliers


def clone_layer(P):
    from paper_2411_00850_amd.binding import PackedLayer
    return PackedLayer(P.N, P.K, P.bits, P.ppm, P.n_outliers, P.qweight.clone(), P.scales.clone(),
                       P.zeros.clone(), P.row_ptr.clone(), P.col_idx.clone(), P.out_val.clone(),
                       P.index.clone() if P.index is not None else None, P.group)


def settle(fn, seconds=0.1):
    """Run fn for a while before timing it: the first calls after lighter work run below the settled rate."""
    import torch
    t = time.perf_counter()
    while time.perf_counter() - t < seconds:
        fn()
        torch.cuda.synchronize()


def source_hash():
    """SHA-1 (12 hex digits) of the decode kernels' sources: ties a counter summary to the code it measured."""
    import hashlib
    h = hashlib.sha1()
    for name in ("gwq_decode.hip", "gwq_dequant.h", "gwq_internal.h"):
        h.update(open(os.path.join(ROOT, "paper_2411_00850_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:12]


def read_traffic():
    """HBM bytes per decode launch from the committed rocprofv3 counter summary - only when the summary was
    made from the decode sources as they are now (its `source_sha1` line), else None."""
    path = os.path.join(ROOT, "profiles", "decode_gemv_7b_int4_m1_pmc.txt")
    traffic, made_from = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
            if line.startswith("source_sha1:"):
                made_from = line.split(":")[1].strip()
    except OSError:
        return None
    return traffic if made_from == source_hash() else None


def median_replay_ms(graph, min_replays):
    """Median duration of one replay of `graph`, from a pair of HIP events on the launch stream around each."""
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min_replays)]
    torch.cuda.synchronize()
    for a, b in evs:
        a.record()
        graph.replay()
        b.record()
    torch.cuda.synchronize()
    return float(np.median([a.elapsed_time(b) for a, b in evs]))


def result_rows(gwq, gs, dev, torch):
    """extras.rows: for configurations 1-4 (the 4096 x 4096 layer and the 7B shapes) the full matrices - the
    oracle selects, encodes and multiplies on the host, the library packs and multiplies on the GPU, and the
    two are compared (packing byte for byte, outputs by the two error measures of the tolerance); for
    configuration 5 (70B shapes) the kernel runs the full matrices and the oracle a slab of 1024 channels,
    its times scaled by N / 1024 and marked as such.  Oracle times: `all` = the cores of this process
    (OpenMP over channels in the product; selection and encoding are serial code), `one` = one thread."""
    import ctypes
    from oracle import gwq_oracle as orc
    gomp = ctypes.CDLL("libgomp.so.1")
    cores = len(os.sched_getaffinity(0))

    def timed(fn, threads):
        gomp.omp_set_num_threads(threads)
        t = time.perf_counter()
        r = fn()
        dt = time.perf_counter() - t
        gomp.omp_set_num_threads(cores)
        return r, dt

    def gpu_us(Ps, M, K, N, index=None):
        x = torch.from_numpy(gs.activations(M, K, gs.rng_for(9, M, K))).to(dev)
        y = torch.empty((M, N), dtype=torch.float16, device=dev)
        calls = [gwq.prepare_linear(P, x, y, index=index[i] if index else None) for i, P in enumerate(Ps)]
        for c in calls:
            c()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for c in calls:
                c()
        settle(graph.replay, 0.05)
        us = median_replay_ms(graph, max(10, 120 // len(Ps))) * 1e3 / len(Ps)
        return us, x, y

    def errors(Yg, Yr):
        Yg = Yg.astype(np.float64)
        return (float(np.linalg.norm(Yg - Yr) / max(np.linalg.norm(Yr), 1e-300)),
                float(np.abs(Yg - Yr).max() / max(np.abs(Yr).max(), 1e-300)))

    rows = []
    plan = [(1, "single 4096x4096", 4096, 4096, lambda: gs.config1()[:2], [(4, (1,))]),
            (2, "q/k/v/o 4096x4096", 4096, 4096, lambda: gs.layer_matrix(2, 0, 4096, 4096), [(4, (1, 4, 16, 2048)), (3, (1, 8))]),
            (2, "gate/up 11008x4096", 11008, 4096, lambda: gs.layer_matrix(2, 4, 11008, 4096), [(4, (1, 4, 16, 2048)), (3, (1, 8))]),
            (2, "down 4096x11008", 4096, 11008, lambda: gs.layer_matrix(2, 6, 4096, 11008), [(4, (1, 4, 16, 2048)), (3, (1, 8))])]
    for cfg, shape, N, K, make, variants in plan:
        W, S = make()
        mask, t_sel = timed(lambda: orc.select(S, 10000), 1)
        Wd, Sd = torch.from_numpy(W).to(dev), torch.from_numpy(S).to(dev)
        for bits, Ms in variants:
            P, t_enc = timed(lambda: orc.encode(W, mask, bits, 10000), 1)
            D = gwq.pack(Wd, Sd, bits, 10000)
            settle(lambda: gwq.pack(Wd, Sd, bits, 10000), 0.05)
            t = time.perf_counter()
            for _ in range(3):
                D = gwq.pack(Wd, Sd, bits, 10000)
            torch.cuda.synchronize()
            pack_ms = (time.perf_counter() - t) / 3 * 1e3
            g = N * (K // 128)
            exact = all(np.array_equal(a.reshape(b.shape), b) for a, b in (
                (D.qweight.cpu().numpy().view(np.uint32), P.qweight), (D.scales.cpu().numpy().view(np.uint16)[:g], P.scales),
                (D.zeros.cpu().numpy()[:g], P.zeros), (D.row_ptr.cpu().numpy(), P.row_ptr),
                (D.col_idx.cpu().numpy().view(np.uint16)[:D.n_outliers], P.col_idx),
                (D.out_val.cpu().numpy().view(np.uint16)[:D.n_outliers], P.out_val)))
            pack_bytes = 6 * N * K + D.nbytes()
            rows.append({"config": cfg, "shape": shape, "bits": bits, "op": "gwq_pack", "bytes": pack_bytes,
                         "gpu_ms": round(pack_ms, 3), "GB/s": round(pack_bytes / pack_ms / 1e6, 1),
                         "frac_hbm_peak": round(pack_bytes / pack_ms / 1e6 / HBM_PEAK_GBS, 4),
                         "oracle_s": {"select": round(t_sel, 2), "encode": round(t_enc, 2), "threads": 1},
                         "pack_bit_exact": bool(exact)})
            clones = [D] + [clone_layer(D) for _ in range(5)]
            for M in Ms:
                cfg_m = 4 if M == 2048 else (3 if bits == 3 and cfg == 2 else cfg)
                if M <= 16:
                    us, x, y = gpu_us(clones, M, K, N)
                else:
                    us, x, y = gpu_us(clones[:2], M, K, N)
                Yg = y.cpu().numpy()
                X = x.cpu().numpy()
                b, fl = algorithmic_bytes(D, M), flops(D, M)
                row = {"config": cfg_m, "shape": shape, "bits": bits, "op": "gwq_linear", "M": M, "bytes": b, "flops": fl,
                       "gpu_us": round(us, 2), "GB/s": round(b / us / 1e3, 1), "TFLOP/s": round(fl / us / 1e6, 2),
                       "kernel": gwq.linear_plan(D, M).split(" ")[0]}
                if M <= 64:
                    row["bound"], row["frac"] = "hbm", round(b / us / 1e3 / HBM_PEAK_GBS, 4)
                else:
                    row["bound"], row["frac"] = "mfma", round(fl / us / 1e6 / MFMA_F16_PEAK_TFLOPS, 4)
                if M <= 16:
                    Yr, t_all = timed(lambda: orc.linear_f64(P, X), cores)
                    _, t_one = timed(lambda: orc.linear_f64(P, X), 1)
                    row["oracle_s"] = {"all": round(t_all, 4), "one": round(t_one, 4), "cores": cores}
                    row["rel_fro"], row["max_abs"] = errors(Yg, Yr)
                else:                                   # a stated subset of channels, scaled to the matrix
                    sub = np.arange(0, N, N // 256, dtype=np.int32)[:256]
                    Yr, t_all = timed(lambda: orc.linear_f64(P, X, sub), cores)
                    _, t_one = timed(lambda: orc.linear_f64(P, X, sub[:16]), 1)
                    row["oracle_s"] = {"all": round(t_all * N / sub.size, 2), "one": round(t_one * N / 16, 1), "cores": cores,
                                       "sample": f"{sub.size} channels (every {N // 256}th) on all cores, 16 on one; scaled to N"}
                    row["rel_fro"], row["max_abs"] = errors(Yg[:, sub], Yr)
                row["within_tolerance"] = bool(row["rel_fro"] <= 2e-3 and row["max_abs"] <= 1e-2)
                rows.append(row)
                del x, y
            del clones, D
            torch.cuda.empty_cache()
        del Wd, Sd
    # configuration 5: full-size kernels on device-drawn weights, oracle on a slab of 1024 channels
    gen = torch.Generator(device=dev)
    gen.manual_seed(75)
    for name, N, K in gs.SHAPES_70B:
        rng = gs.rng_for(5, N % 97, K % 89)
        Ws = gs.weight(1024, K, rng)
        Ss = gs.score_from_weight(Ws, rng)
        Wd = (torch.randn((N, K), device=dev, generator=gen) * 0.02).half()
        Sd = torch.rand((N, K), device=dev, generator=gen)
        for bits in (4, 3):
            Pslab, t_pack = timed(lambda: orc.pack(Ws, Ss, bits, 10000), 1)
            D = gwq.pack(Wd, Sd, bits, 10000)
            clones = [D, clone_layer(D), clone_layer(D)]
            for M in (1, 64, 2048):
                us, x, y = gpu_us(clones if M == 1 else clones[:2], M, K, N)
                b, fl = algorithmic_bytes(D, M), flops(D, M)
                row = {"config": 5, "shape": f"{name} {N}x{K}", "bits": bits, "op": "gwq_linear", "M": M, "bytes": b, "flops": fl,
                       "gpu_us": round(us, 2), "GB/s": round(b / us / 1e3, 1), "TFLOP/s": round(fl / us / 1e6, 2),
                       "kernel": gwq.linear_plan(D, M).split(" ")[0]}
                if M <= 64:
                    row["bound"], row["frac"] = "hbm", round(b / us / 1e3 / HBM_PEAK_GBS, 4)
                else:
                    row["bound"], row["frac"] = "mfma", round(fl / us / 1e6 / MFMA_F16_PEAK_TFLOPS, 4)
                X = x.cpu().numpy()
                rows_all = None if M <= 64 else np.arange(0, 1024, 16, dtype=np.int32)
                n_all = 1024 if M <= 64 else 64
                _, t_all = timed(lambda: orc.linear_f64(Pslab, X, rows_all), cores)
                one_rows = np.arange(0, 1024, 1024 // (64 if M == 1 else 8 if M == 64 else 2), dtype=np.int32)
                _, t_one = timed(lambda: orc.linear_f64(Pslab, X, one_rows), 1)
                row["oracle_s"] = {"all": round(t_all * N / n_all, 3), "one": round(t_one * N / one_rows.size, 2), "cores": cores,
                                   "pack_one_thread": round(t_pack * N / 1024, 1),
                                   "sample": f"a slab of 1024 channels of the same K ({n_all} of them on all cores, "
                                             f"{one_rows.size} on one), scaled to N; parity of these shapes: tests/test_gpu_linear.py"}
                rows.append(row)
                del x, y
            del clones, D
            torch.cuda.empty_cache()
        del Wd, Sd
    return rows


def layer_loop(gwq, gs, dev, torch, copies, tokens=512):
    x0 = torch.from_numpy(gs.activations(1, 4096, gs.rng_for(2, 200, 1))).to(dev) * 0.05
    q, k, v, o = (torch.empty((1, 4096), dtype=torch.float16, device=dev) for _ in range(4))
    h = torch.empty((1, 11008), dtype=torch.float16, device=dev)
    y = torch.empty((1, 4096), dtype=torch.float16, device=dev)
    per_copy = []
    for c in copies:
        per_copy.append([gwq.prepare_linear_batch([c[0], c[1], c[2]], [x0, x0, x0], [q, k, v]),
                         gwq.prepare_linear(c[3], q, o),
                         gwq.prepare_linear_gate_up(c[4], c[5], o, h),
                         gwq.prepare_linear(c[6], h, y)])
    for calls in per_copy:
        for call in calls:
            call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for t in range(tokens):
            for call in per_copy[t % len(per_copy)]:
                call()
    settle(graph.replay, 0.2)
    ms = median_replay_ms(graph, 9)
    packed = sum(P.nbytes() for P in copies[0])
    res = {"tokens": tokens, "launches_per_token": 4, "gwq_int4_ms": round(ms, 3), "gwq_int4_us_per_token": round(ms * 1e3 / tokens, 2),
           "weight_bytes_gwq_int4": packed, "kernels": [gwq.linear_plan([copies[0][0]] * 3, 1).split(" ")[0],
                                                         "decode_small_gate_up_kernel<4,8,1>"]}
    del graph, per_copy
    # FP16 weights, vendor library
    g16 = torch.Generator(device=dev)
    g16.manual_seed(9)
    shapes = [(P.N, P.K) for P in copies[0]]
    w16 = [[(torch.randn(sh, device=dev, generator=g16, dtype=torch.float32) * 0.02).half() for sh in shapes] for _ in range(2)]
    g_, u_ = torch.empty_like(h), torch.empty_like(h)

    def fp16_token(ws):
        torch.matmul(x0, ws[0].t(), out=q); torch.matmul(x0, ws[1].t(), out=k); torch.matmul(x0, ws[2].t(), out=v)
        torch.matmul(q, ws[3].t(), out=o)
        torch.matmul(o, ws[4].t(), out=g_); torch.matmul(o, ws[5].t(), out=u_)
        torch.mul(torch.nn.functional.silu(g_), u_, out=h)
        torch.matmul(h, ws[6].t(), out=y)
    for ws in w16:
        fp16_token(ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for t in range(tokens):
            fp16_token(w16[t % 2])
    settle(graph.replay, 0.2)
    ms16 = median_replay_ms(graph, 5)
    fp16_bytes = sum(2 * n * k_ for n, k_ in shapes)
    res.update({"fp16_library_ms": round(ms16, 3), "speedup_vs_fp16": round(ms16 / ms, 2), "weight_bytes_fp16": fp16_bytes,
                "memory_ratio": round(fp16_bytes / packed, 2),
                "paper_context": "Sec. 4.2 efficiency table: x1.22-1.23 whole-model speedup and 12.83 G -> 4.16 G on an A800 (Llama-2-7B)"})
    del graph, w16
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3000)
    ap.add_argument("--warmup", type=int, default=3000,
                    help="untimed steps first; a few thousand (0.1 s) let the clocks settle: short warm-ups read 3 %% low")
    ap.add_argument("--copies", type=int, default=6, help="rotating copies of the packed layer")
    ap.add_argument("--group", choices=["deps", "none", "all"], default="deps",
                    help="launches per step: 4 grouped by data dependence (default), 7 single, or 1 over all")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="gwq_tuning_set before the run (e.g. decode_waves=8); repeatable")
    ap.add_argument("--launch", choices=["graph", "eager"], default="graph",
                    help="how the timed steps are launched: one HIP graph over all copies, or plain launches")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device copy (reference point for rocprofv3 byte counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the M=4/16, prefill and pack legs")
    ap.add_argument("--extras", default="all", metavar="LIST",
                    help="comma-separated extra legs to run: m,groups,big,fp16,prefill,int3,beta,bf16,pack,rows,loop (default: all)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (--gpus 1); multi-GPU runs are out of scope.")

    import torch
    import gwq_synth as gs
    import paper_2411_00850_amd as gwq
    for kv in args.tune:
        key, _, val = kv.partition("=")
        gwq.tuning_set(key, int(val))

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    # ---- inputs: generate on the host (seeded), pack on the GPU with gwq_pack -------------------
    t0 = time.time()
    want_int3 = not args.no_extras and (args.extras == "all" or "int3" in args.extras.split(","))
    want_beta = not args.no_extras and (args.extras == "all" or "beta" in args.extras.split(","))
    layers, layers3, pack_inputs = [], [], []
    layers_beta = {16: [], 32: [], 64: []}                # the same matrices in smaller quantisation groups
    for mid, (name, N, K) in enumerate(gs.SHAPES_7B):
        W, S = gs.layer_matrix(2, mid, N, K)
        Wd, Sd = torch.from_numpy(W).to(dev), torch.from_numpy(S).to(dev)
        layers.append(gwq.pack(Wd, Sd, 4, 10000))
        if want_int3:
            layers3.append(gwq.pack(Wd, Sd, 3, 10000))
        for group, lst in layers_beta.items() if want_beta else ():
            lst.append(gwq.pack(Wd, Sd, 4, 10000, group=group))
        if name in ("q", "gate", "down"):
            pack_inputs.append((name, Wd, Sd))
        else:
            del Wd, Sd
    torch.cuda.synchronize()
    log(f"[bench] generated and packed 7 matrices in {time.time() - t0:.1f} s")

    copies = [layers] + [[clone_layer(P) for P in layers] for _ in range(args.copies - 1)]
    torch.cuda.synchronize()

    def make_xy(M):
        xs = {K: torch.from_numpy(gs.activations(M, K, gs.rng_for(2, 100, K))).to(dev) for K in (4096, 11008)}
        ys = [torch.empty((M, P.N), dtype=torch.float16, device=dev) for P in layers]
        return xs, ys

    GROUPS = {"deps": [[0, 1, 2], [3], [4, 5], [6]], "none": [[i] for i in range(7)], "all": [list(range(7))]}

    def decode_leg(M, steps, warmup, mode, grouping="deps", copies=copies):
        """mode "graph": all copies x 7 launches captured once into a HIP graph and replayed (the
        launch-bound loop of a serving engine), bracketed by two HIP events on the launch stream whose
        elapsed time over the number of launches is the per-launch duration; "eager": plain launches;
        "events": eager with one HIP event between consecutive launches."""
        xs, ys = make_xy(M)
        groups = GROUPS[grouping]
        layers = copies[0]
        n_launch, n_copies = sum(len({layers[j].K for j in g}) for g in groups), len(copies)   # a grouped call launches once per distinct K
        calls = [[gwq.prepare_linear_batch([c[j] for j in g], [xs[c[j].K] for j in g], [ys[j] for j in g])
                  if len(g) > 1 else gwq.prepare_linear(c[g[0]], xs[c[g[0]].K], ys[g[0]]) for g in groups]
                 for c in copies]
        for i in range(warmup):
            for call in calls[i % n_copies]:
                call()
        torch.cuda.synchronize()
        kernel_ms, median_step_ms = None, None
        if mode == "graph":
            ref = [y.clone() for y in ys]               # eager result of the last warm-up step
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for c in calls:
                    for call in c:
                        call()
            graph.replay()
            torch.cuda.synchronize()
            if warmup and not all(torch.equal(a, b) for a, b in zip(ref, ys)):
                sys.exit("bench.py: graph replay does not reproduce the eager result")
            # Whatever W was asked for, the chip gets 0.1 s of the same replays before the timed region:
            # right after lighter work the first milliseconds run about 3 % below the settled rate.
            settle(graph.replay)
            rounds, rest = divmod(steps, n_copies)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t = time.perf_counter()
            e0.record()                                  # HIP events on the launch stream
            for _ in range(rounds):
                graph.replay()
            for call in [c for cc in calls[:rest] for c in cc]:
                call()
            e1.record()
            torch.cuda.synchronize()
            wall = time.perf_counter() - t
            kernel_ms = e0.elapsed_time(e1) / (steps * n_launch)
            # at least 200 more steps, one pair of events per replay (n_copies steps), median
            median_step_ms = median_replay_ms(graph, max(20, -(-200 // n_copies))) / n_copies
        else:
            ev = mode == "events"
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(n_launch + 1)] for _ in range(steps)] if ev else None
            torch.cuda.synchronize()
            t = time.perf_counter()
            for i in range(steps):
                if ev:
                    evs[i][0].record()
                for j, call in enumerate(calls[(warmup + i) % n_copies]):
                    call()
                    if ev:
                        evs[i][j + 1].record()
            torch.cuda.synchronize()
            wall = time.perf_counter() - t
            if ev:
                kernel_ms = sum(evs[i][j].elapsed_time(evs[i][j + 1]) for i in range(steps) for j in range(n_launch))
                kernel_ms /= steps * n_launch
        bytes_step = sum(algorithmic_bytes(P, M) for P in layers)
        decode_leg.median_step_ms = median_step_ms      # of the leg that ran last
        decode_leg.plans = [gwq.linear_plan([layers[j] for j in g if layers[j].K == k], M)
                            for g in groups for k in dict.fromkeys(layers[j].K for j in g)]
        return wall / steps, kernel_ms, bytes_step, n_launch

    def stream_read_leg(M, grouping, layer_set):
        """The ceiling: one plain streaming read (gwq_probe_stream) per launch of the decode pass, over exactly
        the launch's algorithmic bytes, the same number of rotating copies, replayed from one graph."""
        groups = GROUPS[grouping]
        per_launch = [sum(algorithmic_bytes(layer_set[j], M) for j in g if layer_set[j].K == k) // 16 * 16
                      for g in groups for k in dict.fromkeys(layer_set[j].K for j in g)]
        bufs = [[torch.empty(b, dtype=torch.uint8, device=dev).random_(0, 255) for b in per_launch] for _ in range(args.copies)]
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        for c in bufs:
            for t in c:
                gwq.probe_stream(t, sink)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for c in bufs:
                for t in c:
                    gwq.probe_stream(t, sink)
        settle(graph.replay)
        ms = median_replay_ms(graph, max(20, -(-200 // args.copies))) / args.copies
        del graph, bufs
        torch.cuda.empty_cache()
        return {"us_per_step": round(ms * 1e3, 2), "GB/s": round(sum(per_launch) / ms / 1e6, 1),
                "launches_per_step": len(per_launch), "what": "plain streaming read of the same bytes, same launches and rotation"}

    # ---- the timed steps: decode M = 1 ---------------------------------------------------------------
    step_s, launch_ms, bytes_step, n_launch = decode_leg(1, args.steps, args.warmup, args.launch, args.group)
    value = bytes_step / step_s / 1e9
    if launch_ms is None:
        # Eager launches are CPU-bound: time the kernels with one HIP event between consecutive launches.
        _, launch_ms, _, _ = decode_leg(1, args.steps, args.warmup, "events", args.group)
    bytes_launch = bytes_step / n_launch
    achieved_timed = bytes_launch / (launch_ms * 1e-3) / 1e9
    med_ms = decode_leg.median_step_ms
    if med_ms is not None:
        launch_ms = med_ms / n_launch                   # the figure the roofline uses: median over >= 200 steps
    achieved = bytes_launch / (launch_ms * 1e-3) / 1e9
    plans = decode_leg.plans
    kernels = sorted({p.split(" ")[0] for p in plans})
    ceiling = stream_read_leg(1, args.group, layers) if args.launch == "graph" else None
    out = {
        "metric": "gwq_linear decode GB/s (% HBM peak) & prefill TFLOP/s (% MFMA peak), 7B shapes",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_s * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "7B decoder layer (q,k,v,o 4096x4096; gate,up 11008x4096; down 4096x11008), "
                               "int4 g128 + 1% fp16 CSR outliers, decode M=1",
                   "launches_per_step": n_launch, "grouping": {"deps": "qkv | o | gate,up | down", "none": "one launch per matrix",
                                                               "all": "one call over the 7 matrices (one launch per distinct K)"}[args.group],
                   "copies_rotated": args.copies, "bytes_per_step": bytes_step, "launch": args.launch},
        "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
        "roofline": {"bound": "hbm", "kernel": kernels[0] if len(kernels) == 1 else kernels, "launches": plans,
                     "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": read_traffic(), "bytes_per_launch": round(bytes_launch),
                     "avg_launch_us": round(launch_ms * 1e3, 3),
                     "timing": "median over >= 200 steps, HIP events around each graph replay" if med_ms is not None
                               else "mean over the timed steps",
                     "achieved_in_timed_steps": round(achieved_timed, 1)},
    }
    if ceiling:
        out["roofline"]["achievable"] = ceiling
        out["roofline"]["frac_of_achievable"] = round(bytes_step / (launch_ms * n_launch * 1e-3) / 1e9 / ceiling["GB/s"], 4)

    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)                              # one copy kernel: reads and writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    legs = set("m,groups,big,fp16,prefill,int3,beta,bf16,pack,rows,loop".split(",")) if args.extras == "all" else set(args.extras.split(","))
    if not args.no_extras:
        extra = {}
        for M in (4, 16) if "m" in legs else ():
            s, _, b, _ = decode_leg(M, max(args.steps // 3, 12), max(args.warmup // 3, 12), args.launch, args.group)
            if decode_leg.median_step_ms:
                s = decode_leg.median_step_ms * 1e-3
            extra[f"decode_M{M}"] = {"GB/s": round(b / s / 1e9, 1), "ms_per_step": round(s * 1e3, 5),
                                     "pct_hbm_peak": round(100 * b / s / 1e9 / HBM_PEAK_GBS, 2),
                                     "kernels": sorted({p.split(" ")[0] for p in decode_leg.plans})}
        for grouping in ("none", "all") if "groups" in legs else ():   # the same M = 1 pass with 7 launches / 1 launch per step
            if grouping != args.group:
                s, _, b, nl = decode_leg(1, max(args.steps // 3, 12), max(args.warmup // 3, 12), args.launch, grouping)
                extra[f"decode_M1_group_{grouping}"] = {"GB/s": round(b / s / 1e9, 1), "ms_per_step": round(s * 1e3, 5),
                                                        "launches_per_step": nl}
        # decode M = 1 on 70B-shaped matrices (one launch each; weights drawn on the device, three
        # rotating copies of each so that they stream from HBM): how the same kernel does when the
        # fixed cost of a launch is spread over 4-14 times the bytes
        big, big_m = {}, {}
        gen = torch.Generator(device=dev)
        gen.manual_seed(70)
        for name, N, K in gs.SHAPES_70B if "big" in legs else ():
            Wd = (torch.randn((N, K), device=dev, generator=gen) * 0.02).half()
            Sd = torch.rand((N, K), device=dev, generator=gen)
            P0 = gwq.pack(Wd, Sd, 4, 10000)
            del Wd, Sd
            Ps = [P0, clone_layer(P0), clone_layer(P0)]
            x = torch.randn((1, K), device=dev, generator=gen).half()
            y = torch.empty((1, N), dtype=torch.float16, device=dev)
            calls = [gwq.prepare_linear(P, x, y) for P in Ps]
            for call in calls:
                call()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for call in calls:
                    call()
            settle(graph.replay)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            us = median_replay_ms(graph, 70) * 1e3 / len(calls)      # 210 launches
            bb = algorithmic_bytes(P0, 1)
            big[f"{name}_{N}x{K}"] = {"us": round(us, 2), "GB/s": round(bb / us / 1e3, 1),
                                      "pct_hbm_peak": round(100 * bb / us / 1e3 / HBM_PEAK_GBS, 2),
                                      "kernel": gwq.linear_plan(P0, 1).split(" ")[0]}
            del calls, graph
            # the same bytes through the plain streaming read, three rotating buffers, one graph
            sink = torch.zeros(4, dtype=torch.int32, device=dev)
            pb = [torch.empty(bb // 16 * 16, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(3)]
            for t in pb:
                gwq.probe_stream(t, sink)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for t in pb:
                    gwq.probe_stream(t, sink)
            settle(graph.replay)
            us_s = median_replay_ms(graph, 70) * 1e3 / 3
            big[f"{name}_{N}x{K}"]["achievable_GB/s"] = round(bb / us_s / 1e3, 1)
            big[f"{name}_{N}x{K}"]["frac_of_achievable"] = round(us_s / us, 4)
            del graph, pb
            # the same matrices at M = 64 and M = 2048 (prebuilt index; eager launches, rotating copies)
            indexes = [gwq.linear_index(P) for P in Ps]
            for M in (64, 2048):
                x = torch.randn((M, K), device=dev, generator=gen).half()
                y = torch.empty((M, N), dtype=torch.float16, device=dev)
                calls = [gwq.prepare_linear(P, x, y, index=ix) for P, ix in zip(Ps, indexes)]
                for call in calls:
                    call()
                torch.cuda.synchronize()
                reps = 4 if M == 2048 else 10
                e0.record()
                for _ in range(reps):
                    for call in calls:
                        call()
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / (reps * len(calls))
                big_m.setdefault(f"M{M}", {})[f"{name}_{N}x{K}"] = {
                    "us": round(us, 1), "TFLOP/s": round(flops(P0, M) / us / 1e6, 1),
                    "GB/s": round(algorithmic_bytes(P0, M) / us / 1e3, 1)}
                del calls, x, y
            del Ps, P0, indexes
            torch.cuda.empty_cache()
        if big:
            extra["decode_M1_70b_shapes"] = big
            extra["linear_70b_shapes"] = big_m
        # The same decode pass with FP16 weights through the vendor library (torch's F.linear), as the
        # paper's efficiency table does (Sec. 4.2: speed and memory against FP16): 7 products per pass,
        # two rotated copies of the FP16 layer (809 MB), graph replay.  Comparison only, not a product path.
        try:
            if "fp16" not in legs:
                raise KeyError("skipped")
            g16 = torch.Generator(device=dev)
            g16.manual_seed(7)
            w16 = [[(torch.randn((P.N, P.K), device=dev, generator=g16, dtype=torch.float32) * 0.02).half()
                    for P in layers] for _ in range(2)]
            xs, _ = make_xy(1)
            outs = [torch.empty((1, P.N), dtype=torch.float16, device=dev) for P in layers]

            def fp16_pass(ws):
                for j, P in enumerate(layers):
                    torch.matmul(xs[P.K], ws[j].t(), out=outs[j])
            for _ in range(3):
                fp16_pass(w16[0]); fp16_pass(w16[1])
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                fp16_pass(w16[0]); fp16_pass(w16[1])
            graph.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 50
            e0.record()
            for _ in range(reps):
                graph.replay()
            e1.record()
            torch.cuda.synchronize()
            fp16_ms = e0.elapsed_time(e1) / (2 * reps)
            fp16_bytes = sum(2 * P.N * P.K for P in layers)
            packed_bytes = sum(P.nbytes() for P in layers)
            extra["fp16_library_decode_M1"] = {"ms_per_step": round(fp16_ms, 5), "GB/s": round(fp16_bytes / fp16_ms / 1e6, 1),
                                               "speedup_of_gwq_int4": round(fp16_ms / (step_s * 1e3), 2),
                                               "weight_bytes_fp16": fp16_bytes, "weight_bytes_gwq_int4": packed_bytes,
                                               "memory_ratio": round(fp16_bytes / packed_bytes, 2)}
            del w16, graph, outs
            torch.cuda.empty_cache()
        except KeyError:
            pass
        except Exception as ex:                            # the comparison must not take the benchmark down
            extra["fp16_library_decode_M1"] = {"error": str(ex)[:200]}
        # prefill: M = 2048 over the 7 matrices, one copy (compute-bound).  Two ways: gwq_linear, which
        # rebuilds its per-layer index in the workspace on every call, and gwq_linear_indexed with the
        # index built once per layer beforehand (it depends on the weights only).
        if "prefill" in legs:
            M = 2048
            xs, ys = make_xy(M)
            fl = sum(flops(P, M) for P in layers)

            def time_prefill(calls, reps=20):
                # Warm up for a fifth of a second: the first passes after lighter work run up to 10 %
                # slower than the settled rate, whichever variant comes first.
                t = time.perf_counter()
                while time.perf_counter() - t < 0.2:
                    for c in calls:
                        c()
                    torch.cuda.synchronize()
                t = time.perf_counter()
                for _ in range(reps):
                    for c in calls:
                        c()
                torch.cuda.synchronize()
                s = (time.perf_counter() - t) / reps
                return {"TFLOP/s": round(fl / s / 1e12, 1), "ms_per_pass": round(s * 1e3, 4),
                        "pct_mfma_f16_peak": round(100 * fl / s / 1e12 / MFMA_F16_PEAK_TFLOPS, 2),
                        "roofline": {"bound": "mfma", "achieved": round(fl / s / 1e12, 1),
                                     "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                     "frac": round(fl / s / 1e12 / MFMA_F16_PEAK_TFLOPS, 4)}}

            # gwq_linear on layers as gwq_pack returns them (index filled at pack time), on the same layers
            # without that index (gwq_linear then builds one in its workspace on every call), and
            # gwq_linear_indexed with an index built by gwq_linear_index.
            import dataclasses
            extra["prefill_M2048"] = time_prefill([gwq.prepare_linear(P, xs[P.K], ys[j]) for j, P in enumerate(layers)])
            # The ceiling beside it: 32x32x16 FP16 MFMAs issued out of registers on every SIMD (two blocks of four
            # waves per CU), no memory, no LDS - what the matrix cores give at the clock they settle at.
            sink = torch.zeros(4, dtype=torch.int32, device=dev)
            pblocks, piters = 2 * torch.cuda.get_device_properties(dev).multi_processor_count, 4000
            pfl = gwq.probe_mfma(pblocks, piters, sink)
            settle(lambda: gwq.probe_mfma(pblocks, piters, sink), 0.2)
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(15)]
            for a, b in evs:
                a.record(); gwq.probe_mfma(pblocks, piters, sink); b.record()
            torch.cuda.synchronize()
            probe_tf = pfl / (float(np.median([a.elapsed_time(b) for a, b in evs])) * 1e-3) / 1e12
            for key in ("prefill_M2048",):
                r = extra[key]["roofline"]
                r["kernel"] = sorted({gwq.linear_plan(P, M).split(" ")[0] for P in layers})
                r["achievable"] = {"TFLOP/s": round(probe_tf, 1), "what": "register-only 32x32x16 FP16 MFMA loop on all CUs"}
                r["frac_of_achievable"] = round(r["achieved"] / probe_tf, 4)
            bare = [dataclasses.replace(P, index=None) for P in layers]
            extra["prefill_M2048_index_per_call"] = time_prefill(
                [gwq.prepare_linear(P, xs[P.K], ys[j]) for j, P in enumerate(bare)])
            indexes = [gwq.linear_index(P) for P in layers]
            extra["prefill_M2048_indexed"] = time_prefill(
                [gwq.prepare_linear(P, xs[P.K], ys[j], index=indexes[j]) for j, P in enumerate(bare)])
            del indexes, bare
            # The same seven products with FP16 weights through the vendor library (torch.matmul), for
            # scale: what a plain GEMM of these shapes reaches on this chip without any dequantisation.
            if "fp16" in legs:
                try:
                    g16 = torch.Generator(device=dev)
                    g16.manual_seed(8)
                    w16 = [(torch.randn((P.N, P.K), device=dev, generator=g16, dtype=torch.float32) * 0.02).half()
                           for P in layers]
                    lib = time_prefill([(lambda j=j, P=P: torch.matmul(xs[P.K], w16[j].t(), out=ys[j]))
                                        for j, P in enumerate(layers)])
                    fl_dense = sum(2 * M * P.N * P.K for P in layers)
                    lib["TFLOP/s"] = round(fl_dense / (lib["ms_per_pass"] * 1e-3) / 1e12, 1)
                    lib.pop("roofline"), lib.pop("pct_mfma_f16_peak")
                    lib["gwq_int4_indexed_relative_speed"] = round(
                        lib["ms_per_pass"] / extra["prefill_M2048_indexed"]["ms_per_pass"], 3)
                    extra["fp16_library_prefill_M2048"] = lib
                    del w16
                except Exception as ex:                    # the comparison must not take the benchmark down
                    extra["fp16_library_prefill_M2048"] = {"error": str(ex)[:200]}
            del xs, ys
        # The same layer packed at 3 bits (13 words per group): decode M = 1 and M = 8 the way the headline
        # is timed (grouped launches, six rotating copies, graph replay), and the prefill pass.
        if "int3" in legs and layers3:
            copies3 = [layers3] + [[clone_layer(P) for P in layers3] for _ in range(args.copies - 1)]
            int3 = {}
            for M in (1, 8):
                s, _, b, _ = decode_leg(M, max(args.steps // 3, 12), max(args.warmup // 3, 12), args.launch, args.group, copies=copies3)
                if decode_leg.median_step_ms:
                    s = decode_leg.median_step_ms * 1e-3
                int3[f"decode_M{M}"] = {"GB/s": round(b / s / 1e9, 1), "ms_per_step": round(s * 1e3, 5),
                                        "pct_hbm_peak": round(100 * b / s / 1e9 / HBM_PEAK_GBS, 2),
                                        "kernels": sorted({p.split(" ")[0] for p in decode_leg.plans})}
            if args.launch == "graph":
                int3["decode_M1_achievable"] = stream_read_leg(1, args.group, layers3)
            del copies3
            M = 2048
            xs, ys = make_xy(M)
            fl3 = sum(flops(P, M) for P in layers3)
            indexes = [gwq.linear_index(P) for P in layers3]
            calls = [gwq.prepare_linear(P, xs[P.K], ys[j], index=indexes[j]) for j, P in enumerate(layers3)]
            for _ in range(3):
                for c in calls:
                    c()
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(10):
                for c in calls:
                    c()
            torch.cuda.synchronize()
            s3 = (time.perf_counter() - t) / 10
            int3["prefill_M2048_indexed"] = {"TFLOP/s": round(fl3 / s3 / 1e12, 1), "ms_per_pass": round(s3 * 1e3, 4),
                                             "pct_mfma_f16_peak": round(100 * fl3 / s3 / 1e12 / MFMA_F16_PEAK_TFLOPS, 2)}
            int3["weight_bytes"] = sum(P.nbytes() for P in layers3)
            extra["int3"] = int3
            del indexes, calls, xs, ys
            torch.cuda.empty_cache()
        # The same layer in groups of 16 (the size Sec. 3.2 names), 32 and 64 weights, 4 bits: decode M = 1 and 16 the
        # way the headline is timed, and the prefill pass at 16.  More scales and zero points to read (3 bytes per
        # group), and the kernels multiply FP16 operands s * (q - z) instead of scaling a group's sum.
        if "beta" in legs and want_beta:
            beta = {}
            for group, lb in layers_beta.items():
                copies_b = [lb] + [[clone_layer(P) for P in lb] for _ in range(args.copies - 1)]
                row = {"weight_bytes": sum(P.nbytes() for P in lb)}
                for M in (1, 16):
                    s, _, b, _ = decode_leg(M, max(args.steps // 3, 12), max(args.warmup // 3, 12), args.launch, args.group, copies=copies_b)
                    if decode_leg.median_step_ms:
                        s = decode_leg.median_step_ms * 1e-3
                    row[f"decode_M{M}"] = {"GB/s": round(b / s / 1e9, 1), "ms_per_step": round(s * 1e3, 5),
                                           "pct_hbm_peak": round(100 * b / s / 1e9 / HBM_PEAK_GBS, 2),
                                           "kernels": sorted({p.split(" ")[0] for p in decode_leg.plans})}
                del copies_b
                if group == 16:
                    M = 2048
                    xs, ys = make_xy(M)
                    flb = sum(flops(P, M) for P in lb)
                    calls = [gwq.prepare_linear(P, xs[P.K], ys[j]) for j, P in enumerate(lb)]
                    settle(lambda: [c() for c in calls], 0.2)
                    t = time.perf_counter()
                    for _ in range(10):
                        for c in calls:
                            c()
                    torch.cuda.synchronize()
                    sb = (time.perf_counter() - t) / 10
                    row["prefill_M2048"] = {"TFLOP/s": round(flb / sb / 1e12, 1), "ms_per_pass": round(sb * 1e3, 4),
                                            "pct_mfma_f16_peak": round(100 * flb / sb / 1e12 / MFMA_F16_PEAK_TFLOPS, 2),
                                            "kernels": sorted({gwq.linear_plan(P, M).split(" ")[0] for P in lb})}
                    del calls, xs, ys
                beta[f"group_{group}"] = row
                torch.cuda.empty_cache()
            extra["int4_smaller_groups"] = beta
        # gwq_linear_bf16 on the 4-bit layer: bfloat16 activations and results.  Decode M = 1 and 16 (the kernel for any
        # M <= 16 takes these; rotating copies, one launch per matrix, replayed from a graph) and the prefill pass.
        if "bf16" in legs:
            bf = {}
            for M in (1, 16, 2048):
                xs = {K: torch.from_numpy(gs.activations(M, K, gs.rng_for(2, 100, K))).to(dev).to(torch.bfloat16) for K in (4096, 11008)}
                ys = [torch.empty((M, P.N), dtype=torch.bfloat16, device=dev) for P in layers]
                ws = [gwq.linear_workspace(P, M, dev) for P in layers]
                sets = copies if M <= 16 else copies[:1]

                def one_pass(c):
                    for j, P in enumerate(c):
                        gwq.linear_bf16(P, xs[P.K], ys[j], workspace=ws[j])
                for c in sets:
                    one_pass(c)
                torch.cuda.synchronize()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    for c in sets:
                        one_pass(c)
                settle(graph.replay, 0.2)
                ms = median_replay_ms(graph, 30) / len(sets)
                del graph
                if M <= 16:
                    b = sum(algorithmic_bytes(P, M) for P in layers)
                    bf[f"decode_M{M}"] = {"GB/s": round(b / ms / 1e6, 1), "ms_per_step": round(ms, 5),
                                          "pct_hbm_peak": round(100 * b / ms / 1e6 / HBM_PEAK_GBS, 2), "launches_per_step": 7}
                else:
                    fl = sum(flops(P, M) for P in layers)
                    bf["prefill_M2048"] = {"TFLOP/s": round(fl / ms / 1e9, 1), "ms_per_pass": round(ms, 4),
                                           "pct_mfma_bf16_peak": round(100 * fl / ms / 1e9 / MFMA_F16_PEAK_TFLOPS, 2)}
                del xs, ys, ws
            extra["bf16_activations"] = bf
            torch.cuda.empty_cache()
        # gwq_pack: score (4 B) + W (2 B) read once, packed layer written
        pk, qual = {}, {}
        for name, Wd, Sd in pack_inputs if "pack" in legs else ():
            settle(lambda: gwq.pack(Wd, Sd, 4, 10000))
            t = time.perf_counter()
            for _ in range(20):
                P = gwq.pack(Wd, Sd, 4, 10000)
            torch.cuda.synchronize()
            s = (time.perf_counter() - t) / 20
            b = Wd.numel() * 6 + P.nbytes()
            pk[name] = {"ms": round(s * 1e3, 3), "GB/s": round(b / s / 1e9, 1)}
            if name == "gate":                          # the same layer ranked by FP16 scores: two select passes, 2-byte reads
                Sh = Sd.half()
                settle(lambda: gwq.pack(Wd, Sh, 4, 10000))
                t = time.perf_counter()
                for _ in range(20):
                    Ph = gwq.pack(Wd, Sh, 4, 10000)
                torch.cuda.synchronize()
                sh = (time.perf_counter() - t) / 20
                bh = Wd.numel() * 4 + Ph.nbytes()
                pk["gate_f16_score"] = {"ms": round(sh * 1e3, 3), "GB/s": round(bh / sh / 1e9, 1)}
                del Sh, Ph
            # gwq_quality on what was just packed: W, score and the packed layer read once
            out3 = gwq.quality(P, Wd, Sd)
            settle(lambda: gwq.quality(P, Wd, Sd, out=out3))
            t = time.perf_counter()
            for _ in range(10):
                gwq.quality(P, Wd, Sd, out=out3)
            torch.cuda.synchronize()
            s = (time.perf_counter() - t) / 10
            qual[name] = {"ms": round(s * 1e3, 3), "GB/s": round(b / s / 1e9, 1),
                          "pct_hbm_peak": round(100 * b / s / 1e9 / HBM_PEAK_GBS, 1),
                          "rms_error": float((out3[0] / Wd.numel()).sqrt())}
        # decode M = 1 against the fraction of weights kept as FP16 outliers (the paper's first table, referenced
        # from Sec. 3, compares 0.1 / 0.5 / 1 % by accuracy; this is what the fraction costs the kernel): q, gate and down,
        # one launch each, six copies rotated, replayed from a graph
        if "pack" in legs and pack_inputs:
            by_ppm = {}
            for ppm in (0, 1000, 5000, 10000):
                first = [gwq.pack(Wd, Sd, 4, ppm) for _, Wd, Sd in pack_inputs]
                sets = [first] + [[clone_layer(P) for P in first] for _ in range(5)]
                xs1 = {K: torch.from_numpy(gs.activations(1, K, gs.rng_for(2, 100, K))).to(dev) for K in (4096, 11008)}
                ys1 = [torch.empty((1, P.N), dtype=torch.float16, device=dev) for P in first]
                calls = [gwq.prepare_linear(P, xs1[P.K], ys1[j]) for c in sets for j, P in enumerate(c)]
                for c in calls:
                    c()
                torch.cuda.synchronize()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    for c in calls:
                        c()
                settle(graph.replay)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(20):
                    graph.replay()
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / 20 / 6          # q + gate + down once
                b = sum(algorithmic_bytes(P, 1) for P in first)
                by_ppm[str(ppm)] = {"us_q_gate_down": round(us, 2), "GB/s": round(b / us / 1e3, 1), "bytes": b}
                del first, sets, calls, graph
                torch.cuda.empty_cache()
            extra["decode_M1_by_outlier_ppm"] = by_ppm
        # gwq_score: the weight gradient dY^T X of a layer from M = 2048 samples (what gwq_pack ranks), FP16 MFMA
        sc = {}
        for name, Wd, Sd in pack_inputs if "pack" in legs else ():
            N, K = Wd.shape
            M = 2048
            g = torch.Generator(device="cuda")
            g.manual_seed(N + K)
            dYd = (0.05 * torch.randn((M, N), device="cuda", generator=g)).half()
            Xd = torch.randn((M, K), device="cuda", generator=g).half()
            So = gwq.score(dYd, Xd)
            settle(lambda: gwq.score(dYd, Xd, out=So))
            t = time.perf_counter()
            for _ in range(10):
                gwq.score(dYd, Xd, out=So)
            torch.cuda.synchronize()
            s = (time.perf_counter() - t) / 10
            fl = 2.0 * M * N * K
            sc[name] = {"ms": round(s * 1e3, 3), "TFLOP/s": round(fl / s / 1e12, 1),
                        "pct_mfma_f16_peak": round(100 * fl / s / 1e12 / MFMA_F16_PEAK_TFLOPS, 2)}
            del dYd, Xd, So
        if pk:
            extra["pack_int4"] = pk
            extra["quality_int4"] = qual
            extra["score_M2048"] = sc
        # The linear layers of a decoder layer over 512 generated tokens, the workload of the paper's efficiency
        # table (Sec. 4.2: time to generate 512 tokens, peak memory, against FP16 on an A800): per token
        # q/k/v in one launch, o, the gated pair gate/up fused with silu and the product, down - four launches,
        # chained through their outputs (q's output stands in for the attention result; attention, norms and
        # residuals are not part of this path).  Against the same chain with FP16 weights through the vendor
        # library (seven products and the gate), both replayed from a graph of 512 steps over rotating copies.
        if "loop" in legs and args.launch == "graph":
            try:
                extra["layer_loop_512_tokens"] = layer_loop(gwq, gs, dev, torch, copies)
            except Exception as ex:                        # a comparison leg must not take the benchmark down
                extra["layer_loop_512_tokens"] = {"error": str(ex)[:300]}
        # One row per (configuration, shape, bits, M): the kernel on rotating copies (median replay) beside the
        # oracle on the host cores (all cores and one), with the parity errors of exactly that row.
        if "rows" in legs:
            extra["rows"] = result_rows(gwq, gs, dev, torch)
        out["extras"] = extra

    if not args.no_cpu_baseline:
        from oracle import gwq_oracle as orc
        name, N, K = gs.SHAPES_7B[0]
        W, S = gs.layer_matrix(2, 0, N, K)
        Pq = orc.pack(W, S, 4, 10000)
        X = gs.activations(1, K, gs.rng_for(2, 100, K))
        cores = len(os.sched_getaffinity(0))
        orc.linear_f64(Pq, X)
        reps, t = 0, time.perf_counter()
        while time.perf_counter() - t < 12.0:
            orc.linear_f64(Pq, X)
            reps += 1
        s = (time.perf_counter() - t) / reps
        b = algorithmic_bytes(layers[0], 1)
        out["cpu_baseline"] = {"value": round(b / s / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
                               "sample": f"q_proj 4096x4096 of the layer, int4, M=1, fp64 oracle linear, "
                                         f"{reps} repetitions in {s * reps:.1f} s (OpenMP over output rows)"}

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
