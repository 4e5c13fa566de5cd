#!/usr/bin/env python3
"""Benchmark of the MMM hot path on one MI355X.

A step is one pass of the whole path on device-resident inputs:
mmm_build_maps (both sides) followed by mmm_matmul.  The default workload is
the benchmark's configs[1] (M=K=N=2048 fp32, 90 % zeros in A, 90 % empty 16-wide
blocks in B).  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg1|cfg3:<i>|cfg4|cfg5]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_VECTOR_PEAK_TFLOPS = 157.3
FP32_MFMA_PEAK_TFLOPS = 157.3


def parse_workload(name):
    import mmm_synth as synth
    if name.startswith("cfg3"):       # cfg3:<i> = diagonal point i of the sweep; cfg3:<ia>:<ib> = keep index of A, of B
        f = name.split(":")
        ia = int(f[1]) if len(f) > 1 else 3
        ib = int(f[2]) if len(f) > 2 else ia
        return synth.config(3, ia, ib)
    if name == "colsparse":   # beyond the five configurations: column-structured A, MLP down-projection shape
        return synth.column_sparse(2048, 16384, 4096, 32, 0.1, 1.0, 1.0, 2001)
    return synth.config(int(name[3:]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", help="cfg1 | cfg2 | cfg3:<0..4>[:<0..4>] | cfg4 | cfg5 | colsparse")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--variant", type=int, default=-1)
    ap.add_argument("--split-k", type=int, default=0)
    ap.add_argument("--cold-sets", type=int, default=0,
                    help="also time the steps over this many separate copies of all buffers used in turn (enough "
                         "copies to exceed the 256 MB of last-level cache give the cold-cache step time)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 64 MiB device copy a few times, so that a counter run "
                         "(rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) holds a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards without communication, "
              "by rows or by block columns of C); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import mmm_synth as synth
    import paper_2402_14118_amd as mm

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    w = parse_workload(args.workload)
    esz = 4 if w.dtype == synth.DT_F32 else 2

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    if w.dtype != synth.DT_F32:
        X, Y = up(w.X_bits.view(np.int16)), up(w.Y_bits.view(np.int16))
    else:
        X, Y = up(w.X), up(w.Y)
    keep_a = None if w.keep_a is None else up(w.keep_a.view(np.int64))
    keep_rows = None if w.keep_rows is None else up(w.keep_rows.view(np.int64))
    keep_blocks = None if w.keep_blocks is None else up(w.keep_blocks.view(np.int64))
    C = torch.empty((w.M, w.N), dtype=torch.float32, device="cuda")
    eng = mm.MaskedMatmul(w.M, w.K, w.N, w.bw, w.dtype)
    mm.mmm_set_option("matmul_variant", args.variant)
    mm.mmm_set_option("split_k", args.split_k)

    def build():
        eng.build_maps(X, Y, w.pred, w.threshold, keep_a, keep_rows, keep_blocks)

    def matmul():
        eng.matmul(X, Y, C)

    build()
    matmul()
    nnz_a, occ_b, useful_macs = eng.stats()
    variant, split_k, workgroups = eng.plan()

    for _ in range(args.warmup):
        build()
        matmul()
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # timed region: exactly `steps` steps, launched back to back on the current stream
    K = args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        build()
        matmul()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3
    ms_per_step = wall_ms / K

    # the paper's protocol beside it: 10 trials of 20 steps each, median and minimum
    trials = []
    for _ in range(10):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(20):
            build()
            matmul()
        torch.cuda.synchronize()
        trials.append((time.perf_counter() - t0) * 1e3 / 20)
    trials.sort()

    # the same K steps once more with an event after every launch (events on the launch stream):
    # per-kernel durations for the roofline.  The events themselves cost several microseconds per
    # step, which is why this pass is not the one that gives the throughput.
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    torch.cuda.synchronize()
    for i in range(K):
        ev[i][0].record()
        build()
        ev[i][1].record()
        matmul()
        ev[i][2].record()
    torch.cuda.synchronize()
    build_ms = np.array([ev[i][0].elapsed_time(ev[i][1]) for i in range(K)])
    matmul_ms = np.array([ev[i][1].elapsed_time(ev[i][2]) for i in range(K)])
    t_build, t_matmul = float(build_ms.mean()), float(matmul_ms.mean())

    cold_ms = None
    if args.cold_sets > 1:
        # the same K steps over several copies of every buffer, used in turn: what the caches hold is stale
        sets = []
        for _ in range(args.cold_sets):
            e = mm.MaskedMatmul(w.M, w.K, w.N, w.bw, w.dtype)
            sets.append((e, X.clone(), Y.clone(), torch.empty_like(C),
                         None if keep_a is None else keep_a.clone(),
                         None if keep_rows is None else keep_rows.clone(),
                         None if keep_blocks is None else keep_blocks.clone()))

        def cold_step(i):
            e, Xs, Ys, Cs, ka, kr, kb = sets[i % len(sets)]
            e.build_maps(Xs, Ys, w.pred, w.threshold, ka, kr, kb)
            e.matmul(Xs, Ys, Cs)

        for i in range(len(sets)):
            cold_step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(K):
            cold_step(i)
        torch.cuda.synchronize()
        cold_ms = (time.perf_counter() - t0) * 1e3 / K
        bytes_per_set = sum(t.numel() * t.element_size() for t in sets[0][1:] if t is not None) + sets[0][0].workspace.numel()
        cold_info = {"sets": len(sets), "bytes_per_set": bytes_per_set, "ms_per_step": cold_ms}
        del sets

    useful_flops = 2.0 * useful_macs
    dense_flops = 2.0 * w.M * w.K * w.N
    value = useful_flops / (ms_per_step * 1e-3) / 1e9

    # algorithmic bytes of one launch: what the method itself must move (lists, occupied blocks, maps, C)
    WA, NB = (w.K + 63) // 64, w.N // w.bw
    WB = (NB + 63) // 64
    a_bits_b, colany_b = w.M * WA * 8, ((w.M + 31) // 32) * WA * 8
    b_bits_b, bt_b = w.K * WB * 8, NB * WA * 8
    a_blocks = ((w.M + 63) // 64) * ((w.K + 127) // 128)
    a_list_b = nnz_a * 8 + a_blocks * 4            # {slab offset, value} per non-zero, one count per block
    kb = np.ones((w.K, NB), dtype=bool)             # blocks the keep bitmaps leave switched on: the builder must read them
    if w.keep_rows is not None:
        kb &= synth.unpack_bits(w.keep_rows.reshape(1, -1), w.K)[0][:, None]
    if w.keep_blocks is not None:
        kb &= synth.unpack_bits(w.keep_blocks, NB)
    kept_blocks = int(kb.sum())
    keep_in_b = (a_bits_b if w.keep_a is not None else 0) + (b_bits_b if w.keep_blocks is not None else 0) \
        + (WA * 8 if w.keep_rows is not None else 0)
    build_bytes = w.M * w.K * esz + kept_blocks * w.bw * esz + keep_in_b \
        + a_bits_b + colany_b + a_list_b + b_bits_b + bt_b
    matmul_bytes = a_list_b + occ_b * w.bw * esz + colany_b + bt_b + w.M * w.N * 4
    dominant = "mmm_matmul_kernel" if t_matmul >= t_build else "mmm_build_kernel"
    dom_ms = max(t_matmul, t_build)
    dom_bytes = matmul_bytes if t_matmul >= t_build else build_bytes
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    traffic = None                                   # HBM bytes per launch from rocprofv3 --pmc runs, if recorded
    tfile = os.path.join(ROOT, "profiles", f"hbm_traffic_{w.name}.txt")
    if os.path.exists(tfile):
        for line in open(tfile):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == dominant:
                traffic = float(f[2])
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "algorithmic_bytes": dom_bytes, "avg_launch_us": dom_ms * 1e3,
                "build": {"avg_launch_us": t_build * 1e3, "algorithmic_bytes": build_bytes,
                          "achieved_GBs": build_bytes / (t_build * 1e-3) / 1e9},
                "matmul": {"avg_launch_us": t_matmul * 1e3, "algorithmic_bytes": matmul_bytes,
                           "achieved_GBs": matmul_bytes / (t_matmul * 1e-3) / 1e9,
                           "useful_TFLOPs": useful_flops / (t_matmul * 1e-3) / 1e12,
                           "useful_frac_of_fp32_vector_peak": useful_flops / (t_matmul * 1e-3) / 1e12 / FP32_VECTOR_PEAK_TFLOPS,
                           "mfma_TFLOPs_issued": 2.0 * w.M * occ_b * w.bw / (t_matmul * 1e-3) / 1e12,
                           "mfma_frac_of_fp32_matrix_peak": 2.0 * w.M * occ_b * w.bw / (t_matmul * 1e-3) / 1e12 / FP32_MFMA_PEAK_TFLOPS}}

    out = {
        "metric": "useful_gflops", "value": value, "unit": "GFLOP/s", "n_gpus": 1, "steps": K,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": {synth.DT_F32: "f32", synth.DT_BF16: "bf16", synth.DT_F16: "f16"}[w.dtype], "data": "synthetic",
        "config": {"workload": w.name, "M": w.M, "K": w.K, "N": w.N, "block_width": w.bw,
                   "nnz_a": nnz_a, "occupied_blocks_b": occ_b, "useful_macs": useful_macs,
                   "a_density": nnz_a / (w.M * w.K), "b_block_density": occ_b / (w.K * NB),
                   "variant": mm.mmm_matmul_variant_name(variant), "split_k": split_k, "workgroups": workgroups},
        "dense_equivalent_gflops": dense_flops / (ms_per_step * 1e-3) / 1e9,
        "t_build_us": t_build * 1e3, "t_matmul_us": t_matmul * 1e3,
        "kernel_timing": "second pass of the same steps with a HIP event after every launch",
        "trials_10x20": {"median_ms_per_step": 0.5 * (trials[4] + trials[5]), "min_ms_per_step": trials[0]},
        "roofline": roofline,
    }
    if cold_ms is not None:
        out["cold_cache"] = cold_info

    if not args.no_dense:
        # comparison point only: a dense GEMM of the materialised masked operands, same dtype
        def unpack(bits, cols):     # device bitmap [rows, words] int64 -> bool [rows, cols]
            sh = torch.arange(64, device="cuda", dtype=torch.int64)
            return (((bits.unsqueeze(-1) >> sh) & 1) != 0).reshape(bits.shape[0], -1)[:, :cols]

        torch.cuda.synchronize()
        def widen(t):     # device operand -> float32 values
            if w.dtype == synth.DT_BF16:
                return (t.to(torch.int32) << 16).view(torch.float32)
            return t.view(torch.float16).float() if w.dtype == synth.DT_F16 else t

        Xf, Yf = widen(X), widen(Y)
        A = torch.where(unpack(eng.a_bits(), w.K), Xf, torch.zeros((), device="cuda"))
        B = torch.where(unpack(eng.b_bits(), NB).repeat_interleave(w.bw, dim=1), Yf, torch.zeros((), device="cuda"))
        if w.dtype == synth.DT_BF16:
            A, B = A.bfloat16(), B.bfloat16()
        elif w.dtype == synth.DT_F16:
            A, B = A.half(), B.half()
        torch.backends.cuda.matmul.allow_tf32 = False
        for _ in range(5):
            D = torch.matmul(A, B)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(5, min(50, K))
        e0.record()
        for _ in range(reps):
            D = torch.matmul(A, B)
        e1.record()
        torch.cuda.synchronize()
        t_dense = e0.elapsed_time(e1) / reps
        out["dense_gemm_ms"] = t_dense
        out["dense_gemm_tflops"] = dense_flops / (t_dense * 1e-3) / 1e12
        out["speedup_vs_dense"] = t_dense / ms_per_step
        out["speedup_vs_dense_matmul_only"] = t_dense / t_matmul
        del A, B, D

    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: whole rows of C until about 10 s of CPU work; maps always in full
        t = time.perf_counter()
        ab = oracle.a_bits(w.X, w.pred, w.threshold, w.keep_a)
        bb = oracle.b_bits(w.Y, w.bw, w.keep_rows, w.keep_blocks)
        t_maps = time.perf_counter() - t
        probe = max(1, min(w.M, 64))
        t = time.perf_counter()
        oracle.mmm(w.X, w.Y, ab, bb, w.bw, want_mag=False, rows=(0, probe))
        t_probe = time.perf_counter() - t
        rows = int(min(w.M, max(probe, 10.0 / max(t_probe / probe, 1e-9))))

        def timed_rows(nrows, budget):   # small workloads: repeat the sample until it has run for about `budget` s
            reps, total = 0, 0.0
            while reps == 0 or (total < budget and reps < 1000):
                t = time.perf_counter()
                oracle.mmm(w.X, w.Y, ab, bb, w.bw, want_mag=False, rows=(0, nrows))
                total += time.perf_counter() - t
                reps += 1
            return total / reps, reps

        t_rows, reps = timed_rows(rows, 2.0)
        a_rows = synth.unpack_bits(ab[:rows], w.K).sum(axis=0).astype(np.int64)
        b_rows = synth.unpack_bits(bb, NB).sum(axis=1).astype(np.int64)
        macs_sample = int((a_rows * b_rows).sum()) * w.bw
        t_total = t_rows + t_maps * rows / w.M
        cores = oracle.threads()
        out["cpu_baseline"] = {"value": 2.0 * macs_sample / t_total / 1e9, "unit": "GFLOP/s",
                               "cores": cores, "kind": "oracle",
                               "sample": f"rows 0..{rows} of {w.M} (maps in full, pro-rated), {t_total * 1e3:.1f} ms per run, mean of {reps} runs",
                               "ms_per_step_extrapolated": t_total * w.M / rows * 1e3}
        # the same multiplication on one core (a smaller sample of rows)
        rows1 = max(1, rows // cores)
        oracle.set_threads(1)
        t1, reps1 = timed_rows(rows1, 2.0)
        oracle.set_threads(cores)
        a1 = synth.unpack_bits(ab[:rows1], w.K).sum(axis=0).astype(np.int64)
        out["cpu_baseline"]["one_core"] = {"value": 2.0 * int((a1 * b_rows).sum()) * w.bw / t1 / 1e9, "unit": "GFLOP/s",
                                           "sample": f"rows 0..{rows1}, multiplication only, mean of {reps1} runs"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
