#!/usr/bin/env python3
"""Benchmark of the MMM hot path on one MI355X.

A step is one pass of the whole path on device-resident inputs:
mmm_build_maps (both sides) followed by mmm_matmul.

With no --workload the run covers the sparsity sweep the metric is quoted on
(benchmark configs[2]: M=K=N=4096 fp32, the same keep fraction for the
elements of A and the 16-wide blocks of B, 0.40 ... 0.05, i.e. 60-95 % zeros;
the counterpart of the paper's Fig. 1 and of its section 4 "Varying sparsity").
`value` is the useful GFLOP/s of the point with 80 % zeros (the sparsity the
paper's headline comparison is made at); every point of the sweep is in `sweep`,
the other configurations (cfg2, cfg4, cfg5) in `others`.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W]
                  [--workload cfg1|cfg2|cfg3:<i>[:<j>]|cfg4|cfg5|colsparse]   (one workload only)
"""
import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0             # MI355X HBM3E, published
FP32_VECTOR_PEAK_TFLOPS = 157.3   # 256 CUs x 4 SIMDs x 16 lanes x 2 (packed) x 2 flops x 2.4 GHz
FP32_MFMA_PEAK_TFLOPS = 157.3
FP64_VECTOR_PEAK_TFLOPS = 78.6    # published; the pair kernel's FMAs on double inputs
BF16_MFMA_PEAK_TFLOPS = 2500.0    # dense bf16 / fp16 matrix peak, published
HEADLINE_POINT = 2                # index into the sweep: keep fraction 0.20 = 80 % zeros


def parse_workload(name):
    import mmm_synth as synth
    if name.startswith("cfg3") and not name.startswith("cfg3_f64"):       # cfg3:<i> = diagonal point i of the sweep; cfg3:<ia>:<ib> = keep index of A, of B
        f = name.split(":")
        ia = int(f[1]) if len(f) > 1 else 3
        ib = int(f[2]) if len(f) > 2 else ia
        return synth.config(3, ia, ib)
    if name == "colsparse":   # beyond the five configurations: column-structured A, MLP down-projection shape
        return synth.column_sparse(2048, 16384, 4096, 32, 0.1, 1.0, 1.0, 2001)
    if name == "cfg2_f64":    # double precision (the paper reports float and double): the shape and densities of cfg2
        return synth.random_masked(2048, 2048, 2048, 16, 0.1, 0.1, 1002, "normal", 0.0, 1.0, name="cfg2_2048_p10_bw16_f64",
                                   dtype=synth.DT_F64)
    if name.startswith("cfg3_f64"):
        ip = int(name.split(":")[1]) if ":" in name else 3
        p = synth.SWEEP_P[ip]
        return synth.random_masked(4096, 4096, 4096, 16, p, p, 3000 + 11 * ip, "uniform", -1.0, 1.0,
                                   name=f"cfg3_4096_p{int(p*100):02d}_bw16_f64", dtype=synth.DT_F64)
    if name == "colsparse_bf16":
        return synth.column_sparse(2048, 16384, 4096, 32, 0.1, 1.0, 1.0, 2001, dtype=synth.DT_BF16)
    return synth.config(int(name[3:]))


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def recorded_traffic(wname, kernel):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if there is one."""
    tfile = os.path.join(ROOT, "profiles", f"hbm_traffic_{wname}.txt")
    if os.path.exists(tfile):
        for line in open(tfile):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel:
                return float(f[2])
    return None


def measure(w, steps, warmup, args, dense=True, trials=True):
    """Time the hot path on one workload.  Returns a dict of figures (times in microseconds)."""
    import torch
    import mmm_synth as synth
    import paper_2402_14118_amd as mm

    esz = {synth.DT_F32: 4, synth.DT_F64: 8}.get(w.dtype, 2)
    csz = 8 if w.dtype == synth.DT_F64 else 4

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    if w.dtype == synth.DT_F64:
        X, Y = up(np.asarray(w.X, dtype=np.float64)), up(np.asarray(w.Y, dtype=np.float64))
    elif w.dtype != synth.DT_F32:
        X, Y = up(w.X_bits.view(np.int16)), up(w.Y_bits.view(np.int16))
    else:
        X, Y = up(w.X), up(w.Y)
    keep_a = None if w.keep_a is None else up(w.keep_a.view(np.int64))
    keep_rows = None if w.keep_rows is None else up(w.keep_rows.view(np.int64))
    keep_blocks = None if w.keep_blocks is None else up(w.keep_blocks.view(np.int64))
    C = torch.empty((w.M, w.N), dtype=torch.float64 if w.dtype == synth.DT_F64 else torch.float32, device="cuda")
    eng = mm.MaskedMatmul(w.M, w.K, w.N, w.bw, w.dtype)

    def build():
        eng.build_maps(X, Y, w.pred, w.threshold, keep_a, keep_rows, keep_blocks)

    def build_a_only():     # the B side (static weights) stays as built: section 3, rows of B are preprocessed once
        eng.build_maps(X, None, w.pred, w.threshold, keep_a, None, None)

    def matmul():
        eng.matmul(X, Y, C)

    build()
    matmul()
    nnz_a, occ_b, useful_macs = eng.stats()     # also gives the library its density estimate for the choice of kernel
    variant, split_k, workgroups = eng.plan()
    path = eng.path()

    for _ in range(warmup):
        build()
        matmul()
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # timed region: exactly `steps` steps, launched back to back on the current stream
    K = steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        build()
        matmul()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / K

    # the same with the B side cached: only the A side is rebuilt in a step
    for _ in range(min(warmup, 5)):
        build_a_only()
        matmul()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        build_a_only()
        matmul()
    torch.cuda.synchronize()
    ms_cached = (time.perf_counter() - t0) * 1e3 / K

    # and with the A mask evaluated inside the multiplication (one launch per step, B side cached)
    for _ in range(min(warmup, 5)):
        eng.matmul_fused(X, Y, C, w.pred, w.threshold, keep_a)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        eng.matmul_fused(X, Y, C, w.pred, w.threshold, keep_a)
    torch.cuda.synchronize()
    ms_fused = (time.perf_counter() - t0) * 1e3 / K

    out_trials = None
    if trials:   # the paper's protocol beside it: 10 trials of 20 steps each, median and minimum
        tr = []
        for _ in range(10):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(20):
                build()
                matmul()
            torch.cuda.synchronize()
            tr.append((time.perf_counter() - t0) * 1e3 / 20)
        tr.sort()
        out_trials = {"median_ms_per_step": 0.5 * (tr[4] + tr[5]), "min_ms_per_step": tr[0]}

    # the same K steps once more with an event after every launch (events on the launch stream):
    # per-kernel durations for the roofline.  The events themselves cost a few microseconds per
    # step, which is why this pass is not the one that gives the throughput.
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K)]
    torch.cuda.synchronize()
    for i in range(K):
        ev[i][0].record()
        build()
        ev[i][1].record()
        matmul()
        ev[i][2].record()
        build_a_only()
        ev[i][3].record()
    torch.cuda.synchronize()
    t_build = float(np.mean([ev[i][0].elapsed_time(ev[i][1]) for i in range(K)]))
    t_matmul = float(np.mean([ev[i][1].elapsed_time(ev[i][2]) for i in range(K)]))
    t_build_a = float(np.mean([ev[i][2].elapsed_time(ev[i][3]) for i in range(K)]))
    del ev

    cold_info = None
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
    # matrix path: every occupied block of B against all rows of A; pair path: the surviving products only
    issued_flops = 2.0 * w.M * occ_b * w.bw if path == mm.MMM_PATH_MATRIX else useful_flops

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
    del kb
    keep_in_b = (a_bits_b if w.keep_a is not None else 0) + (b_bits_b if w.keep_blocks is not None else 0) \
        + (WA * 8 if w.keep_rows is not None else 0)
    build_bytes = w.M * w.K * esz + kept_blocks * w.bw * esz + keep_in_b \
        + a_bits_b + colany_b + a_list_b + b_bits_b + bt_b
    if path == mm.MMM_PATH_MATRIX:   # lists of A, occupied blocks of Y, the two small maps, C
        matmul_bytes = a_list_b + occ_b * w.bw * esz + colany_b + bt_b + w.M * w.N * csz
    else:                            # pair kernel: the non-zero elements of X, both bitmaps, occupied blocks of Y, C
        matmul_bytes = nnz_a * esz + a_bits_b + bt_b + occ_b * w.bw * esz + w.M * w.N * csz

    # arithmetic peak the multiplication is priced against: fp32 inputs run on fp32 units (vector FMA and the fp32
    # matrix instruction share one peak); 16-bit inputs on the matrix path run on the 16-bit matrix instructions
    mfma16 = w.dtype != synth.DT_F32 and path == mm.MMM_PATH_MATRIX
    arith_peak, arith_name = (BF16_MFMA_PEAK_TFLOPS, "mfma") if mfma16 else (FP32_VECTOR_PEAK_TFLOPS, "alu")
    if w.dtype == synth.DT_F64:
        arith_peak = FP64_VECTOR_PEAK_TFLOPS

    def floors(nbytes, flops, t_ms):
        """Roofline of one kernel: the floor is the larger of the time its algorithmic bytes need at the HBM peak
        and the time its useful flops need at the arithmetic peak."""
        t_hbm = nbytes / (HBM_PEAK_GBS * 1e9) * 1e6
        t_alu = flops / (arith_peak * 1e12) * 1e6
        t_us = t_ms * 1e3
        bound = arith_name if t_alu > t_hbm else "hbm"
        r = {"avg_launch_us": t_us, "algorithmic_bytes": nbytes, "useful_flops": flops,
             "t_hbm_floor_us": t_hbm, "t_alu_floor_us": t_alu, "bound": bound,
             "frac_hbm": t_hbm / t_us, "frac_alu": t_alu / t_us, "frac": max(t_hbm, t_alu) / t_us,
             "achieved_GBs": nbytes / (t_us * 1e-6) / 1e9, "achieved_TFLOPs": flops / (t_us * 1e-6) / 1e12}
        return r

    rb = floors(build_bytes, 0.0, t_build)
    rm = floors(matmul_bytes, useful_flops, t_matmul)
    rm["issued_TFLOPs"] = issued_flops / (t_matmul * 1e-3) / 1e12
    rm["issued_frac_of_arith_peak"] = rm["issued_TFLOPs"] / arith_peak
    rm["arith_peak_TFLOPs"] = arith_peak
    rm["useful_over_issued"] = useful_flops / issued_flops if issued_flops else None
    mm_kernel = "mmm_matmul_kernel" if path == mm.MMM_PATH_MATRIX else "mmm_pairs_kernel"
    dom_name, dom = (mm_kernel, rm) if t_matmul >= t_build else ("mmm_build_kernel", rb)
    if dom["bound"] != "hbm":
        roofline = {"bound": dom["bound"], "achieved": dom["achieved_TFLOPs"], "peak": arith_peak, "unit": "TFLOP/s"}
    else:
        roofline = {"bound": "hbm", "achieved": dom["achieved_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    roofline.update({"frac": dom["frac"], "traffic": recorded_traffic(w.name, dom_name),
                     "traffic_source": "profiles/hbm_traffic_%s.txt (rocprofv3 --pmc, recorded earlier)" % w.name,
                     "kernel": dom_name, "build": rb, "matmul": rm})

    row = {
        "workload": w.name, "M": w.M, "K": w.K, "N": w.N, "block_width": w.bw,
        "dtype": {synth.DT_F32: "f32", synth.DT_BF16: "bf16", synth.DT_F16: "f16", synth.DT_F64: "f64"}[w.dtype],
        "nnz_a": nnz_a, "occupied_blocks_b": occ_b, "useful_macs": useful_macs,
        "a_density": nnz_a / (w.M * w.K), "b_block_density": occ_b / (w.K * NB),
        "path": "matrix" if path == mm.MMM_PATH_MATRIX else "pairs",
        "variant": mm.mmm_matmul_variant_name(variant) if path == mm.MMM_PATH_MATRIX else None,
        "split_k": split_k if path == mm.MMM_PATH_MATRIX else None, "workgroups": workgroups,
        "steps": K, "step_us": ms_per_step * 1e3, "build_us": t_build * 1e3, "matmul_us": t_matmul * 1e3,
        "useful_gflops": useful_flops / (ms_per_step * 1e-3) / 1e9,
        "useful_gflops_matmul_only": useful_flops / (t_matmul * 1e-3) / 1e9,
        "dense_equivalent_gflops": dense_flops / (ms_per_step * 1e-3) / 1e9,
        "dense_equivalent_gflops_matmul_only": dense_flops / (t_matmul * 1e-3) / 1e9,
        "cached_b": {"step_us": ms_cached * 1e3, "build_a_us": t_build_a * 1e3,
                     "useful_gflops": useful_flops / (ms_cached * 1e-3) / 1e9,
                     "fused_step_us": ms_fused * 1e3},
        "roofline": roofline,
    }
    if out_trials:
        row["trials_10x20"] = out_trials
    if cold_info:
        row["cold_cache"] = cold_info

    if dense:
        # comparison point only: a dense GEMM of the materialised masked operands, same dtype
        def unpack(bits, cols):     # device bitmap [rows, words] int64 -> bool [rows, cols]
            sh = torch.arange(64, device="cuda", dtype=torch.int64)
            return (((bits.unsqueeze(-1) >> sh) & 1) != 0).reshape(bits.shape[0], -1)[:, :cols]

        def widen(t):     # device operand -> float32 values
            if w.dtype == synth.DT_BF16:
                return (t.to(torch.int32) << 16).view(torch.float32)
            return t.view(torch.float16).float() if w.dtype == synth.DT_F16 else t     # f32 and f64 as they are

        torch.cuda.synchronize()
        zero = torch.zeros((), device="cuda", dtype=torch.float64 if w.dtype == synth.DT_F64 else torch.float32)
        A = torch.where(unpack(eng.a_bits(), w.K), widen(X), zero)
        B = torch.where(unpack(eng.b_bits(), NB).repeat_interleave(w.bw, dim=1), widen(Y), zero)
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
        row["dense_gemm_us"] = t_dense * 1e3
        row["dense_gemm_tflops"] = dense_flops / (t_dense * 1e-3) / 1e12
        row["speedup_vs_dense"] = t_dense / ms_per_step
        row["speedup_vs_dense_matmul_only"] = t_dense / t_matmul
        row["cached_b"]["speedup_vs_dense"] = t_dense / ms_cached
        row["cached_b"]["fused_speedup_vs_dense"] = t_dense / ms_fused
        del A, B, D
    eng.close()
    del eng, X, Y, C, keep_a, keep_rows, keep_blocks
    gc.collect()
    torch.cuda.empty_cache()
    return row


def cpu_baseline(w):
    """The oracle as it stands on the host cores, on a bounded sample (whole rows of C for about 10 s of work)."""
    import mmm_synth as synth
    import oracle
    NB = w.N // w.bw
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

    t_rows, reps = timed_rows(rows, 10.0)
    a_rows = synth.unpack_bits(ab[:rows], w.K).sum(axis=0).astype(np.int64)
    b_rows = synth.unpack_bits(bb, NB).sum(axis=1).astype(np.int64)
    macs_sample = int((a_rows * b_rows).sum()) * w.bw
    t_total = t_rows + t_maps * rows / w.M
    cores = oracle.threads()
    out = {"value": 2.0 * macs_sample / t_total / 1e9, "unit": "GFLOP/s", "cores": cores, "cpu_model": cpu_model(),
           "host_cpus": os.cpu_count(), "kind": "oracle", "workload": w.name,
           "sample": f"rows 0..{rows} of {w.M} (maps in full, pro-rated), {t_total * 1e3:.1f} ms per run, "
                     f"mean of {reps} runs",
           "ms_per_step_extrapolated": t_total * w.M / rows * 1e3}
    rows1 = max(1, rows // cores)     # the same multiplication on one core (a smaller sample of rows)
    oracle.set_threads(1)
    t1, reps1 = timed_rows(rows1, 3.0)
    oracle.set_threads(cores)
    a1 = synth.unpack_bits(ab[:rows1], w.K).sum(axis=0).astype(np.int64)
    out["one_core"] = {"value": 2.0 * int((a1 * b_rows).sum()) * w.bw / t1 / 1e9, "unit": "GFLOP/s",
                       "sample": f"rows 0..{rows1}, multiplication only, mean of {reps1} runs"}
    return out


SLIM_KEYS = ("workload", "a_density", "b_block_density", "path", "variant", "split_k", "step_us", "build_us", "matmul_us",
             "useful_gflops", "useful_gflops_matmul_only", "dense_equivalent_gflops", "dense_gemm_us",
             "speedup_vs_dense", "speedup_vs_dense_matmul_only", "cached_b", "roofline")


def slim(row):
    return {k: row[k] for k in SLIM_KEYS if k in row}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None,
                    help="one workload only: cfg1 | cfg2 | cfg3:<0..4>[:<0..4>] | cfg4 | cfg5 | colsparse | colsparse_bf16 | "
                         "cfg2_f64 | cfg3_f64:<0..4> "
                         "(default: the cfg3 sweep, then cfg2, cfg4 and cfg5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="sweep only: skip cfg2, cfg4 and cfg5")
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
    mm.mmm_set_option("matmul_variant", args.variant)
    mm.mmm_set_option("split_k", args.split_k)
    K, W = args.steps, args.warmup

    sweep, others = None, None
    if args.workload is not None:
        w = parse_workload(args.workload)
        head = measure(w, K, W, args, dense=not args.no_dense)
        label = w.name
    else:
        sweep, w = [], None
        for ip in range(len(synth.SWEEP_P)):
            wi = synth.config(3, ip)
            print(f"bench: {wi.name}", file=sys.stderr, flush=True)
            row = measure(wi, K, W, args, dense=not args.no_dense, trials=(ip == HEADLINE_POINT))
            row["keep_fraction"] = synth.SWEEP_P[ip]
            sweep.append(row)
            if ip == HEADLINE_POINT:
                w = wi
            del wi
        head = sweep[HEADLINE_POINT]
        label = "cfg3 sweep M=K=N=4096 fp32 bw16, keep fraction of A elements = of B blocks in " \
                "{.40,.30,.20,.10,.05}; value = the point with 80 %% zeros (%s)" % head["workload"]
        if not args.no_others:
            others = {}
            for name in ("cfg2", "cfg4", "cfg5"):
                wo = parse_workload(name)
                print(f"bench: {wo.name}", file=sys.stderr, flush=True)
                others[name] = slim(measure(wo, K, W, args, dense=not args.no_dense, trials=False))
                del wo

    out = {
        "metric": "useful_gflops", "value": head["useful_gflops"], "unit": "GFLOP/s", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": head["step_us"] * 1e-3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": label, "M": head["M"], "K": head["K"], "N": head["N"], "block_width": head["block_width"],
                   "nnz_a": head["nnz_a"], "occupied_blocks_b": head["occupied_blocks_b"],
                   "useful_macs": head["useful_macs"], "a_density": head["a_density"],
                   "b_block_density": head["b_block_density"], "path": head["path"], "variant": head["variant"],
                   "split_k": head["split_k"], "workgroups": head["workgroups"]},
        "step": "mmm_build_maps (both sides) + mmm_matmul; cached_b.step_us = the A side only + mmm_matmul; "
                "cached_b.fused_step_us = mmm_matmul_fused alone (A mask evaluated inside the multiplication)",
        "dense_equivalent_gflops": head["dense_equivalent_gflops"],
        "t_build_us": head["build_us"], "t_matmul_us": head["matmul_us"],
        "kernel_timing": "second pass of the same steps with a HIP event after every launch",
        "cached_b": head["cached_b"],
        "roofline": head["roofline"],
    }
    for k in ("trials_10x20", "cold_cache", "dense_gemm_us", "dense_gemm_tflops", "speedup_vs_dense",
              "speedup_vs_dense_matmul_only"):
        if k in head:
            out[k] = head[k]
    if sweep is not None:
        out["sweep"] = [dict(slim(r), keep_fraction=r["keep_fraction"]) for r in sweep]
    if others is not None:
        out["others"] = others
    if not args.no_cpu_baseline:
        print("bench: cpu baseline", file=sys.stderr, flush=True)
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
