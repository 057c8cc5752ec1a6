#!/usr/bin/env python3
"""Benchmark of the 2:4 sparse matrix-multiply hot path on one MI355X.

The line is for the large int8 product (8192 x 8192 x 8192, `square_i8`) unless
--workload names another; the other configurations follow as extra keys of the
same line (`other_workloads`: kernels back to back and the vendor's dense
product only).

A step is one pass of the whole path over one batch of synthetic input:
prune -> compress (tiled layout) -> decompress -> sparse product -> same-shape
dense product.  All inputs are resident in HBM before the timed region; every
step works on the next of several rotating copies of the inputs so that the
footprint of the loop exceeds the 256 MB last-level cache.

Prints one JSON line.  `value` is the metric: dense-equivalent TFLOP/s of the
sparse product, 2*M*N*K divided by its mean duration, measured with HIP events
on the launch stream: the whole-path steps give `ms_per_step` (wall time of a
step) and `step_ms` (event pair around every launch), and every operation is
then timed as back-to-back launches on the same rotating inputs
(`kernel_ms_back_to_back`: five batches, the median), which is the duration
`value`, the speedups and `roofline` use; `kernel_ms_cache_warm` is the
same on one input set (operands resident in the last-level cache), for
comparison only.  `speedup_vs_dense` is over the faster of the own dense kernel
and the vendor library's dense product on the same inputs (both ratios are
kept beside it).  `roofline` describes the sparse product kernel (`traffic`
is read from the counter sections of profiles/<workload>_path_rocprofv3.txt),
`cpu_baseline` the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published peaks: dense matrix cores per input type, and HBM3E
PEAK_DENSE = {"f16": 2.5e15, "bf16": 2.5e15, "i8": 5.0e15}
PEAK_HBM = 8.0e12

# dense-equivalent op/s of v_smfmac_*_32x32 in a register-only loop on all compute units, random operands (sp24_probe)
MEASURED_SPARSE_ISSUE = {"f16": 3.105e15, "bf16": 3.221e15, "i8": 6.656e15}



def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=3)
    p.add_argument("--workload", default="square_i8",
                   help="tiny_f16 | ffn_bf16 | conv3x3_f16 | square_i8 | skinny_bf16: the workload of the line "
                        "(default: the large int8 product the target is stated on); the others follow under `other_workloads`")
    p.add_argument("--no-others", action="store_true", help="the one workload only (profiling aid)")
    p.add_argument("--cpu-seconds", type=float, default=10.0, help="budget of the CPU-oracle leg (0 = skip)")
    p.add_argument("--only", default="", help="comma list of ops to run in a step (profiling aid); default all")
    p.add_argument("--materialised", action="store_true",
                   help="conv3x3_f16 only: multiply by the im2col matrix built beforehand instead of gathering it implicitly")
    p.add_argument("--extras", action="store_true",
                   help="also time the operations beyond the five-step path on this workload's operands: the retraining "
                        "support (mask apply, fixed-mask compress, row-and-column pruning) and, for int8, the product "
                        "with the quantised path's epilogue; each beside the CPU oracle on a sample")
    p.add_argument("--sweep", action="store_true",
                   help="add the counterpart of the paper's speedup plot (Sec. 3.2, Fig. 3): M = N = 8192, the inner dimension "
                        "swept, sparse product against the own and the vendor's dense product (bf16 and int8 workloads)")
    p.add_argument("--few-tiles", action="store_true",
                   help="add products with few output tiles (32 < N <= 128 at large M and K; small M x N with a long K) in this "
                        "workload's types: as they are and with the inner dimension split across workgroups")
    p.add_argument("--operand-dependence", action="store_true",
                   help="add the workload's products on operands of other values (zeros, ones, values near zero): the share of "
                        "the time that depends on the data through the power cap (ffn_bf16 and square_i8)")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run one 1 GiB device copy, so that a counter profile of this run holds a kernel of known traffic")
    return p.parse_args()


def cpu_baseline(name, A, Bt, budget_s):
    """The oracle as it stands, on a bounded sample: compress + decompress + triple-loop product of the first
    rows of A with the first columns of B (all of K)."""
    import numpy as np
    import oracle
    from paper_2104_08378_amd import synth
    w = synth.WORKLOADS[name]
    dt, K = w["dtype"], w["K"]
    rows, cols = 32, min(w["N"], 1024)

    def run(r, c):
        As = np.ascontiguousarray(A[:r])
        Bs = np.ascontiguousarray(Bt[:c].T)
        t0 = time.perf_counter()
        V, meta = oracle.compress(As, dt)
        P = oracle.decompress(V, meta, dt)
        oracle.gemm(P, Bs, dt)
        return time.perf_counter() - t0

    t = run(rows, cols)
    for _ in range(3):                                       # grow the sample towards the budget: rows first, then columns of B
        grow = min(16.0, budget_s / max(t, 1e-3))
        if grow < 1.5:
            break
        if rows < w["M"]:
            rows = int(min(w["M"], rows * grow)) // 32 * 32
        elif cols < w["N"]:
            cols = int(min(w["N"], cols * grow)) // 64 * 64
        else:
            break
        t = run(rows, cols)
    cores = oracle.threads()
    # the same on one thread, on a sample cut down by the thread count
    rows1 = max(32, rows // max(cores, 1) // 32 * 32)
    before = oracle.set_threads(1)
    t1 = run(rows1, cols)
    oracle.set_threads(before)
    return {"value": 2.0 * rows * cols * K / t / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"first {rows} rows of A x first {cols} columns of B, K={K}: compress + decompress + "
                      f"{'int32' if dt == 'i8' else 'fp64'} triple loop, {t:.1f} s",
            "value_one_thread": 2.0 * rows1 * cols * K / t1 / 1e12,
            "sample_one_thread": f"first {rows1} rows, {t1:.1f} s"}


def extras(name, As, Bs, V, meta, P, D, Dd, out_dt, A_host, steps, conv):
    """Back-to-back timings of the operations outside the five-step path, each with its algorithmic bytes against
    the HBM peak (or, for the scaled product, dense-equivalent op/s), and the oracle's time on the first rows."""
    import numpy as np
    import oracle
    import torch
    from paper_2104_08378_amd import sp24, synth
    w = synth.WORKLOADS[name]
    dt, M, K, N = w["dtype"], w["M"], w["K"], w["N"]
    es = 1 if dt == "i8" else 2
    R = len(As)

    def timed(fn):
        for i in range(3):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(steps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps * 1e-3

    rows = min(M, 512)
    sample = np.ascontiguousarray(A_host[:rows])
    _, smeta = oracle.compress(sample, dt)

    def cpu(fn):
        t0 = time.perf_counter()
        fn()
        return (time.perf_counter() - t0) * M / rows       # scaled from `rows` rows to the whole matrix

    # outputs rotate like the inputs (a fixed output buffer would stay in the last-level cache from launch to launch)
    Pms = [torch.empty_like(As[0]) for _ in range(R)]
    Vms = [torch.empty_like(V) for _ in range(R)]
    perm_h = np.random.default_rng(0).permutation(K).astype(np.int32)
    perm_d = torch.from_numpy(perm_h).cuda()
    rperm_d = torch.from_numpy(np.random.default_rng(1).permutation(M).astype(np.int32)).cuda()
    total = torch.empty(1, dtype=torch.float64, device="cuda")
    out = {}
    ops = {
        "mask_apply": (lambda i: sp24.sp24_mask_apply(As[i % R], meta, layout="tiled", out=Pms[i % R]), 2.0 * M * K * es + M * K / 8,
                       lambda: oracle.mask_apply(sample, smeta, dt)),
        "compress_masked": (lambda i: sp24.sp24_compress_masked(As[i % R], meta, layout="tiled", out=Vms[i % R]), 1.5 * M * K * es + M * K / 8,
                            lambda: oracle.compress_masked(sample, smeta, dt)),
        "prune_transposable": (lambda i: sp24.sp24_prune_transposable(As[i % R], out=Pms[i % R]), 2.0 * M * K * es,
                               lambda: oracle.prune_transposable(sample, dt)),
        # channel permutations: the gather reads and writes the matrix once, the figure of merit reads it once
        "permute_columns": (lambda i: sp24.sp24_permute_columns(As[i % R], perm_d, out=Pms[i % R]), 2.0 * M * K * es + 4.0 * K,
                            lambda: oracle.permute_columns(sample, perm_h, dt)),
        "retained_magnitude": (lambda i: sp24.sp24_retained_magnitude(As[i % R], perm_d, out=total), 1.0 * M * K * es + 4.0 * K,
                               lambda: oracle.retained_magnitude(sample, dt, perm=perm_h)),
        "retained_magnitude_given_order": (lambda i: sp24.sp24_retained_magnitude(As[i % R], out=total), 1.0 * M * K * es,
                                           lambda: oracle.retained_magnitude(sample, dt)),
        "permute_rows": (lambda i: sp24.sp24_permute_rows(As[i % R], rperm_d, out=Pms[i % R]), 2.0 * M * K * es + 4.0 * M,
                         lambda: oracle.permute_rows(sample, np.random.default_rng(1).permutation(rows).astype(np.int32), dt)),
    }
    for op, (fn, nbytes, cfn) in ops.items():
        t = timed(fn)
        out[op] = {"us": t * 1e6, "GBps": nbytes / t / 1e9, "frac_of_hbm_peak": nbytes / t / PEAK_HBM,
                   "cpu_oracle_us_scaled_from_%d_rows" % rows: cpu(cfn) * 1e6}
    # the search for a column order (one sweep from the columns as they are): time of the sweep, what it gains in
    # retained magnitude, and the oracle's sweep on the first rows scaled to the whole matrix
    perm_s = torch.arange(K, dtype=torch.int32, device="cuda")
    sp24.sp24_permute_search(As[0], sweeps=1, perm=perm_s.clone())          # warm-up
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    sp24.sp24_permute_search(As[0], sweeps=1, perm=perm_s)
    e1.record()
    torch.cuda.synchronize()
    srows = min(M, 64)
    ssample = np.ascontiguousarray(A_host[:srows])
    t0 = time.perf_counter()
    oracle.permute_search(ssample, dt, sweeps=1)
    t_cpu = (time.perf_counter() - t0) * M / srows
    rounds = max(1, int(np.ceil(np.log2(K // 4))))
    out["permute_search_one_sweep"] = {
        "us": e0.elapsed_time(e1) * 1e3, "rounds": rounds,
        "GBps_one_read_of_A_per_round": rounds * 1.0 * M * K * es / (e0.elapsed_time(e1) * 1e-3) / 1e9,
        "retained_magnitude_before": float(sp24.sp24_retained_magnitude(As[0]).cpu()[0]),
        "retained_magnitude_after": float(sp24.sp24_retained_magnitude(As[0], perm_s).cpu()[0]),
        "cpu_oracle_us_scaled_from_%d_rows" % srows: t_cpu * 1e6}
    if dt == "i8" and not conv:
        ws = torch.full((M,), 1.0e-3, dtype=torch.float32, device="cuda")
        bs = torch.zeros(M, dtype=torch.float32, device="cuda")
        D8, D8d = torch.empty((M, N), dtype=torch.int8, device="cuda"), torch.empty((M, N), dtype=torch.int8, device="cuda")
        ts = timed(lambda i: sp24.sp24_spmm_i8_scaled(V, meta, Bs[i % R], torch.int8, ws, 0.02, bs, True, 30.0, layout="tiled", out=D8))
        td = timed(lambda i: sp24.sp24_gemm_dense_i8_scaled(P, Bs[i % R], torch.int8, ws, 0.02, bs, True, 30.0, out=D8d))
        out["spmm_i8_scaled_int8_out"] = {"us": ts * 1e6, "dense_us": td * 1e6, "speedup_vs_dense": td / ts,
                                          "dense_equiv_Tops": 2.0 * M * N * K / ts / 1e12,
                                          "frac_of_sparse_peak": M * N * K / ts / PEAK_DENSE[dt]}
        # the same shape on 8-bit floats (4 exponent, 3 fraction bits): operands N(0, 0.5) and N(0, 1) rounded to the
        # type, fp32 accumulation, bf16 output; against the chip's dense fp8 matrix-core peak (5.0 PFLOP/s)
        f8 = torch.float8_e4m3fn
        A8s = [(torch.randn((M, K), device="cuda") * 0.5).to(f8) for _ in range(2)]
        B8s = [torch.randn((N, K), device="cuda").to(f8) for _ in range(R)]
        VM8 = [sp24.sp24_compress(a_, layout="tiled") for a_ in A8s]
        P8 = [sp24.sp24_prune(a_) for a_ in A8s]
        Df8 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        ts = timed(lambda i: sp24.sp24_spmm(VM8[i % 2][0], VM8[i % 2][1], B8s[i % R], torch.bfloat16, layout="tiled", out=Df8))
        td = timed(lambda i: sp24.sp24_gemm_dense(P8[i % 2], B8s[i % R], torch.bfloat16, out=Df8))
        out["spmm_f8_bf16_out"] = {"us": ts * 1e6, "dense_us": td * 1e6, "speedup_vs_dense": td / ts,
                                   "dense_equiv_Tflops": 2.0 * M * N * K / ts / 1e12,
                                   "frac_of_sparse_peak": M * N * K / ts / 5.0e15}
        del A8s, B8s, VM8, P8, Df8
    return out


def sweep(name, steps):
    """Sparse against dense over the inner dimension at M = N = 8192 (the paper's Fig. 3 plots the speedup over GEMM-K
    for large M and N).  Inputs drawn on the device with torch's seeded generator, same distributions as the workload;
    enough rotating sets that the operands do not stay in the last-level cache."""
    import torch
    from paper_2104_08378_amd import sp24, synth
    from paper_2104_08378_amd.bits import OUT_DT
    w = synth.WORKLOADS[name]
    dt, out_dt = w["dtype"], OUT_DT[w["out"]]
    M = N = 8192
    gen = torch.Generator(device="cuda").manual_seed(0)

    def draw(rows, cols, sigma):
        if dt == "i8":
            return torch.randint(-127, 128, (rows, cols), dtype=torch.int8, device="cuda", generator=gen)
        x = torch.randn((rows, cols), dtype=torch.float32, device="cuda", generator=gen) * sigma
        return x.to(torch.bfloat16 if dt == "bf16" else torch.float16)

    def timed(fn):
        for i in range(5):
            fn(i)
        batches = []
        for rep in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for i in range(steps):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            batches.append(e0.elapsed_time(e1) / steps)
        return sorted(batches)[1] * 1e-3

    rows = []
    for K in (512, 1024, 2048, 4096, 8192, 16384):
        es = 1 if dt == "i8" else 2
        R = max(2, min(24, int(600e6 // ((M + N) * K * es)) + 1))
        As = [draw(M, K, 0.02) for _ in range(R)]
        Bs = [draw(N, K, 1.0) for _ in range(R)]
        VM = [sp24.sp24_compress(a, layout="tiled") for a in As]
        Ps = [sp24.sp24_prune(a) for a in As]
        D = torch.empty((M, N), dtype=out_dt, device="cuda")
        t_sp = timed(lambda i: sp24.sp24_spmm(VM[i % R][0], VM[i % R][1], Bs[i % R], out_dt, layout="tiled", out=D))
        t_dn = timed(lambda i: sp24.sp24_gemm_dense(Ps[i % R], Bs[i % R], out_dt, out=D))
        mm = (lambda a, b: torch._int_mm(a, b.t())) if dt == "i8" else (lambda a, b: torch.matmul(a, b.t()))
        t_v = timed(lambda i: mm(Ps[i % R], Bs[i % R]))
        rows.append({"K": K, "sparse_us": t_sp * 1e6, "dense_us": t_dn * 1e6, "vendor_dense_us": t_v * 1e6,
                     "speedup_vs_dense": t_dn / t_sp, "speedup_vs_vendor_dense": t_v / t_sp,
                     "sparse_dense_equiv_Tops": 2.0 * M * N * K / t_sp / 1e12})
        del As, Bs, VM, Ps, D
        torch.cuda.empty_cache()
    return {"M": M, "N": N, "rows": rows}


def few_tiles(name, steps):
    """Products with few output tiles -- 32 < N <= 128 at large M and K, small M x N with a long K, N <= 32 with few rows or with
    very many (a transformer's projections on a batch of 8 - 64 tokens, the last one onto 32000 outputs): the sparse
    and the dense product as they are, and with the inner dimension split across workgroups (partial products in a
    workspace, second kernel adds them), beside the vendor library's dense product.  Inputs as in sweep()."""
    import torch
    from paper_2104_08378_amd import sp24, synth
    from paper_2104_08378_amd.bits import OUT_DT
    w = synth.WORKLOADS[name]
    dt, out_dt = w["dtype"], OUT_DT[w["out"]]
    gen = torch.Generator(device="cuda").manual_seed(0)
    tdt = {"i8": torch.int8, "bf16": torch.bfloat16, "f16": torch.float16}[dt]

    def draw(rows, cols, sigma):
        if dt == "i8":
            return torch.randint(-127, 128, (rows, cols), dtype=torch.int8, device="cuda", generator=gen)
        return (torch.randn((rows, cols), dtype=torch.float32, device="cuda", generator=gen) * sigma).to(tdt)

    def timed(fn):
        for i in range(5):
            fn(i)
        batches = []
        for rep in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for i in range(steps):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            batches.append(e0.elapsed_time(e1) / steps)
        return sorted(batches)[1] * 1e3

    rows = []
    for M, N, K in ((8192, 64, 8192), (8192, 128, 8192), (512, 512, 8192), (256, 256, 16384), (2048, 256, 4096),
                    (4096, 16, 16384), (512, 32, 16384), (4096, 64, 4096), (11008, 32, 4096), (32000, 8, 4096)):
        es = 1 if dt == "i8" else 2
        R = max(2, min(24, int(600e6 // ((M + N) * K * es)) + 1))
        As = [draw(M, K, 0.02) for _ in range(R)]
        Bs = [draw(N, K, 1.0) for _ in range(R)]
        VM = [sp24.sp24_compress(a, layout="tiled") for a in As]
        Ps = [sp24.sp24_prune(a) for a in As]
        D = torch.empty((M, N), dtype=out_dt, device="cuda")
        need = sp24.sp24_splitk_workspace_bytes(M, N, K, tdt)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        t_sp = timed(lambda i: sp24.sp24_spmm(VM[i % R][0], VM[i % R][1], Bs[i % R], out_dt, layout="tiled", out=D))
        t_sps = timed(lambda i: sp24.sp24_spmm_splitk(VM[i % R][0], VM[i % R][1], Bs[i % R], out_dt, layout="tiled", workspace=ws, out=D))
        t_dn = timed(lambda i: sp24.sp24_gemm_dense(Ps[i % R], Bs[i % R], out_dt, out=D))
        t_dns = timed(lambda i: sp24.sp24_gemm_dense_splitk(Ps[i % R], Bs[i % R], out_dt, workspace=ws, out=D))
        mm = (lambda a, b: torch._int_mm(a, b.t())) if dt == "i8" else (lambda a, b: torch.matmul(a, b.t()))
        t_v = timed(lambda i: mm(Ps[i % R], Bs[i % R]))
        rows.append({"M": M, "N": N, "K": K, "workspace_MiB": need / 2 ** 20, "sparse_us": t_sp, "sparse_split_us": t_sps,
                     "dense_us": t_dn, "dense_split_us": t_dns, "vendor_dense_us": t_v})
        del As, Bs, VM, Ps, D, ws
        torch.cuda.empty_cache()
    return rows


def operand_dependence(name, steps):
    """The workload's sparse and dense product, and the vendor library's dense product, on operands of other
    values -- same shapes, kernels and bytes: all zeros, all ones, and values concentrated near zero (a normal
    distribution with a tenth of the workload's spread; for int8, sigma = 12).  What changes is how many bits toggle
    in the data paths, hence the clock the power cap allows.  The pattern of A is the workload's own in every row."""
    import torch
    from paper_2104_08378_amd import sp24, synth
    from paper_2104_08378_amd.bits import OUT_DT, to_gpu
    w = synth.WORKLOADS[name]
    dt, M, K, N, out_dt = w["dtype"], w["M"], w["K"], w["N"], OUT_DT[w["out"]]
    A, Bt = synth.make(name)
    Ad, Bd = to_gpu(A, dt), to_gpu(Bt, dt)
    V, meta = sp24.sp24_compress(Ad, layout="tiled")
    D = torch.empty((M, N), dtype=out_dt, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(3)

    def like(t, kind, spread):
        if kind == "workload":
            return t
        if kind == "zeros":
            return torch.zeros_like(t)
        if kind == "ones":
            return torch.ones_like(t)
        x = torch.randn(t.shape, dtype=torch.float32, device="cuda", generator=gen) * spread
        return x.round().clamp(-127, 127).to(torch.int8) if dt == "i8" else x.to(t.dtype)

    def timed(fn):
        for _ in range(5):
            fn()
        batches = []
        for rep in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            batches.append(e0.elapsed_time(e1) / steps)
        return sorted(batches)[1] * 1e3

    spread_a = 12.0 if dt == "i8" else float(Ad.float().std()) * 0.1
    spread_b = 12.0 if dt == "i8" else float(Bd.float().std()) * 0.1
    rows = []
    for ka, kb in (("workload", "workload"), ("workload", "zeros"), ("zeros", "workload"), ("zeros", "zeros"), ("ones", "ones"),
                   ("narrow", "narrow")):
        Vk, Bk = like(V, ka, spread_a), like(Bd, kb, spread_b)
        P = sp24.sp24_decompress(Vk, meta, layout="tiled")
        mm = (lambda: torch._int_mm(P, Bk.t())) if dt == "i8" else (lambda: torch.matmul(P, Bk.t()))
        rows.append({"A": ka, "B": kb,
                     "sparse_us": timed(lambda: sp24.sp24_spmm(Vk, meta, Bk, out_dt, layout="tiled", out=D)),
                     "dense_us": timed(lambda: sp24.sp24_gemm_dense(P, Bk, out_dt, out=D)),
                     "vendor_dense_us": timed(mm)})
    return rows


def measured_traffic(name):
    """HBM bytes per launch of the workload's sparse product kernel, from the counter sections of the committed
    rocprofv3 summary profiles/<workload>_path_rocprofv3.txt: FETCH_SIZE and WRITE_SIZE of that kernel, each scaled by
    what the same counter read for the 1 GiB device copy of the same run (2^20 KiB read, 2^20 KiB written).
    None when the summary is missing or does not hold those lines."""
    import ast
    path = os.path.join(ROOT, "profiles", name + "_path_rocprofv3.txt")
    if not os.path.exists(path):
        return None
    got = {}
    section = None
    for ln in open(path):
        if ln.startswith("== counters"):
            section = "FETCH_SIZE" if "--pmc FETCH_SIZE" in ln else "WRITE_SIZE" if "--pmc WRITE_SIZE" in ln else None
            continue
        if ln.startswith("=="):
            section = None
        if section is None or "{" not in ln:
            continue
        kernel = ln[:ln.index("{")]
        sparse = "k_spmm_pipe" in kernel or "k_conv_patch" in kernel or ("k_mm_skinny" in kernel and "true" in kernel)
        who = "kernel" if sparse else "copy" if "copyBuffer" in kernel else None
        if who and (who, section) not in got:
            got[(who, section)] = float(ast.literal_eval(ln[ln.index("{"):ln.index("}") + 1])[section])
    try:
        kib = (got[("kernel", "FETCH_SIZE")] * 2 ** 20 / got[("copy", "FETCH_SIZE")] +
               got[("kernel", "WRITE_SIZE")] * 2 ** 20 / got[("copy", "WRITE_SIZE")])
    except KeyError:
        return None
    return kib * 1024.0


def measure(name, args, brief=False):
    """All measurements of one workload.  brief: the kernels back to back and the vendor's dense product only (no
    whole-path steps with an event pair per launch, no cache-warm leg, no options)."""
    import numpy as np
    import torch
    from paper_2104_08378_amd import sp24, synth
    from paper_2104_08378_amd.bits import OUT_DT, to_gpu

    w = synth.WORKLOADS[name]
    dt, M, K, N = w["dtype"], w["M"], w["K"], w["N"]
    es = 1 if dt == "i8" else 2
    out_dt = OUT_DT[w["out"]]
    os_ = torch.empty((), dtype=out_dt).element_size()
    A, Bt = synth.make(name)
    # the convolution workload runs as its title says, an implicit GEMM on the NHWC activations (no im2col matrix
    # in device memory); --materialised times the product with the im2col matrix built beforehand instead
    conv = name == "conv3x3_f16" and not args.materialised
    Bsrc = synth.conv_activations() if conv else Bt
    per_set = A.nbytes + Bsrc.nbytes
    R = max(2, min(96, int(600e6 // per_set) + 1))          # rotating input sets: footprint beyond the last-level cache
    As = [to_gpu(A, dt) for _ in range(R)]
    Bs = [to_gpu(Bsrc, dt) for _ in range(R)]
    # every buffer a step touches rotates with the inputs -- outputs and the compressed pair included -- so that no
    # launch finds what it reads, or the lines it overwrites, in the 256 MB last-level cache from the launch before
    Ps = [torch.empty_like(As[0]) for _ in range(R)]
    P2s = [torch.empty_like(As[0]) for _ in range(R)]
    d_bytes = M * N * os_
    Rd = max(2, min(R, int(1.5e9 // max(d_bytes, 1))))        # copies of each product's output
    Ds = [torch.empty((M, N), dtype=out_dt, device="cuda") for _ in range(Rd)]
    Dds = [torch.empty((M, N), dtype=out_dt, device="cuda") for _ in range(Rd)]
    ops = ["prune", "compress", "decompress", "spmm", "dense"]
    only = ([o for o in args.only.split(",") if o] if not brief else []) or list(ops)
    VMs = [sp24.sp24_compress(a_, layout="tiled") for a_ in As]
    for a_, p_ in zip(As, Ps):
        sp24.sp24_prune(a_, out=p_)
    V, meta = VMs[0]
    P, P2, D, Dd = Ps[0], P2s[0], Ds[0], Dds[0]

    def step(i, ev=None):
        a, b = As[i % R], Bs[i % R]
        p_, p2_, (v_, m_) = Ps[i % R], P2s[i % R], VMs[i % R]
        d_, dd_ = Ds[i % Rd], Dds[i % Rd]
        k = 0

        def mark():
            nonlocal k
            if ev is not None:
                ev[k].record()
            k += 1
        mark()
        if "prune" in only:
            sp24.sp24_prune(a, out=p_)
        mark()
        if "compress" in only:
            sp24.sp24_compress(a, layout="tiled", out=(v_, m_))
        mark()
        if "decompress" in only:
            sp24.sp24_decompress(v_, m_, layout="tiled", out=p2_)
        mark()
        if "spmm" in only:
            if conv:
                sp24.sp24_spmm_conv2d(v_, m_, b, out_dt, 3, 3, (1, 1), (1, 1), layout="tiled", out=d_)
            else:
                sp24.sp24_spmm(v_, m_, b, out_dt, layout="tiled", out=d_)
        mark()
        if "dense" in only:
            if conv:
                sp24.sp24_conv2d_dense(p_, b, out_dt, 3, 3, (1, 1), (1, 1), out=dd_)
            else:
                sp24.sp24_gemm_dense(p_, b, out_dt, out=dd_)
        mark()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ms, ms_per_step = None, None
    if not brief:
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i, events[i])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms = {o: float(np.mean([events[i][j].elapsed_time(events[i][j + 1]) for i in range(args.steps)])) for j, o in enumerate(ops)}
        ms_per_step = wall * 1e3 / args.steps

    # Kernel durations.  An event pair around a single launch also counts the dispatch latency of that launch
    # (about 3.5 us here, a fifth of the skinny product); a kernel profiler does not.  So every operation is
    # timed once more as `steps` back-to-back launches, on the same rotating inputs, one event pair around
    # the batch: the mean of that is what rocprofv3 --kernel-trace reports as the kernel's average duration.
    # Five batches each, the median reported.  `same_inputs`: every launch on input set 0, i.e. operands resident in
    # the 256 MB last-level cache -- reported separately (`kernel_ms_cache_warm`), never used for `value`.
    def back_to_back(op, same_inputs=False):
        if op not in only:
            return 0.0
        saved = list(only)
        only[:] = [op]
        for i in range(5):
            step(0 if same_inputs else i)
        batches = []
        for rep in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for i in range(args.steps):
                step(0 if same_inputs else i)
            e1.record()
            torch.cuda.synchronize()
            batches.append(e0.elapsed_time(e1) / args.steps)
        only[:] = saved
        return float(np.median(batches))
    ms_b2b = {o: back_to_back(o) for o in ops}
    ms_warm = None if brief else {"spmm": back_to_back("spmm", True), "dense": back_to_back("dense", True)}

    # The vendor library's dense GEMM on the same shape and the same rotating inputs (torch.matmul / torch._int_mm,
    # i.e. hipBLASLt or rocBLAS), the counterpart of the paper's dense denominator (Sec. 3.2, Fig. 3 use the
    # vendor's dense library).  Output type: the input type (int32 for int8 inputs).
    def vendor_dense():
        if "dense" not in only or "spmm" not in only or (name == "conv3x3_f16" and not conv):
            return None
        try:
            if conv:
                # the vendor's convolution on the same NHWC activations (channels-last tensors; weights [M][r][s][c] as
                # the inner dimension orders them), the pruned weights as a dense filter bank
                wt = P.view(M, 3, 3, K // 9).permute(0, 3, 1, 2)                  # logical NCHW view of channels-last storage
                xs = [b.view(-1, 14, 14, K // 9).permute(0, 3, 1, 2) for b in Bs]
                run = lambda i: torch.nn.functional.conv2d(xs[i % R], wt, padding=1)
            elif dt == "i8":
                run = lambda i: torch._int_mm(Ps[i % R], Bs[i % R].t())
            else:
                run = lambda i: torch.matmul(Ps[i % R], Bs[i % R].t())
            for i in range(5):
                run(i)
            batches = []
            for rep in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for i in range(args.steps):
                    run(i)
                e1.record()
                torch.cuda.synchronize()
                batches.append(e0.elapsed_time(e1) / args.steps)
            t = float(np.median(batches))
            return {"ms": t, "speedup_of_sparse": t / ms_b2b["spmm"], "own_dense_over_vendor": ms_b2b["dense"] / t,
                    "library": "torch %s (%s)" % (torch.__version__, "conv2d, channels-last" if conv else "torch._int_mm" if dt == "i8" else "torch.matmul")}
        except Exception as e:                               # a shape the library call does not take
            return {"error": repr(e)[:200]}
    vendor = vendor_dense()

    # The 256-cubed configuration is bound by launch latency: the same launches recorded in a HIP graph and replayed
    # (the library allocates and synchronises nothing, so it can be captured).  Per sparse product, in microseconds.
    def graph_replay():
        if name != "tiny_f16" or "spmm" not in only:
            return None
        g, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for i in range(args.steps):
                    sp24.sp24_spmm(V, meta, Bs[i % R], out_dt, layout="tiled", out=D)
        for _ in range(3):
            g.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (5 * args.steps) * 1e3
    graph_us = graph_replay()
    if args.calibrate_copy and not brief:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    flops_equiv = 2.0 * M * N * K
    # (--only without an operation: its time is taken as infinite, so that its rates read 0 instead of dividing by 0)
    t_of = {o: (ms_b2b[o] * 1e-3 if o in only else float("inf")) for o in ops}
    t_sp, t_dn = t_of["spmm"], t_of["dense"]
    value = flops_equiv / t_sp / 1e12 if "spmm" in only else 0.0
    bytes_pc = M * K * es * 1.5 + M * K / 8                  # fused prune+compress: read A, write V + meta
    b_bytes = Bsrc.nbytes                                    # the second operand as it lies in memory
    bytes_spmm = M * K * es / 2 + M * K / 8 + b_bytes + M * N * os_
    bytes_dense = M * K * es + b_bytes + M * N * os_
    # the bound is whichever of the two algorithmic minima is longer at the published peaks
    compute_bound = (flops_equiv / 2 / PEAK_DENSE[dt]) >= (bytes_spmm / PEAK_HBM)
    if compute_bound:
        roof = {"bound": "mfma", "achieved": flops_equiv / 2 / t_sp / 1e12, "peak": PEAK_DENSE[dt] / 1e12, "unit": "TFLOP/s",
                "kernel": "sparse product",
                "note": "algorithmic math = the kept half of the products, M*N*K flops per launch, against the dense "
                        "matrix-core peak (equivalently 2*M*N*K against the 2x sparse peak)"}
    else:
        roof = {"bound": "hbm", "achieved": bytes_spmm / t_sp / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                "kernel": "sparse product", "note": "algorithmic bytes = V + meta + B (the NHWC input for the convolution) + D per launch"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    if compute_bound:
        # context: what a register-only loop of the same sparse instruction sustains on this chip with random
        # operands (profiles/chip_ceilings_sp24_probe.txt; the part clocks down under real toggle rates)
        roof["frac_of_measured_issue_rate"] = flops_equiv / t_sp / MEASURED_SPARSE_ISSUE[dt]
    roof["traffic"] = None if (name == "conv3x3_f16" and not conv) else measured_traffic(name)
    # the speedup the paper plots (Sec. 3.2, Fig. 3) is over the best dense product available: the own dense kernel
    # or the vendor library's, whichever is faster on this shape
    both = "dense" in only and "spmm" in only
    t_vendor = vendor["ms"] * 1e-3 if vendor and "ms" in vendor else float("inf")
    t_best = min(t_dn, t_vendor)
    line = {
        "metric": "2:4 SpGEMM dense-equiv TFLOP/s on 1 MI355X; speedup vs same-shape dense GEMM",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"f16": "f16", "bf16": "bf16", "i8": "int8"}[dt], "data": "synthetic",
        "config": {"workload": name, "M": M, "N": N, "K": K, "out": w["out"], "layout": "tiled",
                   "b_order": "implicit im2col of NHWC 64x14x14x256, 3x3, pad 1" if conv else "k-major",
                   "rotating_input_sets": R},
        "step_ms": ms, "kernel_ms_back_to_back": ms_b2b, "kernel_ms_cache_warm": ms_warm,
        "speedup_vs_dense": (t_best / t_sp) if both else None,
        "speedup_vs_dense_is_over": None if not both else ("own dense kernel" if t_dn <= t_vendor else "vendor dense library"),
        "speedup_vs_own_dense": (t_dn / t_sp) if both else None,
        "speedup_vs_vendor_dense": (t_vendor / t_sp) if both and t_vendor != float("inf") else None,
        "dense_tflops": flops_equiv / t_dn / 1e12 if "dense" in only else None,
        "vendor_dense": vendor,
        "graph_replay_us_per_spmm": graph_us,
        "spmm_GBps": bytes_spmm / t_sp / 1e9 if "spmm" in only else None,
        "dense_GBps": bytes_dense / t_dn / 1e9 if "dense" in only else None,
        "prune_GBps": 2.0 * M * K * es / t_of["prune"] / 1e9 if "prune" in only else None,
        "compress_GBps": bytes_pc / t_of["compress"] / 1e9 if "compress" in only else None,
        "decompress_GBps": bytes_pc / t_of["decompress"] / 1e9 if "decompress" in only else None,
        "roofline": roof,
    }
    if brief:
        keep = ("value", "unit", "dtype", "config", "kernel_ms_back_to_back", "speedup_vs_dense", "speedup_vs_dense_is_over",
                "speedup_vs_own_dense", "speedup_vs_vendor_dense", "vendor_dense", "graph_replay_us_per_spmm", "spmm_GBps",
                "prune_GBps", "compress_GBps", "decompress_GBps", "roofline")
        line = {k: line[k] for k in keep}
        line["roofline"] = {k: roof[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
    else:
        if args.sweep and name in ("ffn_bf16", "square_i8"):
            line["sweep_over_K"] = sweep(name, max(5, args.steps // 2))
        if args.few_tiles:
            line["few_tiles"] = few_tiles(name, args.steps)
        if args.operand_dependence and name in ("ffn_bf16", "square_i8"):
            line["operand_dependence"] = operand_dependence(name, args.steps)
        if args.extras:
            line["extras"] = extras(name, As, Bs, V, meta, P, D, Dd, out_dt, A, args.steps, conv)
        if args.cpu_seconds > 0:
            line["cpu_baseline"] = cpu_baseline(name, A, Bt, args.cpu_seconds)
    del As, Bs, Ps, P2s, Ds, Dds, VMs, P, P2, D, Dd, V, meta
    torch.cuda.empty_cache()
    return line


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; --gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2104_08378_amd import synth
    torch.cuda.set_device(0)
    line = measure(args.workload, args)
    if not args.only and not args.no_others:
        # the other configurations, kernels back to back only, as extra keys of the same line
        line["other_workloads"] = {n: measure(n, args, brief=True) for n in synth.WORKLOADS if n != args.workload}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
