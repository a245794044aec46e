#!/usr/bin/env python3
"""Benchmark of the FastH hot path on one MI355X.

A "step" is one pass of the whole path over one mini-batch of synthetic input: fasth_forward
(Algorithm 1: block factors + block chain) followed by fasth_backward (Algorithm 2: gradient chain
+ per-block dV products), with V, X, G already resident in HBM. The workload is the paper's timing
experiment (Section 4.1): one d x d matrix of Householder vectors, X and G ~ N(0,1), m = 32; the
headline size is d = 1024 with block size 32.

Prints ONE JSON line. `value` is GFLOP/s on the paper-algorithm FLOP count
F_paper = 20 d n m + 2 d n k (Algorithm 1 + Algorithm 2 as written), so it is comparable across
block sizes and with the one-reflection-at-a-time kernel (F_seq = 16 d n m), whose time is
reported beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_MATRIX_PEAK_TFLOPS = 157.3  # MI355X published dense fp32 matrix (MFMA) and packed-vector peak
HBM_PEAK_GBS = 8000.0
CHAIN_TRAFFIC_BYTES = {"d1024_m32_k32": 17522.0 * 1024 * 2.0 + 4340.0 * 1024,
                       # chain_tile_kernel with the block inputs saved (profiles/kernel_trace_and_mfma_d1024_m4096_k32.txt)
                       "d1024_m4096_k32": 33445.0 * 1024 * 2.0 + 557000.0 * 1024}


def f_paper(d, n, m, k):
    return 20.0 * d * n * m + 2.0 * d * n * k


def f_seq(d, n, m):
    return 16.0 * d * n * m


def f_exec(d, n, m, k):
    # Gram products 2dnk (upper tiles only: about half of it is issued), two chains 4dnm each,
    # dV products 4dnm + 2dnk.
    return 12.0 * d * n * m + 4.0 * d * n * k


def chain_flops(d, n, m):
    return 4.0 * d * n * m  # B = V_i a and a -= V_i^T C over all blocks: 2 * 2dnm


def bench_svd_layer(args, name, w) -> int:
    """Non-default workload: the SVD-reparameterised layer (Section 2.2, Table 1 "Inverse"). A step is
    apply + backward, once for W X and once for W^-1 X; each is two Householder products forward and
    two backward plus the diagonal steps, i.e. 2 x F_paper FLOPs on the paper's count."""
    import torch
    from paper_2009_13977_amd import binding as B
    from paper_2009_13977_amd import synthetic
    d, n, m, k = w.d, w.n, w.m, w.k
    p = synthetic.workload_inputs(name)
    dev = torch.device("cuda:0")
    Uv, sg, Vv, X, G = (torch.from_numpy(p[a]).to(dev) for a in ("Uv", "sigma", "Vv", "X", "G"))
    Y = torch.empty_like(X); dX = torch.empty_like(X)
    dU = torch.empty_like(Uv); dVv = torch.empty_like(Vv); ds = torch.empty_like(sg)
    ws = B.new_workspace(B.svd_layer_workspace_bytes(d, n, m, k))

    def step_apply():
        B.svd_layer_apply(Uv, sg, Vv, X, Y, ws, k)
        B.svd_layer_apply_backward(Uv, sg, Vv, G, dU, ds, dVv, dX, ws, k)

    def step_inverse():
        B.svd_layer_inverse_apply(Uv, sg, Vv, X, Y, ws, k)
        B.svd_layer_inverse_apply_backward(Uv, sg, Vv, G, dU, ds, dVv, dX, ws, k)

    def timed(fn, reps):
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    for _ in range(args.warmup):
        step_apply(); step_inverse()
    ms_apply = timed(step_apply, args.steps)
    ms_inverse = timed(step_inverse, args.steps)
    flops = 2.0 * f_paper(d, n, m, k)
    # the dominant kernel (the chain, four launches per step) timed by the library's HIP events in a separate pass
    B.fasth_profile_enable(True)
    for _ in range(args.steps):
        step_apply()
    torch.cuda.synchronize()
    prof = B.fasth_profile_collect()
    B.fasth_profile_enable(False)
    kernels = {kn: {"ms_avg": t / c, "launches_per_step": c / args.steps} for kn, (t, c) in prof.items() if c}
    chain_tflops = chain_flops(d, n, m) / (kernels["chain_kernel"]["ms_avg"] * 1e-3) / 1e12
    out = {
        "metric": "svd_layer_fwd_bwd_gflops_paper_count",
        "value": flops / (ms_apply * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_apply,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": name, "d": d, "n": n, "m": m, "k": k, "seed": w.seed},
        "ms_inverse_apply_step": ms_inverse,
        "gflops_inverse": flops / (ms_inverse * 1e-3) / 1e9,
        "flops": {"paper": flops},
        "kernels": kernels,
        "roofline": {
            "kernel": "chain_kernel", "bound": "alu", "achieved": chain_tflops, "peak": FP32_MATRIX_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": chain_tflops / FP32_MATRIX_PEAK_TFLOPS, "traffic": None,
        },
    }
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None, help="name in paper_2009_13977_amd.synthetic.WORKLOADS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sequential", action="store_true")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run a plain device-to-device copy of this many MiB (three times) so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command can be scaled by a kernel "
                         "of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path shards over mini-batch columns; "
              "each GPU would take a share of them and the only exchange would be one sum of dV). Re-run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2009_13977_amd import binding as B
    from paper_2009_13977_amd import synthetic

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    B.load_library()  # raises if the HIP library is missing: there is no fallback
    name = args.workload or synthetic.HEADLINE
    w = synthetic.WORKLOADS[name]
    if w.svd_layer:
        return bench_svd_layer(args, name, w)
    d, n, m, k = w.d, w.n, w.m, w.k
    p = synthetic.workload_inputs(name)
    dev = torch.device("cuda:0")
    V = torch.from_numpy(p["V"]).to(dev)
    X = torch.from_numpy(p["X"]).to(dev)
    G = torch.from_numpy(p["G"]).to(dev)
    A = torch.empty_like(X); dX = torch.empty_like(X); dV = torch.empty_like(V)
    ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))

    def step():
        B.fasth_forward(V, X, A, ws, k)
        B.fasth_backward(V, G, dV, dX, ws, k)

    def timed(fn, reps):
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps  # ms per call

    if args.copy_calibration_mib > 0:
        src = torch.ones(args.copy_calibration_mib * 1024 * 1024 // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ms_step = timed(step, args.steps)

    # per-step spread (the paper reports mean +- sigma over 100 repetitions)
    per = []
    for _ in range(min(args.steps, 100)):
        per.append(timed(step, 1))
    per = np.array(per)
    ms_fwd = timed(lambda: B.fasth_forward(V, X, A, ws, k), args.steps)
    # factors built once and reused (Section 3.3: recurrent and convolutional layers, inference): chain only
    B.fasth_prepare(V, m, ws, k)
    ms_apply = timed(lambda: B.fasth_apply(V, X, A, ws, k, False, False), args.steps)
    B.fasth_forward(V, X, A, ws, k)
    ms_bwd = timed(lambda: B.fasth_backward(V, G, dV, dX, ws, k), args.steps)

    # per-kernel durations from HIP events around every launch (separate pass: the events perturb
    # end-to-end timing)
    B.fasth_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = B.fasth_profile_collect()
    B.fasth_profile_enable(False)
    kernels = {kn: {"ms_avg": t / c, "launches_per_step": c / args.steps} for kn, (t, c) in prof.items() if c}
    chain_ms = kernels["chain_kernel"]["ms_avg"]
    chain_tflops = chain_flops(d, n, m) / (chain_ms * 1e-3) / 1e12
    # More than 1024 columns (d <= 1024) run the chain on the matrix cores; below that it is one workgroup per
    # column on the vector units.
    chain_on_matrix_cores = m > 1024 and d <= 1024 and d % 4 == 0 and k % 16 == 0

    out = {
        "metric": "fasth_fwd_bwd_gflops_paper_count",
        "value": f_paper(d, n, m, k) / (ms_step * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": name, "d": d, "n": n, "m": m, "k": k, "seed": w.seed},
        "layers_per_sec": 1e3 / ms_step,
        "pct_fp32_mfma_peak_paper_count": 100.0 * f_paper(d, n, m, k) / (ms_step * 1e-3) / (FP32_MATRIX_PEAK_TFLOPS * 1e12),
        "gflops_exec_count": f_exec(d, n, m, k) / (ms_step * 1e-3) / 1e9,
        "flops": {"paper": f_paper(d, n, m, k), "exec": f_exec(d, n, m, k), "sequential": f_seq(d, n, m)},
        "ms_forward": ms_fwd,
        "ms_backward": ms_bwd,
        "ms_apply_prepared": ms_apply,
        "tflops_apply_prepared": chain_flops(d, n, m) / (ms_apply * 1e-3) / 1e12,
        "ms_step_single": {"mean": float(per.mean()), "std": float(per.std()), "min": float(per.min())},
        "kernels": kernels,
        "roofline": {
            "kernel": "chain_kernel",
            "bound": "mfma" if chain_on_matrix_cores else "alu",
            "achieved": chain_tflops,
            "peak": FP32_MATRIX_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": chain_tflops / FP32_MATRIX_PEAK_TFLOPS,
            # HBM bytes per launch from rocprofv3 FETCH_SIZE (x2.0) + WRITE_SIZE (x1.0), scaled by a 256 MiB
            # copy in the same run; measured for the headline and the 4096-column workloads
            # (profiles/hbm_traffic_d1024_m32_k32.txt, profiles/kernel_trace_and_mfma_d1024_m4096_k32.txt).
            "traffic": CHAIN_TRAFFIC_BYTES.get(name),
        },
    }

    if not args.no_sequential:
        wss = B.new_workspace(B.fasth_sequential_workspace_bytes(d, n, m))

        def seq_step():
            B.fasth_sequential_forward(V, X, A)
            B.fasth_sequential_backward(V, X, G, dV, dX, wss)

        seq_step()
        ms_seq = timed(seq_step, max(3, min(20, args.steps)))
        out["sequential_gpu"] = {"ms_per_step": ms_seq, "gflops_seq_count": f_seq(d, n, m) / (ms_seq * 1e-3) / 1e9,
                                 "speedup_fasth": ms_seq / ms_step}
        del wss

    if not args.no_cpu_baseline:
        # The fp64 one-reflection-at-a-time checker, as it stands, on this machine's host cores.
        from threadpoolctl import threadpool_limits
        from oracle import householder as orc
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            reps = 0
            while reps < 3 or (time.perf_counter() - t0 < 10.0 and reps < 200):
                orc.product_gradients(p["V"], p["X"], p["G"])
                reps += 1
            sec = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {
            "value": f_paper(d, n, m, k) / sec / 1e9,
            "unit": "GFLOP/s",
            "cores": 1,
            "kind": "oracle",
            "sample": f"{reps} full fwd+bwd passes of workload {name} (numpy fp64, one reflection at a time), "
                      f"{sec * 1e3:.1f} ms each; same F_paper numerator as `value`",
            "ms_per_step": sec * 1e3,
            "host_cpus": os.cpu_count(),
        }

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
