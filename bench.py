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
reported beside it. The line also carries
  roofline      the dominant kernel as launched, against the published and the measured peak
  peaks         fp32 matrix-instruction rate and HBM streaming rates measured by plain kernels in this run
  configs       the other benchmark sizes (d = 64, 256, 2048 with k = 32/64/128, the SVD layer both ways)
  cpu_baseline  the fp64 CPU checker timed on this machine's host cores (one core, and all of them)
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_MATRIX_PEAK_TFLOPS = 157.3  # MI355X published dense fp32 matrix (MFMA) and packed-vector peak
HBM_PEAK_GBS = 8000.0
OTHER_CONFIGS = ("d64_m32_k32", "d256_m32_k32", "d2048_m64_k32", "d2048_m64_k64", "d2048_m64_k128")
SVD_CONFIG = "svd_d1024_m32_k32"


def f_paper(d, n, m, k):
    return 20.0 * d * n * m + 2.0 * d * n * k


def f_seq(d, n, m):
    return 16.0 * d * n * m


def f_exec(d, n, m, k):
    # Gram products 2dnk (upper tiles only: about half of it is issued), two chains 4dnm each,
    # dV products 4dnm + 2dnk.
    return 12.0 * d * n * m + 4.0 * d * n * k


def kernel_flops(slot, d, n, m, k):
    """Algorithmic FLOP of one launch of the kernel in a profiler slot."""
    if slot == "chain_kernel":
        return 4.0 * d * n * m                       # B = V_i a and a -= V_i^T C over all blocks
    if slot == "dv_kernel":
        return 4.0 * d * n * m + 2.0 * d * n * k     # the three products per block
    if slot in ("factor_fused_kernel", "team_factor_kernel"):
        return 2.0 * d * n * k                       # Gram products (upper tiles: about half is issued)
    return None


def chain_algorithmic_bytes(d, n, m, k):
    """HBM bytes one chain launch must move: V, the factors and the input in; the saved block inputs, the
    coefficients and the output out."""
    nb = n // k
    return 4.0 * (d * n + nb * k * k + d * m) + 4.0 * (nb * d * m + n * m + d * m)


def _norm_kernel_name(name):
    name = re.sub(r"^void\s+", "", name.strip())
    name = re.sub(r"\(.*\)$", "", name)
    name = name.replace("fasth::", "").replace(" ", "").replace("false", "0").replace("true", "1")
    return name


def traffic_from_profiles(workload, kernel_variant):
    """HBM bytes per launch of `kernel_variant` from the tracked rocprofv3 counter summary of this workload
    (lines `#traffic kernel="..." fetch_kib=.. write_kib=.. fetch_scale=.. write_scale=..`), or (None, why)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None, f"no counter summary profiles/hbm_traffic_{workload}.txt"
    want = _norm_kernel_name(kernel_variant)
    seen = []
    for line in open(path):
        mt = re.match(r'#traffic kernel="([^"]+)" fetch_kib=([\d.]+) write_kib=([\d.]+) fetch_scale=([\d.]+) write_scale=([\d.]+)', line)
        if not mt:
            continue
        seen.append(mt.group(1))
        if _norm_kernel_name(mt.group(1)) == want:
            return (float(mt.group(2)) * float(mt.group(4)) + float(mt.group(3)) * float(mt.group(5))) * 1024.0, \
                f"profiles/hbm_traffic_{workload}.txt"
    return None, f"the counter summary covers {seen}, the kernel launched is {kernel_variant}"


# ---------------------------------------------------------------------------------------------------------
# CPU legs (run before anything touches the GPU: the all-cores leg forks worker processes)
# ---------------------------------------------------------------------------------------------------------

_CPU = {}


def _cpu_worker(cols):
    from threadpoolctl import threadpool_limits
    from oracle import householder as orc
    with threadpool_limits(limits=1):
        lo, hi = cols
        return orc.product_gradients(_CPU["V"], _CPU["X"][:, lo:hi], _CPU["G"][:, lo:hi])[1]


def cpu_baseline(name, budget_s=10.0):
    """The fp64 one-reflection-at-a-time checker, as it stands, on this machine's host cores: whole forward +
    backward passes of the workload on one core, then with the mini-batch columns dealt to all cores."""
    import multiprocessing as mp
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import householder as orc
    from paper_2009_13977_amd import synthetic
    w = synthetic.WORKLOADS[name]
    p = synthetic.workload_inputs(name)
    d, n, m, k = w.d, w.n, w.m, w.k
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        reps = 0
        while reps < 3 or (time.perf_counter() - t0 < budget_s and reps < 200):
            orc.product_gradients(p["V"], p["X"], p["G"])
            reps += 1
        sec1 = (time.perf_counter() - t0) / reps
    out = {
        "value": f_seq(d, n, m) / sec1 / 1e9,
        "unit": "GFLOP/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"{reps} full fwd+bwd passes of workload {name} (numpy fp64, one reflection at a time), "
                  f"{sec1 * 1e3:.1f} ms each; numerator F_seq = 16 d n m, the FLOP that algorithm executes",
        "ms_per_step": sec1 * 1e3,
        "gflops_paper_count": f_paper(d, n, m, k) / sec1 / 1e9,
        "host_cpus": os.cpu_count(),
    }
    ncpu = max(1, min(os.cpu_count() or 1, m))
    _CPU.update(V=p["V"], X=p["X"], G=p["G"])
    bounds = [(m * i // ncpu, m * (i + 1) // ncpu) for i in range(ncpu)]
    try:
        with mp.get_context("fork").Pool(ncpu) as pool:
            pool.map(_cpu_worker, bounds)  # start-up and first touch, not timed
            t0 = time.perf_counter()
            reps = 0
            while reps < 3 or (time.perf_counter() - t0 < budget_s and reps < 400):
                parts = pool.map(_cpu_worker, bounds)
                dV = np.sum(parts, axis=0)
                reps += 1
            secn = (time.perf_counter() - t0) / reps
        out["all_cores"] = {
            "value": f_seq(d, n, m) / secn / 1e9, "unit": "GFLOP/s", "cores": ncpu, "ms_per_step": secn * 1e3,
            "sample": f"{reps} passes, the {m} columns dealt to {ncpu} processes of one thread each, dV partials "
                      f"summed by the parent",
        }
        del dV
    except Exception as exc:  # a box that forbids worker processes: report the one-core leg alone
        out["all_cores"] = {"value": None, "why": repr(exc)}
    return out


# ---------------------------------------------------------------------------------------------------------
# GPU legs
# ---------------------------------------------------------------------------------------------------------

def _timed(torch, fn, reps):
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps  # ms per call


def _profiled(torch, B, fn, reps):
    """Per-kernel durations from the library's HIP events around every launch (a pass of its own: the events
    perturb end-to-end timing), with the instantiation each slot launched."""
    B.fasth_profile_enable(True)
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    prof = B.fasth_profile_collect()
    variants = B.fasth_profile_variants()
    B.fasth_profile_enable(False)
    return {kn: {"ms_avg": t / c, "launches_per_step": c / reps, "launched": variants.get(kn, "")}
            for kn, (t, c) in prof.items() if c}


def _dominant(kernels):
    return max(kernels, key=lambda kn: kernels[kn]["ms_avg"] * kernels[kn]["launches_per_step"])


def measure_product(torch, B, synthetic, name, steps, warmup, sequential=True):
    """One Householder product workload: fasth_forward + fasth_backward per step."""
    w = synthetic.WORKLOADS[name]
    d, n, m, k = w.d, w.n, w.m, w.k
    p = synthetic.workload_inputs(name)
    dev = torch.device("cuda:0")
    V, X, G = (torch.from_numpy(p[a]).to(dev) for a in ("V", "X", "G"))
    A = torch.empty_like(X); dX = torch.empty_like(X); dV = torch.empty_like(V)
    ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))

    def step():
        B.fasth_forward(V, X, A, ws, k)
        B.fasth_backward(V, G, dV, dX, ws, k)

    for _ in range(warmup):
        step()
    ms = _timed(torch, step, steps)
    kernels = _profiled(torch, B, step, min(steps, 50))
    dom = _dominant(kernels)
    flops = kernel_flops(dom, d, n, m, k)
    tflops = flops / (kernels[dom]["ms_avg"] * 1e-3) / 1e12 if flops else None
    out = {
        "workload": name, "d": d, "n": n, "m": m, "k": k, "steps": steps,
        "ms_per_step": ms,
        "gflops_paper_count": f_paper(d, n, m, k) / (ms * 1e-3) / 1e9,
        "gflops_exec_count": f_exec(d, n, m, k) / (ms * 1e-3) / 1e9,
        "pct_fp32_mfma_peak_paper_count": 100.0 * f_paper(d, n, m, k) / (ms * 1e-3) / (FP32_MATRIX_PEAK_TFLOPS * 1e12),
        "layers_per_sec": 1e3 / ms,
        "dominant_kernel": kernels[dom]["launched"] or dom,
        "dominant_kernel_ms": kernels[dom]["ms_avg"],
        "dominant_kernel_tflops": tflops,
        "dominant_kernel_frac": tflops / FP32_MATRIX_PEAK_TFLOPS if tflops else None,
        "kernels": kernels,
    }
    if sequential:
        wss = B.new_workspace(B.fasth_sequential_workspace_bytes(d, n, m))

        def seq_step():  # 3 n dependent reflection steps: n forward, 2 n backward (Eq. 4 and the gradient)
            B.fasth_sequential_forward(V, X, A)
            B.fasth_sequential_backward(V, A, G, dV, dX, wss)

        seq_step()
        ms_seq = _timed(torch, seq_step, max(3, min(20, steps)))
        out["sequential_gpu"] = {"ms_per_step": ms_seq, "gflops_seq_count": f_seq(d, n, m) / (ms_seq * 1e-3) / 1e9,
                                 "speedup_fasth": ms_seq / ms}
        del wss
    return out, (V, X, G, A, dV, dX, ws, step)


def measure_svd_layer(torch, B, synthetic, name, steps, warmup):
    """The SVD-reparameterised layer (Section 2.2, Table 1 "Inverse"). A step is apply + backward, once for
    W X and once for W^-1 X; each is two Householder products forward and two backward plus the diagonal
    steps, i.e. 2 x F_paper FLOP on the paper's count."""
    w = synthetic.WORKLOADS[name]
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

    flops = 2.0 * f_paper(d, n, m, k)
    res = []
    for label, fn in (("W X", step_apply), ("W^-1 X", step_inverse)):
        for _ in range(warmup):
            fn()
        ms = _timed(torch, fn, steps)
        kernels = _profiled(torch, B, fn, min(steps, 50))
        dom = _dominant(kernels)
        kf = kernel_flops(dom, d, n, m, k)
        tflops = kf / (kernels[dom]["ms_avg"] * 1e-3) / 1e12 if kf else None
        res.append({
            "workload": name, "direction": label, "d": d, "n": n, "m": m, "k": k, "steps": steps,
            "ms_per_step": ms, "gflops_paper_count": flops / (ms * 1e-3) / 1e9,
            "pct_fp32_mfma_peak_paper_count": 100.0 * flops / (ms * 1e-3) / (FP32_MATRIX_PEAK_TFLOPS * 1e12),
            "layers_per_sec": 1e3 / ms,
            "dominant_kernel": kernels[dom]["launched"] or dom, "dominant_kernel_ms": kernels[dom]["ms_avg"],
            "dominant_kernel_tflops": tflops,
            "dominant_kernel_frac": tflops / FP32_MATRIX_PEAK_TFLOPS if tflops else None,
            "kernels": kernels,
        })
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None, help="name in paper_2009_13977_amd.synthetic.WORKLOADS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sequential", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="only the named workload, not the other benchmark sizes")
    ap.add_argument("--no-peaks", action="store_true", help="skip the measurement of the GPU's own peaks")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run a plain device-to-device copy of this many MiB (three times) so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command can be scaled by a kernel "
                         "of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path shards over mini-batch columns; "
              "each GPU would take a share of them and the only exchange would be one sum of dV). Re-run with --gpus 1.", file=sys.stderr)
        return 2

    from paper_2009_13977_amd import synthetic
    name = args.workload or synthetic.HEADLINE
    w = synthetic.WORKLOADS[name]

    cpu = None
    if not args.no_cpu_baseline and not w.svd_layer:
        cpu = cpu_baseline(name)  # before the GPU is initialised: its second leg forks

    import numpy as np
    import torch
    from paper_2009_13977_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    B.load_library()  # raises if the HIP library is missing: there is no fallback
    dev = torch.device("cuda:0")

    if args.copy_calibration_mib > 0:
        src = torch.ones(args.copy_calibration_mib * 1024 * 1024 // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if w.svd_layer:
        res = measure_svd_layer(torch, B, synthetic, name, args.steps, args.warmup)
        a = res[0]
        out = {
            "metric": "svd_layer_fwd_bwd_gflops_paper_count", "value": a["gflops_paper_count"], "unit": "GFLOP/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": a["ms_per_step"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": name, "d": w.d, "n": w.n, "m": w.m, "k": w.k, "seed": w.seed},
            "ms_inverse_apply_step": res[1]["ms_per_step"], "gflops_inverse": res[1]["gflops_paper_count"],
            "kernels": a["kernels"],
            "roofline": {"kernel": a["dominant_kernel"], "bound": "alu", "achieved": a["dominant_kernel_tflops"],
                         "peak": FP32_MATRIX_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": a["dominant_kernel_frac"],
                         "traffic": None},
            "configs": res,
        }
        print(json.dumps(out))
        return 0

    d, n, m, k = w.d, w.n, w.m, w.k
    head, (V, X, G, A, dV, dX, ws, step) = measure_product(torch, B, synthetic, name, args.steps, args.warmup,
                                                          sequential=not args.no_sequential)
    ms_step = head["ms_per_step"]
    # per-step spread (the paper reports mean +- sigma over 100 repetitions)
    per = np.array([_timed(torch, step, 1) for _ in range(min(args.steps, 100))])
    ms_fwd = _timed(torch, lambda: B.fasth_forward(V, X, A, ws, k), args.steps)
    # factors built once and reused (Section 3.3: recurrent and convolutional layers, inference): chain only
    B.fasth_prepare(V, m, ws, k)
    ms_apply = _timed(torch, lambda: B.fasth_apply(V, X, A, ws, k, False, False), args.steps)
    B.fasth_forward(V, X, A, ws, k)
    ms_bwd = _timed(torch, lambda: B.fasth_backward(V, G, dV, dX, ws, k), args.steps)

    kernels = head["kernels"]
    dom = _dominant(kernels)
    launched = kernels[dom]["launched"] or dom
    dom_ms = kernels[dom]["ms_avg"]
    dom_tflops = head["dominant_kernel_tflops"]
    on_matrix_cores = launched.startswith(("chain_tile_kernel", "chain_quad_kernel", "dv_kernel", "factor_fused_kernel", "team_factor_kernel"))
    traffic, traffic_source = traffic_from_profiles(name, launched)
    alg_bytes = chain_algorithmic_bytes(d, n, m, k) if dom == "chain_kernel" else None
    roofline = {
        "kernel": launched,                      # the instantiation that ran, as the launcher picked it
        "slot": dom,
        "bound": "mfma" if on_matrix_cores else "alu",
        "achieved": dom_tflops,
        "peak": FP32_MATRIX_PEAK_TFLOPS,
        "unit": "TFLOP/s",
        "frac": dom_tflops / FP32_MATRIX_PEAK_TFLOPS if dom_tflops else None,
        "ms_avg": dom_ms,
        # HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE, each scaled by what the same counter
        # reads for a plain copy of known size in the same run; taken from the tracked summary only if it is
        # of the very kernel that ran here
        "traffic": traffic,
        "traffic_source": traffic_source,
        "algorithmic_bytes": alg_bytes,
        "traffic_ratio": traffic / alg_bytes if traffic and alg_bytes else None,
        "hbm_gbs": alg_bytes / (dom_ms * 1e-3) / 1e9 if alg_bytes else None,
        "hbm_frac": alg_bytes / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if alg_bytes else None,
    }

    out = {
        "metric": "fasth_fwd_bwd_gflops_paper_count",
        "value": head["gflops_paper_count"],
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
        "layers_per_sec": head["layers_per_sec"],
        "pct_fp32_mfma_peak_paper_count": head["pct_fp32_mfma_peak_paper_count"],
        "gflops_exec_count": head["gflops_exec_count"],
        "pct_fp32_mfma_peak_exec_count": 100.0 * f_exec(d, n, m, k) / (ms_step * 1e-3) / (FP32_MATRIX_PEAK_TFLOPS * 1e12),
        "flops": {"paper": f_paper(d, n, m, k), "exec": f_exec(d, n, m, k), "sequential": f_seq(d, n, m)},
        "ms_forward": ms_fwd,
        "ms_backward": ms_bwd,
        "ms_apply_prepared": ms_apply,
        "tflops_apply_prepared": 4.0 * d * n * m / (ms_apply * 1e-3) / 1e12,
        "ms_step_single": {"mean": float(per.mean()), "std": float(per.std()), "min": float(per.min())},
        "kernels": kernels,
        "roofline": roofline,
    }
    if "sequential_gpu" in head:
        out["sequential_gpu"] = head["sequential_gpu"]
    del V, X, G, A, dV, dX, ws

    if not args.no_peaks:
        buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)  # 1 GiB: four times the last-level cache
        pk = B.fasth_measure_peaks(buf, 3)
        del buf
        out["peaks"] = {
            "fp32_mfma_tflops": {"published": FP32_MATRIX_PEAK_TFLOPS, "measured": pk["fp32_mfma_tflops"]},
            "hbm_gbs": {"published": HBM_PEAK_GBS, "measured_read": pk["hbm_read_gbs"], "measured_copy": pk["hbm_copy_gbs"]},
            "how": "fasth_measure_peaks: v_mfma_f32_16x16x4_f32 from registers on every compute unit; streaming read "
                   "and copy of a 1 GiB buffer; best of 3",
        }
        if dom_tflops and pk["fp32_mfma_tflops"] > 0:
            roofline["frac_of_measured_peak"] = dom_tflops / pk["fp32_mfma_tflops"]

    if not args.no_configs and name == synthetic.HEADLINE:
        configs = []
        for other in OTHER_CONFIGS:
            small = synthetic.WORKLOADS[other].d <= 256
            res, keep = measure_product(torch, B, synthetic, other, 50 if small else 30, 5,
                                        sequential=not args.no_sequential)
            del keep
            configs.append(res)
        slim = {kk: vv for kk, vv in head.items() if kk != "kernels"}
        slim["kernels"] = kernels
        configs.insert(2, slim)  # the headline between d = 256 and d = 2048, as timed above
        svd = measure_svd_layer(torch, B, synthetic, SVD_CONFIG, 30, 5)
        if "sequential_gpu" in head:
            # the layer is two products each way: compared with twice the one-reflection-at-a-time step at this size
            for r in svd:
                r["sequential_gpu"] = {"ms_per_step": 2.0 * head["sequential_gpu"]["ms_per_step"],
                                       "speedup_fasth": 2.0 * head["sequential_gpu"]["ms_per_step"] / r["ms_per_step"],
                                       "how": "twice the sequential step of d1024_m32_k32 (the layer is two products)"}
        configs.extend(svd)
        out["configs"] = configs

    if cpu is not None:
        out["cpu_baseline"] = cpu

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
