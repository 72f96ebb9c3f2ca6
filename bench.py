#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step is one pass over the whole hot path on one batch of seeded synthetic
input resident in HBM: lu_factor (N=4000), cholesky_factor (N=4000) and mm3
(extralarge rectangular shape).  Prints ONE JSON line with the whole-job
throughput in fp64 GFLOP/s, the roofline of the dominant kernel (the rank-128
trailing update of the two factorisations, timed per launch with HIP events on
the stream it runs on) and the CPU oracle timed on the host cores.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

N_FACTOR = 4000
PEAK_F64_MFMA_TFLOPS = 78.6   # MI355X published dense fp64 matrix peak
METRIC = "fp64 GFLOP/s and % of MFMA fp64 peak for LU/Cholesky/3mm at N=4000"
# HBM bytes per launch of the bulk update kernel (fetch + write) come from the summary of the two rocprofv3
# --pmc passes that `python -m paper_2309_07235_amd.profile_summary traffic` writes (counter readings scaled
# by the same counters' readings for a device copy of known size); null when no summary for this N is there.
def update_traffic_bytes_per_launch(n):
    from paper_2309_07235_amd.profile_summary import read_traffic
    return read_traffic(os.path.join(ROOT, "profiles", f"update_kernel_hbm_traffic_n{n}.txt"), n)


def update_algorithmic_bytes(n, nb=128, lower=False, defer_min_rows=0):
    """(launches, bytes) the bulk updates of one factorisation must move: every element of the region
    read and written once, the panels read once (blocks of 128 rows for the lower-triangular case).
    Mirrors the library's schedule (dla.h, dla_factor_params): sub-panels of nb (nb / 2 for block sizes
    above 128); while the trailing matrix has at least the deferral threshold of rows every other step
    puts its bulk update off and the next one applies both sub-panels at once, to the region behind
    block N3."""
    two_level = nb > 128 or (nb == 128 and defer_min_rows != -1)
    if nb > 128:
        nb, min_rows = nb // 2, 0
    else:
        min_rows = defer_min_rows if defer_min_rows > 0 else 2560  # the library's fp64 defaults (fp32 Cholesky: 4096)

    def region(rows, lead):
        if lower:
            elems = sum(min(128, rows - r0) * min(r0 + 128, rows) for r0 in range(0, rows, 128))
        else:
            elems = rows * rows
        return elems - lead * lead

    launches, total = 0, 0
    k0, owed = 0, False
    while True:
        m = n - k0 - nb
        if m <= 0:
            break
        bn = min(nb, m)
        mr = m - bn
        bn2 = min(nb, mr)
        if mr > bn2:
            rest = mr - bn2
            if not owed and two_level and mr >= min_rows and rest >= 4 * nb:
                owed = True
            else:
                rows, depth, lead = (rest, 2 * nb, min(nb, rest)) if owed else (mr, nb, bn2)
                total += 8 * (2 * region(rows, lead) + (1 if lower else 2) * rows * depth)
                launches += 1
                owed = False
        k0 += nb
    return launches, total


def lu_flops(n):
    return 2.0 * n ** 3 / 3.0


def chol_flops(n):
    return n ** 3 / 3.0


def mm3_flops(d):
    return 2.0 * (d["ni"] * d["nk"] * d["nj"] + d["nj"] * d["nm"] * d["nl"] + d["ni"] * d["nj"] * d["nl"])


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--n", type=int, default=N_FACTOR, help="factorisation size (default: the metric's N=4000)")
    ap.add_argument("--lookahead", type=int, default=None,
                    help="override the factorisations' look-ahead mode; 2 (pipeline ordered by stream events only) "
                         "is the one to use under a profiler that serialises kernels (rocprofv3 --pmc)")
    args = ap.parse_args(argv)
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on ONE GPU; --gpus above 1 is not supported "
              "(no collectives or sharding are part of this build).", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2309_07235_amd import binding as B
    from paper_2309_07235_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, W, n = args.steps, args.warmup, args.n
    dims = inputs.MM3_EXTRALARGE

    # ---- seeded synthetic inputs, host side (also fed to the oracle below) ----------------
    A_lu = inputs.diag_dominant_matrix(n, 5)
    A_ch = inputs.spd_matrix(n, 5)
    ops = inputs.mm3_operands(4, **dims)

    d_lu0 = torch.from_numpy(A_lu).to(dev)
    d_ch0 = torch.from_numpy(A_ch).to(dev)
    d_ops = [torch.from_numpy(x).to(dev) for x in ops]
    d_g = torch.empty((dims["ni"], dims["nl"]), dtype=torch.float64, device=dev)
    # factorisations are in place: stage one fresh copy per step so the timed region holds no restore copies
    total = K + W
    lu_bufs = [d_lu0.clone() for _ in range(total)]
    ch_bufs = [d_ch0.clone() for _ in range(total)]
    p_lu = B.default_params(B.DLA_KERNEL_LU, n)
    p_ch = B.default_params(B.DLA_KERNEL_CHOLESKY, n)
    p_mm = B.default_params(B.DLA_KERNEL_MM3, dims["nk"])
    if args.lookahead is not None:
        p_lu.lookahead = p_ch.lookahead = args.lookahead
    ws_f = torch.empty(B.factor_workspace_bytes(n, B.DLA_F64, p_lu), dtype=torch.uint8, device=dev)
    ws_m = torch.empty(B.mm3_workspace_bytes(dims["ni"], dims["nj"], dims["nl"], B.DLA_F64), dtype=torch.uint8,
                       device=dev)
    info = torch.zeros(2, dtype=torch.int32, device=dev)

    def step(i):
        B.lu_factor(lu_bufs[i], p_lu, workspace=ws_f, info=info[0:1])
        B.cholesky_factor(ch_bufs[i], p_ch, workspace=ws_f, info=info[1:2])
        B.mm3(*d_ops, d_g, p_mm, workspace=ws_m)

    for i in range(W):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(W, total):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert int(info[0].item()) == 0 and int(info[1].item()) == 0, "breakdown reported on a benchmark input"

    flops_step = lu_flops(n) + chol_flops(n) + mm3_flops(dims)
    ms_per_step = elapsed / K * 1e3
    gflops = flops_step * K / elapsed * 1e-9

    # ---- per-kernel figures and the GEMM-phase roofline (a repeat of the timed steps, one
    # kernel at a time, with per-launch events on the stream the GEMM runs on) -------------------
    def timed(fn, reps):
        # device events on the caller's stream (every entry point joins its helper streams back into it):
        # a wall clock would add the cost of the two synchronisations, which is not small against 20 short calls
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for r in range(reps):
            fn(r)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    def restore(bufs, src):
        for b in bufs:
            b.copy_(src)
        torch.cuda.synchronize()

    kernels = {}
    upd_ms = upd_fl = 0.0
    upd_launches = 0
    runs = (("lu", lambda r: B.lu_factor(lu_bufs[r], p_lu, workspace=ws_f, info=info[0:1]), lu_flops(n), lu_bufs, d_lu0),
            ("cholesky", lambda r: B.cholesky_factor(ch_bufs[r], p_ch, workspace=ws_f, info=info[1:2]), chol_flops(n), ch_bufs, d_ch0),
            ("mm3", lambda r: B.mm3(*d_ops, d_g, p_mm, workspace=ws_m), mm3_flops(dims), None, None))

    def phase(ph, reps):
        ms, cnt, pf = B.profile_read(ph)
        return {"launches_per_call": cnt // reps, "ms_per_call": round(ms / reps, 4),
                "avg_launch_us": round(ms / cnt * 1e3, 2) if cnt else None,
                "tflops": round(pf / ms * 1e-9, 2) if ms > 0 and pf > 0 else None}, ms, cnt, pf

    for name, fn, fl, bufs, src in runs:
        reps = min(K, total)
        if bufs is not None:
            restore(bufs, src)
        sec = timed(fn, reps)
        if bufs is not None:
            restore(bufs, src)
        B.profile_enable(True)
        timed(fn, reps)
        B.profile_enable(False)
        gemm, _, _, _ = phase(B.PHASE_GEMM, reps)
        diag, _, _, _ = phase(B.PHASE_DIAG, reps)
        solve, _, _, _ = phase(B.PHASE_TRSM, reps)
        upd, ums, ucnt, ufl = phase(B.PHASE_UPDATE, reps)
        kernels[name] = {
            "ms": round(sec * 1e3, 4), "gflops": round(fl / sec * 1e-9, 1),
            "pct_of_peak": round(fl / sec * 1e-12 / PEAK_F64_MFMA_TFLOPS * 100, 2),
            "tiled_gemm": gemm, "bulk_update": upd, "diag": diag, "solves_and_head": solve,
        }
        upd_ms += ums
        upd_fl += ufl
        upd_launches += ucnt
    achieved = upd_fl / upd_ms * 1e-9 if upd_ms > 0 else 0.0  # TFLOP/s
    measured_peak = B.mfma_peak(B.DLA_F64)  # register-resident MFMA loop, the achievable counterpart of the published peak
    la, ba = update_algorithmic_bytes(n, p_lu.nb or 128, False, p_lu.defer_min_rows)
    lc, bc = update_algorithmic_bytes(n, p_ch.nb or 128, True, p_ch.defer_min_rows)
    alg_launches, alg_bytes = la + lc, ba + bc

    # ---- CPU oracle on the host cores: one pass of the same workload ----------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        t = time.perf_counter()
        oracle.lu(A_lu)
        oracle.cholesky(A_ch)
        oracle.mm3(*ops)
        cs = time.perf_counter() - t
        cpu = {"value": round(flops_step / cs * 1e-9, 2), "unit": "GFLOP/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": f"one full step (LU N={n}, Cholesky N={n}, 3mm extralarge), {cs:.1f} s"}

    out = {
        "metric": METRIC, "value": round(gflops, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"lu_factor N={n} + cholesky_factor N={n} + mm3 1600x2000x1800x2400x2200 per step",
                   "lu": {"nb": p_lu.nb, "lookahead": p_lu.lookahead, "update": p_lu.update.as_tuple(),
                          "defer_min_rows": p_lu.defer_min_rows},
                   "cholesky": {"nb": p_ch.nb, "lookahead": p_ch.lookahead, "update": p_ch.update.as_tuple(),
                                "defer_min_rows": p_ch.defer_min_rows},
                   "mm3": {"e": p_mm.e.as_tuple(), "f": p_mm.f.as_tuple(), "g": p_mm.g.as_tuple()}},
        "pct_of_fp64_mfma_peak": round(gflops * 1e-3 / PEAK_F64_MFMA_TFLOPS * 100, 2),
        "measured_fp64_mfma_peak_tflops": round(measured_peak, 2),
        "pct_of_measured_fp64_mfma_peak": round(gflops * 1e-3 / measured_peak * 100, 2),
        "kernels": kernels,
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_F64_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_F64_MFMA_TFLOPS, 4), "traffic": update_traffic_bytes_per_launch(n),
                     "kernel": "update_kernel (bulk trailing update of lu_factor and cholesky_factor, all launches)",
                     "launches": upd_launches, "avg_launch_ms": round(upd_ms / max(upd_launches, 1), 5),
                     "flops_per_launch": round(upd_fl / max(upd_launches, 1), 1),
                     "algorithmic_bytes_per_launch": round(alg_bytes / max(alg_launches, 1), 1),
                     "how": "HIP start/stop events attached to every launch of the kernel (hipExtLaunchKernelGGL) on the "
                            "stream it runs on, in a repeat of the timed steps with the pipeline's other streams beside it"},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
