"""Per-configuration report of the library against the oracle: ``python -m tests.config_report``.

One block per workload of the paper's case study (Section "Linear Algebra Benchmarks": 3mm on a small
and on the extralarge dataset, LU and Cholesky on the large (N = 2000) and extralarge (N = 4000)
datasets) plus N = 1024 and N = 8192 in fp64, and N = 8192 in fp32 for every block size from 128 to 256:

  - the GPU call: median and minimum of the timed calls (device events on the call's stream, in-place
    inputs restored by an untimed device copy before every call), GFLOP/s, percent of the published and
    of the measured MFMA peak, the split of the call over the library's kernel phases and the rate of
    its GEMM phase alone;
  - parity: the gating maximum relative error against the oracle's result on the same seeded host input
    (fp32 rows: against the fp64 oracle on the fp32-rounded input) and the normwise backward residual
    A - L*U (A - L*L^T; for 3mm the Frobenius distance to the oracle's G), both computed by oracle code
    on the host, with their bounds; above N = 4096 the residual is the largest of eight randomised O(N^2)
    probes |A x - L (U x)| / |A x| with the oracle's matrix-vector routines instead of the O(N^3) product;
  - the oracle itself, timed once on the host cores (threads stated), and single-threaded for N <= 2000.
    A reported baseline, not a target.

It lives beside the tests because it runs the oracle, which only the tests, the smoke check and the
benchmark's baseline leg may do.
"""
from __future__ import annotations

import argparse
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from tests import metrics  # noqa: E402

PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3}   # published dense MFMA peaks of the MI355X
TOL = {"f64": 1e-9, "f32": 1e-4}
EPS = {"f64": metrics.EPS64, "f32": metrics.EPS32}


def _time_calls(torch, fn, restore, warmup: int, calls: int):
    times = []
    for i in range(warmup + calls):
        restore()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        e1.synchronize()
        if i >= warmup:
            times.append(e0.elapsed_time(e1))
    return statistics.median(times), min(times)


def _phases(B, torch, fn, restore, calls: int):
    """ms per call in each kernel phase, and the flop rate of the phases that carry flop counts."""
    B.profile_enable(True)
    for _ in range(calls):
        restore()
        fn()
    torch.cuda.synchronize()
    B.profile_enable(False)
    out = {}
    for name, ph in (("tiled_gemm", B.PHASE_GEMM), ("diag", B.PHASE_DIAG), ("solves", B.PHASE_TRSM),
                     ("bulk_update", B.PHASE_UPDATE)):
        ms, cnt, fl = B.profile_read(ph)
        out[name] = (ms / calls, cnt // calls, (fl / ms * 1e-9) if ms > 0 and fl > 0 else None)
    return out


def _line(label, flops, med, mn, dtype, measured_peak, phases):
    tf = flops / med * 1e-9
    s = (f"{label:<44s} median {med:8.3f} ms  min {mn:8.3f} ms  {tf * 1e3:9.1f} GFLOP/s  "
         f"{tf / PEAK_TFLOPS[dtype] * 100:5.1f} % of {PEAK_TFLOPS[dtype]:.1f}")
    if measured_peak:
        s += f"  {tf / measured_peak * 100:5.1f} % of measured {measured_peak:.1f}"
    print(s)
    parts = []
    gemm_ms = gemm_fl = 0.0
    for name, (ms, cnt, rate) in phases.items():
        if cnt:
            parts.append(f"{name} {ms:.3f} ms / {cnt} launches" + (f" ({rate:.1f} TFLOP/s)" if rate else ""))
            if rate:
                gemm_ms += ms
                gemm_fl += rate * ms
    if parts:
        print("    phases (summed launch times; they overlap across streams): " + "; ".join(parts))
    if gemm_ms > 0:
        r = gemm_fl / gemm_ms
        print(f"    GEMM phase alone: {r:.1f} TFLOP/s = {r / PEAK_TFLOPS[dtype] * 100:.1f} % of the published peak")
    sys.stdout.flush()


def _progress(msg: str) -> None:
    print(f"[config_report] {msg}", file=sys.stderr, flush=True)


def _timed(fn):
    t0 = time.perf_counter()
    out = fn()
    return out, time.perf_counter() - t0


def _oracle_line(oracle, flops, seconds, single=None):
    s = f"    oracle: {seconds:.2f} s on {oracle.num_threads()} host threads ({flops / seconds * 1e-9:.1f} GFLOP/s)"
    if single is not None:
        s += f"; single-threaded {single:.2f} s ({flops / single * 1e-9:.1f} GFLOP/s)"
    print(s, flush=True)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--calls", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--max-n", type=int, default=8192, help="skip factorisations larger than this")
    ap.add_argument("--skip-oracle-above", type=int, default=0,
                    help="no oracle run (timing, parity, residual) for factorisations larger than this; 0: never skip")
    args = ap.parse_args(argv)

    import torch
    import oracle
    from paper_2309_07235_amd import binding as B
    from paper_2309_07235_amd import inputs

    if not torch.cuda.is_available():
        print("config_report: no GPU visible", file=sys.stderr)
        return 1
    dev = torch.device("cuda:0")
    threads_all = oracle.num_threads()
    # the probe twice: the first pass also brings the clocks up
    peaks = {"f64": max(B.mfma_peak(B.DLA_F64), B.mfma_peak(B.DLA_F64)),
             "f32": max(B.mfma_peak(B.DLA_F32), B.mfma_peak(B.DLA_F32))}
    print(f"device: {torch.cuda.get_device_name(0)}; measured MFMA peak fp64 {peaks['f64']:.1f}, fp32 {peaks['f32']:.1f} TFLOP/s; "
          f"{args.calls} timed calls after {args.warmup} warm-ups each; host: {os.cpu_count()} logical CPUs, "
          f"oracle on {threads_all} threads")
    failures = 0

    # ---- 3mm ------------------------------------------------------------------------------------
    small = dict(ni=128, nk=128, nj=128, nm=128, nl=128)
    want_cache = {}
    for label, dims, tiles, dtype, seed in (("3mm 128^3, all tiles 16x16", small, (16, 16, 0, 0, 0, 0), "f64", 1),
                                            ("3mm extralarge 1600x2000x1800x2400x2200", inputs.MM3_EXTRALARGE, None, "f64", 4),
                                            ("3mm extralarge 1600x2000x1800x2400x2200 f32", inputs.MM3_EXTRALARGE, None, "f32", 4)):
        tdt = torch.float64 if dtype == "f64" else torch.float32
        dt = B.DLA_F64 if dtype == "f64" else B.DLA_F32
        host = inputs.mm3_operands(seed, **dims)
        if dtype == "f32":
            host = [x.astype(np.float32).astype(np.float64) for x in host]  # what the GPU is given, exactly
        ops = [torch.from_numpy(x).to(dev).to(tdt) for x in host]
        g = torch.empty((dims["ni"], dims["nl"]), dtype=tdt, device=dev)
        p = B.default_params(B.DLA_KERNEL_MM3, dims["nk"], dt)
        if tiles is not None:
            p = B.Mm3Params(B.GemmParams(*tiles), B.GemmParams(*tiles), B.GemmParams(*tiles))
        ws = torch.empty(B.mm3_workspace_bytes(dims["ni"], dims["nj"], dims["nl"], dt), dtype=torch.uint8, device=dev)
        fl = 2.0 * (dims["ni"] * dims["nk"] * dims["nj"] + dims["nj"] * dims["nm"] * dims["nl"] + dims["ni"] * dims["nj"] * dims["nl"])
        fn = lambda: B.mm3(*ops, g, p, workspace=ws)
        med, mn = _time_calls(torch, fn, lambda: None, args.warmup, args.calls)
        _line(label, fl, med, mn, dtype, peaks[dtype], _phases(B, torch, fn, lambda: None, args.calls))
        want, secs = _timed(lambda: oracle.mm3(*host))
        got = g.cpu().numpy().astype(np.float64)
        err, res = metrics.max_rel_err(got, want), metrics.fro_rel_err(got, want)
        bound = 10 * max(dims["nk"], dims["nj"], dims["nm"]) * EPS[dtype]
        ok = err <= TOL[dtype] and res <= bound
        failures += not ok
        print(f"    parity: max rel err {err:.2e} (<= {TOL[dtype]:.0e}), ||G - G_oracle||_F / ||G_oracle||_F {res:.2e} (<= {bound:.2e})"
              f"  {'ok' if ok else 'FAIL'}")
        single = None
        if max(dims.values()) <= 2000:
            oracle.set_num_threads(1)
            _, single = _timed(lambda: oracle.mm3(*host))
            oracle.set_num_threads(threads_all)
        _oracle_line(oracle, fl, secs, single)

    # ---- factorisations ---------------------------------------------------------------------------
    def factor_case(kind, n, nb, dtype, seed):
        nonlocal failures
        if n > args.max_n:
            return
        tdt = torch.float64 if dtype == "f64" else torch.float32
        key = (kind, n, seed, dtype)
        if key not in want_cache:
            want_cache.clear()  # one input at a time in host memory
            _progress(f"{kind} n={n} {dtype}: input")
            H = inputs.diag_dominant_matrix(n, seed) if kind == "lu" else inputs.spd_matrix(n, seed)
            if dtype == "f32":
                H = H.astype(np.float32).astype(np.float64)
            want_cache[key] = {"H": H}
        entry = want_cache[key]
        H = entry["H"]
        src = torch.from_numpy(H).to(dev).to(tdt)
        work = torch.empty_like(src)
        p = B.FactorParams(nb, -1, B.GemmParams(0, 0, 0, 0, 0, 0), 0)
        dt = B.DLA_F64 if dtype == "f64" else B.DLA_F32
        ws = torch.empty(B.factor_workspace_bytes(n, dt, p), dtype=torch.uint8, device=dev)
        info = torch.zeros(1, dtype=torch.int32, device=dev)
        call = B.lu_factor if kind == "lu" else B.cholesky_factor
        fn = lambda: call(work, p, workspace=ws, info=info)
        restore = lambda: work.copy_(src)
        med, mn = _time_calls(torch, fn, restore, args.warmup, args.calls)
        assert int(info.item()) == 0, "breakdown reported on a report input"
        fl = (2.0 if kind == "lu" else 1.0) * n ** 3 / 3.0
        label = f"{'LU' if kind == 'lu' else 'Cholesky'} N={n} nb={nb} {dtype}"
        _line(label, fl, med, mn, dtype, peaks[dtype], _phases(B, torch, fn, restore, min(args.calls, 5)))
        if args.skip_oracle_above and n > args.skip_oracle_above:
            print("    parity and oracle timing skipped (--skip-oracle-above)")
            return
        got = work.cpu().numpy().astype(np.float64)
        _progress(f"{label}: oracle")
        if "want" not in entry:
            (entry["want"], winfo), entry["secs"] = _timed(lambda: oracle.lu(H) if kind == "lu" else oracle.cholesky(H))
            assert winfo == 0
            entry["single"] = None
            if n <= 2000:
                oracle.set_num_threads(1)
                _, entry["single"] = _timed(lambda: oracle.lu(H) if kind == "lu" else oracle.cholesky(H))
                oracle.set_num_threads(threads_all)
        want = entry["want"]
        if kind == "lu":
            parts = metrics.lu_rel_err_parts(got, want)
            err = max(parts.values())
            detail = ", ".join(f"{k} {v:.1e}" for k, v in parts.items())
            _progress(f"{label}: residual")
            if n <= 4096:
                res, res_name = oracle.lu_residual(H, got), "backward residual"
            else:
                res, res_name = 0.0, "probe residual (8 vectors)"
                for q in range(8):
                    x = inputs.uniform_matrix(seed, 50 + q, n, 1).ravel()
                    y0 = oracle.matvec(H, x)
                    res = max(res, float(np.linalg.norm(y0 - oracle.lu_apply(got, x)) / np.linalg.norm(y0)))
        else:
            low = np.tril(got)
            err = metrics.cholesky_rel_err(low, want)
            detail = f"upper triangle {'all zero' if not np.any(np.triu(got, 1)) else 'NOT zero'}"
            _progress(f"{label}: residual")
            if n <= 4096:
                res, res_name = oracle.cholesky_residual(H, low), "backward residual"
            else:
                res, res_name = 0.0, "probe residual (8 vectors)"
                for q in range(8):
                    x = inputs.uniform_matrix(seed, 60 + q, n, 1).ravel()
                    y0 = oracle.symv_lower(H, x)
                    res = max(res, float(np.linalg.norm(y0 - oracle.cholesky_apply(low, x)) / np.linalg.norm(y0)))
        bound = 10 * n * EPS[dtype]
        ok = err <= TOL[dtype] and res <= bound
        failures += not ok
        print(f"    parity: max rel err {err:.2e} (<= {TOL[dtype]:.0e}; {detail}), {res_name} {res:.2e} (<= {bound:.2e})"
              f"  {'ok' if ok else 'FAIL'}")
        _oracle_line(oracle, fl, entry["secs"], entry["single"])

    factor_case("chol", 1024, 64, "f64", 2)
    factor_case("lu", 2000, 128, "f64", 3)
    factor_case("chol", 2000, 128, "f64", 3)
    factor_case("lu", 4000, 128, "f64", 5)
    factor_case("chol", 4000, 128, "f64", 5)
    factor_case("lu", 8192, 128, "f64", 6)
    factor_case("chol", 8192, 128, "f64", 6)
    for kind in ("lu", "chol"):
        for nb in (128, 160, 192, 224, 256):
            factor_case(kind, 8192, nb, "f32", 6)
    print(f"{'all parity figures inside their bounds' if failures == 0 else str(failures) + ' configuration(s) OUTSIDE their bounds'}")
    return 0 if failures == 0 else 2


if __name__ == "__main__":
    sys.exit(main())
