"""Per-configuration timing report of the library: ``python -m paper_2309_07235_amd.report``.

One block per workload of the paper's case study (Section "Linear Algebra Benchmarks": 3mm on a small
and on the extralarge dataset, LU and Cholesky on the large (N = 2000) and extralarge (N = 4000)
datasets) plus N = 1024 and N = 8192 in fp64 and fp32: median and minimum of the timed calls (device
events on the call's stream, in-place inputs restored by an untimed device copy before every call),
GFLOP/s, percent of the published and of the measured MFMA peak, and the split of the call over the
library's kernel phases with the rate of its GEMM phase alone.  Timing only: parity with the reference
results is what the test-suite checks.
"""
from __future__ import annotations

import argparse
import statistics
import sys

PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3}   # published dense MFMA peaks of the MI355X


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


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--calls", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--max-n", type=int, default=8192, help="skip factorisations larger than this")
    args = ap.parse_args(argv)

    import torch
    from . import binding as B
    from . import inputs

    if not torch.cuda.is_available():
        print("report: no GPU visible", file=sys.stderr)
        return 1
    dev = torch.device("cuda:0")
    # the probe twice: the first pass also brings the clocks up
    peaks = {"f64": max(B.mfma_peak(B.DLA_F64), B.mfma_peak(B.DLA_F64)),
             "f32": max(B.mfma_peak(B.DLA_F32), B.mfma_peak(B.DLA_F32))}
    print(f"device: {torch.cuda.get_device_name(0)}; measured MFMA peak fp64 {peaks['f64']:.1f}, fp32 {peaks['f32']:.1f} TFLOP/s; "
          f"{args.calls} timed calls after {args.warmup} warm-ups each")

    # ---- 3mm ------------------------------------------------------------------------------------
    small = dict(ni=128, nk=128, nj=128, nm=128, nl=128)
    for label, dims, tiles, dtype in (("3mm 128^3, all tiles 16x16", small, (16, 16, 0, 0, 0, 0), "f64"),
                                      ("3mm extralarge 1600x2000x1800x2400x2200", inputs.MM3_EXTRALARGE, None, "f64"),
                                      ("3mm extralarge 1600x2000x1800x2400x2200 f32", inputs.MM3_EXTRALARGE, None, "f32")):
        tdt = torch.float64 if dtype == "f64" else torch.float32
        dt = B.DLA_F64 if dtype == "f64" else B.DLA_F32
        ops = [torch.from_numpy(x).to(dev).to(tdt) for x in inputs.mm3_operands(4 if tiles is None else 1, **dims)]
        g = torch.empty((dims["ni"], dims["nl"]), dtype=tdt, device=dev)
        p = B.default_params(B.DLA_KERNEL_MM3, dims["nk"], dt)
        if tiles is not None:
            p = B.Mm3Params(B.GemmParams(*tiles), B.GemmParams(*tiles), B.GemmParams(*tiles))
        ws = torch.empty(B.mm3_workspace_bytes(dims["ni"], dims["nj"], dims["nl"], dt), dtype=torch.uint8, device=dev)
        fl = 2.0 * (dims["ni"] * dims["nk"] * dims["nj"] + dims["nj"] * dims["nm"] * dims["nl"] + dims["ni"] * dims["nj"] * dims["nl"])
        fn = lambda: B.mm3(*ops, g, p, workspace=ws)
        med, mn = _time_calls(torch, fn, lambda: None, args.warmup, args.calls)
        _line(label, fl, med, mn, dtype, peaks[dtype], _phases(B, torch, fn, lambda: None, args.calls))

    # ---- factorisations ---------------------------------------------------------------------------
    def factor_case(kind, n, nb, dtype, seed):
        if n > args.max_n:
            return
        tdt = torch.float64 if dtype == "f64" else torch.float32
        # the seeded uniform M on the host, the Gram matrix on the device (input synthesis, not the path under test)
        M = torch.from_numpy(inputs.uniform_matrix(seed, 0, n, n)).to(dev)
        S = (M @ M.T) / float(n)
        S = torch.tril(S) + torch.tril(S, -1).T
        S.diagonal().add_(float(n) if kind == "lu" else 1.0)
        src = S.to(tdt)
        del M, S
        work = torch.empty_like(src)
        p = B.FactorParams(nb, -1, B.GemmParams(0, 0, 0, 0, 0, 0))
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

    factor_case("chol", 1024, 64, "f64", 2)
    factor_case("lu", 2000, 128, "f64", 3)
    factor_case("chol", 2000, 128, "f64", 3)
    factor_case("lu", 4000, 128, "f64", 5)
    factor_case("chol", 4000, 128, "f64", 5)
    factor_case("lu", 8192, 128, "f64", 6)
    factor_case("chol", 8192, 128, "f64", 6)
    factor_case("lu", 8192, 128, "f32", 6)
    factor_case("chol", 8192, 128, "f32", 6)
    return 0


if __name__ == "__main__":
    sys.exit(main())
