"""Text summaries of rocprofv3 runs of ``bench.py``: ``python -m paper_2309_07235_amd.profile_summary MODE ...``.

Reads the results databases rocprofv3 writes (``<dir>/<name>_results.db``) and prints the short tables kept
under ``profiles/``:

  trace DB                     per-kernel launch statistics of a ``--kernel-trace --stats`` run
  counters DB                  MFMA and LDS counters per kernel of a ``--pmc`` run
  traffic --fetch DB --write DB --n N
                               HBM bytes per launch of the bulk update kernel from the two ``--pmc`` passes
                               (FETCH_SIZE, WRITE_SIZE), each scaled by what the same counter reads for the
                               device copy of known size that ``bench.py`` makes before every factorisation;
                               the last line is the one ``bench.py`` reads for ``roofline.traffic``

Each mode prints the command that produced its input first.  Nothing here touches the GPU.
"""
from __future__ import annotations

import argparse
import collections
import re
import sqlite3
import sys

TRAFFIC_TAG = "roofline.traffic"   # bench.py looks for a line starting with this

COMMANDS = {
    "trace": "rocprofv3 --kernel-trace --stats -d $R/gpurun_out/prof_bench -o bench -- \\\n"
             "      python3 $R/bench.py --steps 10 --warmup 2 --no-cpu-baseline",
    "counters": "rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU_MFMA_MOPS_F64 \\\n"
                "      SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE GRBM_GUI_ACTIVE -d $R/gpurun_out/pmc_mfma -o bench -- \\\n"
                "      python3 $R/bench.py --steps 2 --warmup 1 --no-cpu-baseline --lookahead 2",
    "fetch": "rocprofv3 --pmc FETCH_SIZE -d $R/gpurun_out/pmc_fetch -o bench -- \\\n"
             "      python3 $R/bench.py --steps 2 --warmup 1 --no-cpu-baseline --lookahead 2",
    "write": "rocprofv3 --pmc WRITE_SIZE -d $R/gpurun_out/pmc_write -o bench -- \\\n"
             "      python3 $R/bench.py --steps 2 --warmup 1 --no-cpu-baseline --lookahead 2",
}
LOOKAHEAD_NOTE = ("--lookahead 2: counter collection runs the kernels one at a time, and the default pipeline (lookahead 1)\n"
                  "has kernels that wait inside the kernel for a predecessor running beside them; mode 2 is the same\n"
                  "pipeline, same kernels and launch shapes, ordered by stream events only.")


def _short(name: str) -> str:
    name = re.sub(r"^void ", "", name).replace("dla::", "")
    return re.sub(r"\(.*", "", name)


def trace(db_path: str, top: int) -> None:
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select name, count(*), sum(end-start), avg(end-start), min(end-start), max(end-start) "
                       "from kernels group by name order by sum(end-start) desc").fetchall()
    total = sum(r[2] for r in rows)
    print("Command (from /tmp with TMPDIR=/tmp on the GPU box; R = repository root):\n")
    print("  " + COMMANDS["trace"] + "\n")
    print("Per-kernel aggregate of the `kernels` view of the results database (nanoseconds -> us / ms):\n")
    print(f"{'kernel':78s} {'calls':>6s} {'total_ms':>10s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}")
    for name, c, s, a, mn, mx in rows[:top]:
        print(f"{_short(name)[:78]:78s} {c:6d} {s / 1e6:10.3f} {a / 1e3:9.2f} {mn / 1e3:9.2f} {mx / 1e3:9.2f} {100 * s / total:6.2f}")
    upd = [(c, a) for name, c, s, a, mn, mx in rows if "update_kernel" in name or "update_span_kernel" in name]
    if upd:
        n = sum(c for c, _ in upd)
        print(f"\nbulk update kernel, all variants: {n} launches, average {sum(c * a for c, a in upd) / n / 1e3:.2f} us per launch")


def _dispatches(db_path: str):
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select dispatch_id, kernel_name, counter_name, value, start, end from counters_collection").fetchall()
    disp = {}
    for d, nm, cn, v, s, e in rows:
        x = disp.setdefault(d, {"name": _short(nm), "dur": e - s, "c": collections.defaultdict(float)})
        x["c"][cn] += v
    return disp


def counters(db_path: str) -> None:
    agg = {}
    for x in _dispatches(db_path).values():
        nm = x["name"]
        if "kernel" not in nm or "at::" in nm or "rocclr" in nm:
            continue
        a = agg.setdefault(nm, {"n": 0, "dur": 0.0, "c": collections.defaultdict(float)})
        a["n"] += 1
        a["dur"] += x["dur"]
        for k, v in x["c"].items():
            a["c"][k] += v
    probe = agg.get("mfma_peak_kernel<double>")
    pr = probe["c"]["SQ_VALU_MFMA_BUSY_CYCLES"] / probe["c"]["GRBM_GUI_ACTIVE"] if probe else None
    print("Command (from /tmp with TMPDIR=/tmp; R = repository root):\n")
    print("  " + COMMANDS["counters"] + "\n")
    print(LOOKAHEAD_NOTE + "\n")
    print("Per kernel, summed over its launches (counters_collection view of the results database):")
    print("  MFMA_TFLOP/s          SQ_INSTS_VALU_MFMA_MOPS_F64 * 512 flop / kernel time (executed MFMA work)")
    print("  MFMA_busy_vs_probe_%  SQ_VALU_MFMA_BUSY_CYCLES / GRBM_GUI_ACTIVE of the kernel, relative to the same ratio of the")
    print("                        register-resident MFMA loop that bench.py runs (mfma_peak_kernel, 100 % by definition)")
    print("  LDS_conflict_%        SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE")
    print("Counter collection serialises the kernels: times are those of isolated launches.\n")
    print(f"{'kernel':50s} {'launches':>8s} {'avg_us':>8s} {'MFMA_TFLOP/s':>12s} {'MFMA_busy_vs_probe_%':>20s} {'LDS_conflict_%':>14s}")
    for nm, a in sorted(agg.items(), key=lambda kv: -kv[1]["dur"]):
        c = a["c"]
        tf = c["SQ_INSTS_VALU_MFMA_MOPS_F64"] * 512 / a["dur"] * 1e-3 if a["dur"] else 0.0
        busy = c["SQ_VALU_MFMA_BUSY_CYCLES"] / c["GRBM_GUI_ACTIVE"] / pr * 100 if pr and c["GRBM_GUI_ACTIVE"] else 0.0
        lds = c["SQ_LDS_BANK_CONFLICT"] / c["SQ_LDS_IDX_ACTIVE"] * 100 if c["SQ_LDS_IDX_ACTIVE"] else 0.0
        print(f"{nm[:50]:50s} {a['n']:8d} {a['dur'] / a['n'] / 1e3:8.1f} {tf:12.1f} {busy:20.1f} {lds:14.1f}")


def _per_kernel(db_path: str):
    agg = collections.defaultdict(list)
    for x in _dispatches(db_path).values():
        agg[x["name"]].append(sum(x["c"].values()))
    return agg


def traffic(fetch_db: str, write_db: str, n: int) -> None:
    f, w = _per_kernel(fetch_db), _per_kernel(write_db)
    copy_kib = n * n * 8 / 1024.0   # bench.py restores each n x n fp64 input with one device-to-device copy
    def copy_reading(agg):
        vals = [v for nm, vs in agg.items() if "copyBuffer" in nm for v in vs if v > 0.4 * copy_kib]
        return sum(vals) / len(vals) if vals else None
    fr, wr = copy_reading(f), copy_reading(w)
    if not fr or not wr:
        print("no device copy of the expected size in the runs: cannot calibrate", file=sys.stderr)
        sys.exit(1)
    ff, wf = copy_kib / fr, copy_kib / wr
    print("Commands (each pass its own run, from /tmp with TMPDIR=/tmp; R = repository root):\n")
    print("  " + COMMANDS["fetch"])
    print("  " + COMMANDS["write"] + "\n")
    print(LOOKAHEAD_NOTE + "\n")
    print("Values are KiB per dispatch, summed over the counter's instances (counters_collection view).")
    print(f"Calibration on the plain device copy of {copy_kib:.0f} KiB that restores each {n} x {n} fp64 input:")
    print(f"  FETCH_SIZE reads {fr:10.1f} KiB -> factor {ff:.2f}")
    print(f"  WRITE_SIZE reads {wr:10.1f} KiB -> factor {wf:.2f}\n")
    print(f"{'kernel':50s} {'dispatches':>10s} {'FETCH avg':>11s} {'FETCH max':>11s} {'WRITE avg':>11s} {'WRITE max':>11s}   (KiB, unscaled)")
    tot_n = 0
    tot_f = tot_w = 0.0
    for nm in sorted(f):
        if not ("update_kernel" in nm or "update_span_kernel" in nm or "gemm_kernel<double, 64, 64" in nm):
            continue
        fv, wv = f[nm], w.get(nm, [0.0])
        print(f"{nm[:50]:50s} {len(fv):10d} {sum(fv) / len(fv):11.1f} {max(fv):11.1f} {sum(wv) / len(wv):11.1f} {max(wv):11.1f}")
        if "update_" in nm:
            tot_n += len(fv)
            tot_f += sum(fv)
            tot_w += sum(wv) * len(fv) / len(wv)
    if tot_n == 0:
        print("no launch of the bulk update kernel in the runs", file=sys.stderr)
        sys.exit(1)
    fetched, written = tot_f / tot_n * ff, tot_w / tot_n * wf
    print(f"\nBulk update kernel, all variants, averaged over {tot_n} launches and scaled:")
    print(f"  fetched {fetched:10.1f} KiB   written {written:10.1f} KiB   total {fetched + written:10.1f} KiB per launch")
    print(f"{TRAFFIC_TAG} n={n} bytes_per_launch={int(round((fetched + written) * 1024))}")


def read_traffic(path: str, n: int):
    """HBM bytes per launch of the bulk update kernel from a summary written by the traffic mode, or None."""
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith(TRAFFIC_TAG):
                    fields = dict(kv.split("=") for kv in line.split()[1:])
                    if int(fields["n"]) == n:
                        return int(fields["bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        pass
    return None


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    sub = ap.add_subparsers(dest="mode", required=True)
    t = sub.add_parser("trace")
    t.add_argument("db")
    t.add_argument("--top", type=int, default=24)
    c = sub.add_parser("counters")
    c.add_argument("db")
    h = sub.add_parser("traffic")
    h.add_argument("--fetch", required=True)
    h.add_argument("--write", required=True)
    h.add_argument("--n", type=int, default=4000)
    args = ap.parse_args(argv)
    if args.mode == "trace":
        trace(args.db, args.top)
    elif args.mode == "counters":
        counters(args.db)
    else:
        traffic(args.fetch, args.write, args.n)
    return 0


if __name__ == "__main__":
    sys.exit(main())
