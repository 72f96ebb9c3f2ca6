"""The benchmark's command line and output line: what the harness that runs bench.py relies on."""
import contextlib
import io
import json
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message(capsys):
    import bench
    assert bench.main(["--gpus", "2"]) != 0
    assert "ONE GPU" in capsys.readouterr().err


def test_flop_counts_of_a_step():
    import bench
    assert bench.lu_flops(3) == 18.0 and bench.chol_flops(3) == 9.0
    assert bench.mm3_flops(dict(ni=2, nk=3, nj=5, nm=7, nl=11)) == 2.0 * (2 * 3 * 5 + 5 * 7 * 11 + 2 * 5 * 11)


@pytest.mark.gpu
def test_output_line_on_the_gpu():
    """A short run (smaller factorisations, two steps): one JSON line with the agreed fields, internally consistent."""
    import bench
    from paper_2309_07235_amd import inputs
    out = io.StringIO()
    with contextlib.redirect_stdout(out):
        rc = bench.main(["--steps", "2", "--warmup", "1", "--n", "1000", "--no-cpu-baseline"])
    assert rc == 0
    lines = [ln for ln in out.getvalue().splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["dtype"] == "f64" and d["unit"] == "GFLOP/s"
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and "workload" in d["config"]
    step_flops = bench.lu_flops(1000) + bench.chol_flops(1000) + bench.mm3_flops(inputs.MM3_EXTRALARGE)
    assert abs(d["value"] - step_flops / d["ms_per_step"] * 1e-6) <= 1e-3 * d["value"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 78.6
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and 0 < r["frac"] < 1
