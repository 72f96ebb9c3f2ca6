"""The profile summariser's host logic on small hand-made results databases (no GPU, no profiler)."""
import contextlib
import io
import sqlite3

from paper_2309_07235_amd import profile_summary as ps


def _db(path, rows):
    con = sqlite3.connect(path)
    con.execute("create table counters_collection (dispatch_id int, kernel_name text, counter_name text, value real, "
                "start int, end int)")
    con.executemany("insert into counters_collection values (?, ?, ?, ?, ?, ?)", rows)
    con.commit()
    con.close()


def test_traffic_summary_scales_by_the_copy_and_bench_reads_it_back(tmp_path):
    n = 64
    copy_kib = n * n * 8 / 1024.0  # 32 KiB
    upd = "void dla::update_kernel<double, false, 2, 128>(dla::UpdateArgs<double>)"
    # the fetch counter reports half of the bytes (two instances of a quarter each for the copy), the write counter all
    fetch = [(1, "__amd_rocclr_copyBuffer", "FETCH_SIZE", copy_kib / 4, 0, 10), (1, "__amd_rocclr_copyBuffer", "FETCH_SIZE", copy_kib / 4, 0, 10),
             (2, upd, "FETCH_SIZE", 10.0, 0, 10), (3, upd, "FETCH_SIZE", 30.0, 0, 10), (4, "other_kernel", "FETCH_SIZE", 999.0, 0, 10)]
    write = [(1, "__amd_rocclr_copyBuffer", "WRITE_SIZE", copy_kib, 0, 10), (2, upd, "WRITE_SIZE", 8.0, 0, 10), (3, upd, "WRITE_SIZE", 16.0, 0, 10)]
    f, w = str(tmp_path / "f.db"), str(tmp_path / "w.db")
    _db(f, fetch)
    _db(w, write)
    out = io.StringIO()
    with contextlib.redirect_stdout(out):
        ps.traffic(f, w, n)
    text = out.getvalue()
    assert "factor 2.00" in text and "factor 1.00" in text
    summary = tmp_path / "summary.txt"
    summary.write_text(text)
    # average fetch 20 KiB * 2, average write 12 KiB * 1  ->  52 KiB per launch
    assert ps.read_traffic(str(summary), n) == 52 * 1024
    assert ps.read_traffic(str(summary), n + 1) is None           # a summary for another size does not count
    assert ps.read_traffic(str(tmp_path / "missing.txt"), n) is None


def test_trace_summary_lists_kernels_by_total_time(tmp_path):
    path = str(tmp_path / "t.db")
    con = sqlite3.connect(path)
    con.execute("create table kernels (name text, start int, end int)")
    con.executemany("insert into kernels values (?, ?, ?)",
                    [("void dla::update_kernel<double, false, 2, 128>(dla::UpdateArgs<double>)", 0, 30000),
                     ("void dla::update_kernel<double, false, 2, 128>(dla::UpdateArgs<double>)", 0, 50000),
                     ("void dla::diag_kernel<double, 0>(dla::DiagArgs<double>)", 0, 35000)])
    con.commit()
    con.close()
    out = io.StringIO()
    with contextlib.redirect_stdout(out):
        ps.trace(path, 10)
    lines = [l for l in out.getvalue().splitlines() if l.startswith(("update_kernel", "diag_kernel"))]
    assert lines[0].startswith("update_kernel<double, false, 2, 128>") and " 2 " in lines[0]
    assert "average 40.00 us per launch" in out.getvalue()
