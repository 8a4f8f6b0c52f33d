"""The reducer behind the text summaries under profiles/: run on a small database with the two views
of a rocprofv3 results database, made here."""
import sqlite3
import subprocess
import sys
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    res = subprocess.run([sys.executable, "-m", "paper_2004_14020_amd.rocprof_summary", *args], cwd=ROOT,
                         capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    return res.stdout


def test_kernel_durations_and_step_structure(tmp_path):
    db = str(tmp_path / "kt_results.db")
    con = sqlite3.connect(db)
    con.execute("create table kernels (name, start, end, queue_id, grid_x, workgroup_x)")
    name = "void caramel::(anonymous namespace)::k_ring_reduce_sm<8, 8, false, true>(caramel::ReduceTile const*)"
    t = 1000
    for step in range(8):                                   # 8 steps of 2 launches, 10 us apart, 100 and 300 ns long
        con.execute("insert into kernels values (?,?,?,?,?,?)", (name, t, t + 100, 1, 1024 * 4, 1024))
        con.execute("insert into kernels values (?,?,?,?,?,?)", (name, t + 150, t + 450, 1, 1024 * 2, 1024))
        t += 10000
    con.execute("insert into kernels values ('other_kernel', 5, 25, 2, 64, 64)")
    con.commit()
    con.close()
    out = run("kernels", db, "--per-step", "2")
    row = [l for l in out.splitlines() if l.startswith("k_ring_reduce_sm<8, 8, false, true>")][0].split()
    assert row[-6:] == ["16", "200.0", "100", "300", "3200", "99.38%"]
    assert "16 launches of this library = 8 steps of 2" in out
    # span 450 ns, busy 400 ns, gap between the two launches 50 ns, period 10 us
    assert "span first start .. last end 0.5 us" in out or "span first start .. last end 0.4 us" in out
    assert "gaps between launches of a queue 0.1 us" in out or "gaps between launches of a queue 0.0 us" in out
    assert "start-to-start period 10.0 us" in out


def test_counter_means_per_dispatch(tmp_path):
    db = str(tmp_path / "pmc_results.db")
    con = sqlite3.connect(db)
    con.execute("create table counters_collection (kernel_name, counter_name, value, dispatch_id)")
    for d, v in enumerate((10.0, 20.0, 30.0)):
        con.execute("insert into counters_collection values ('k_probe<2, 3>(void*)', 'TCC_EA0_WRREQ_sum', ?, ?)", (v, d))
    con.commit()
    con.close()
    out = run("counters", db)
    row = [l for l in out.splitlines() if l.startswith("k_probe<2, 3>")][0].split()
    assert row[-3:] == ["TCC_EA0_WRREQ_sum", "3", "20.0"]
