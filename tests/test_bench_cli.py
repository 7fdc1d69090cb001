"""Host-side behaviour of bench.py that needs no GPU: the one-GPU rule and the table printer behind profiles/."""
import sqlite3
import subprocess
import sys
from pathlib import Path

ROOT = Path(__file__).resolve().parent.parent


def run(*args):
    return subprocess.run([sys.executable, str(ROOT / "bench.py"), *args], capture_output=True, text=True, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_summarize_db_prints_the_group_by_tables(tmp_path):
    db = tmp_path / "t_results.db"
    c = sqlite3.connect(db)
    c.execute("create table kernels (name text, duration integer, grid_x integer, workgroup_x integer, lds_size integer, "
              "vgpr_count integer, accum_vgpr_count integer)")
    c.executemany("insert into kernels values (?,?,?,?,?,?,?)",
                  [("void fp4mr::(anonymous namespace)::k_a(int)", 2000, 1024, 256, 0, 32, 0),
                   ("void fp4mr::(anonymous namespace)::k_a(int)", 4000, 1024, 256, 0, 32, 0),
                   ("k_b", 1000, 64, 64, 128, 8, 4)])
    c.execute("create table counters_collection (kernel_name text, counter_name text, grid_size_x integer, value real)")
    c.executemany("insert into counters_collection values (?,?,?,?)", [("k_a", "FETCH_SIZE", 1024, 10.0), ("k_a", "FETCH_SIZE", 1024, 30.0)])
    c.commit()
    c.close()
    r = run("--summarize-db", str(db))
    assert r.returncode == 0, r.stderr
    line = [l for l in r.stdout.splitlines() if l.startswith("k_a(int)")][0].split()
    assert line[1:6] == ["2", "6.0", "3.00", "2.00", "4.00"]          # calls, total, avg, min, max in microseconds
    r = run("--summarize-db", str(db), "--pmc")
    assert r.returncode == 0, r.stderr
    line = [l for l in r.stdout.splitlines() if l.startswith("k_a")][0].split()
    assert line[1:4] == ["FETCH_SIZE", "1024", "2"] and float(line[4]) == 20.0


def test_sweep_tool_parses_its_arguments_without_a_gpu():
    """`python -m paper_2509_23202_amd.sweep --help` loads the binding (the built library) and prints its usage: nothing
    touches the GPU before the arguments are read."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, "-m", "paper_2509_23202_amd.sweep", "--help"], capture_output=True, text=True, timeout=120,
                       cwd=str(__import__("pathlib").Path(__file__).resolve().parents[1]))
    assert r.returncode == 0 and "--tokens" in r.stdout and "bf16" in r.stdout
