"""CPU-only checks of bench.py's host logic: the one-GPU rule, the workload table and the
kernel-trace summary (no GPU is touched)."""
import os
import sqlite3
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "one GPU" in res.stderr
    assert res.stdout.strip() == ""          # no JSON line that could be mistaken for a result


def test_workload_table_matches_the_shapes():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2006_06762_amd import inputs as I
    table = bench.workload_table(I)
    assert set(I.CONFIG_NAMES) <= set(table)
    # GMM 512^3: 2 M N K FLOPs and each matrix once
    flops, nbytes, bound = table["GMM"]
    assert flops == 2.0 * 512 ** 3 and nbytes == 4.0 * 3 * 512 * 512 and bound == "mfma"
    # C2D: 2 * N * K * OH * OW * C * R * S, padded taps included
    s = I.C2D
    assert table["C2D"][0] == 2.0 * s.N * s.K * s.OH * s.OW * s.C * s.R * s.S
    # the bandwidth-bound rows say so
    assert table["DEP"][2] == "hbm"
    # the step's FLOPs are what the JSON line reports as step_gflop
    total = sum(table[n][0] for n in I.CONFIG_NAMES)
    assert abs(total / 1e9 - 15.53) < 0.01


def test_overlap_plan_launches_every_operator_of_the_step_once():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2006_06762_amd import inputs as I
    flat = [n for ops in bench.OVERLAP_PLAN for n in ops]
    assert sorted(flat) == sorted(I.CONFIG_NAMES)


def test_trace_summary_reads_a_kernel_table(tmp_path):
    sys.path.insert(0, ROOT)
    import bench
    db = str(tmp_path / "t.db")
    con = sqlite3.connect(db)
    con.execute("create table kernels (name text, start integer, end integer)")
    rows = [("void anr::(anonymous namespace)::k1<4>(int)", 0, 5000), ("void anr::(anonymous namespace)::k1<4>(int)", 10000, 17000),
            ("k2", 20000, 21000)]
    con.executemany("insert into kernels values (?, ?, ?)", rows)
    con.commit()
    con.close()
    text = bench.trace_summary(db)
    lines = text.splitlines()
    assert lines[0].split()[:2] == ["kernel", "calls"]
    k1 = [l for l in lines if "k1<4>" in l][0].split()
    assert "anonymous" not in " ".join(k1)
    assert k1[-4:] == ["2", "6.00", "5.00", "6.00"]       # calls, average, minimum, median in microseconds
    assert lines[1].startswith("void anr::k1<4>")         # sorted by total time
