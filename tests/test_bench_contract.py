"""Host-side contract of bench.py that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_flop_accounting_adds_up_to_18_T_d_f():
    sys.path.insert(0, ROOT)
    import bench
    T, d, f = 4096, 4096, 11008
    for grouped, launches in ((True, 4), (False, 7)):
        per_tag = bench.gemm_flops_by_tag(T, d, f, grouped)
        assert sum(v[0] for v in per_tag.values()) == 18.0 * T * d * f
        assert sum(v[1] for v in per_tag.values()) == launches      # GEMM launches per step
        assert set(per_tag) <= set(bench.TAG_NAMES)


def test_traffic_comes_from_the_tracked_table():
    """`roofline.traffic` is read from profiles/bench_7b_hbm_traffic.txt (written by `bench.py --summarize-profiles`
    from rocprofv3 counter runs), not from a constant in the source."""
    sys.path.insert(0, ROOT)
    import bench
    assert os.path.exists(bench.TRAFFIC_TABLE)
    rows = [l.split("\t") for l in open(bench.TRAFFIC_TABLE) if l.count("\t") >= 4 and not l.startswith("kernel\t")]
    assert rows, "the table has no rows"
    name = rows[0][0].strip()
    got = bench.measured_traffic_bytes(name)
    assert got == (float(rows[0][2]) + float(rows[0][3])) * 1e6
    assert bench.measured_traffic_bytes("no_such_kernel") is None
