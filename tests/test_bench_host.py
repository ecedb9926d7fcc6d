"""Host-side checks of bench.py that need no GPU: the committed hardware-counter summary is found and parsed (so the
`traffic` field of the roofline object is a number, not null), and more than one GPU is refused with a message."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_measured_traffic_reads_the_committed_counter_summary():
    sys.path.insert(0, ROOT)
    import bench
    t = bench.measured_traffic("c2_deit_s")
    alg = 44015616                      # algorithmic bytes per GEMM launch of the workload (stated in the same file)
    assert isinstance(t, int) and alg <= t < 2 * alg
    assert bench.measured_traffic("no_such_workload") is None
    text = open(os.path.join(ROOT, "profiles", "forward_c2_deit_s_hbm_traffic.txt")).read()
    assert "algorithmic_bytes_per_launch: %d" % alg in text and "rocprofv3 --pmc FETCH_SIZE" in text


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
