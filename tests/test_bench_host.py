"""Host-side checks of bench.py that need no GPU: the committed hardware-counter summary is found and parsed (so the
`traffic` field of the roofline object is a number, not null), and more than one GPU is refused with a message."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_measured_traffic_reads_the_committed_counter_summary():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2207_01405_amd import synth
    cfg = synth.CONFIGS["c2_deit_s"]
    M, C, F = cfg["B"] * cfg["T"], cfg["C"], cfg["F"]
    # algorithmic bytes of the four Dense launches of a block: activations in, weights, results (and the residual) out,
    # 12 bytes of parameters per output channel
    alg = ((M * C + 3 * C * C + 3 * M * C + 36 * C) + (M * C + C * C + 2 * M * C + 12 * C) + (M * C + F * C + M * F + 12 * F)
           + (M * F + C * F + 2 * M * C + 12 * C)) // 4
    t = bench.measured_traffic("c2_deit_s")
    assert isinstance(t, int) and alg <= t < 2 * alg
    assert bench.measured_traffic("no_such_workload") is None
    text = open(os.path.join(ROOT, "profiles", "forward_c2_deit_s_hbm_traffic.txt")).read()
    assert "algorithmic_bytes_per_launch: %d" % alg in text and "rocprofv3 --pmc FETCH_SIZE" in text
    # the summary names the build it was taken with; against another build the figure is withheld
    build = [l.split(":", 1)[1].strip() for l in text.splitlines() if l.startswith("build_id:")]
    assert len(build) == 1 and bench.measured_traffic("c2_deit_s", build[0]) == t
    assert bench.measured_traffic("c2_deit_s", "0" * 16) is None


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
