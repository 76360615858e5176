"""The benchmark script's contract, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr
    assert p.stdout.strip() == ""


def test_bad_step_counts_are_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "0"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and p.stdout.strip() == ""


def test_traffic_figure_is_tied_to_the_kernel_sources():
    import bench
    from paper_2411_10666_amd.synth import CONFIGS
    digest = bench.kernel_sources_digest()
    assert len(digest) == 16
    for name, m in bench.MEASURED_TRAFFIC.items():
        assert name in CONFIGS
        want = m["bytes_per_match_step"] * 100.0 if m["sources"] == digest else None
        assert bench.measured_traffic(name, 100.0) == want
    assert bench.measured_traffic("cfg1", 100.0) is None   # never measured: never reported
    assert set(bench.ALGO_BYTES_PER_MATCH_STEP) == set(CONFIGS)
    for v in bench.ALGO_BYTES_PER_MATCH_STEP.values():
        assert v["walk"] > v["gather"] > 0
