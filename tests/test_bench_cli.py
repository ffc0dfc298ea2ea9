"""The benchmark's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
    assert not r.stdout.strip().startswith("{")        # no result line


def test_help_lists_the_workloads():
    r = run("--help")
    assert r.returncode == 0
    for word in ("--steps", "--warmup", "--gpus", "swap", "serve", "grid", "--no-cpu-baseline"):
        assert word in r.stdout


def test_roofline_constants_are_the_published_peaks():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.HBM_PEAK_GBPS == 8000.0 and bench.MFMA_F16_PEAK_TFLOPS == 2500.0
    # traffic constants taken from the committed counter summaries stay within a few percent of the algorithmic bytes
    copy = bench.COPY_KERNEL_TRAFFIC["opt6.7b_tp2"]
    assert abs(copy["fetch_bytes"] / 201404416 - 1) < 0.01 and abs(copy["write_bytes"] / 201404416 - 1) < 0.01
    out = bench.COPY_KERNEL_OUT_TRAFFIC["opt6.7b_tp2"]
    assert abs(out["fetch_bytes"] / 201404416 - 1) < 0.01 and abs(out["write_bytes"] / 201404416 - 1) < 0.01
    assert abs(bench.LAYERNORM_TRAFFIC["opt6.7b_tp2"] / (6 * 1024 * 4096) - 1) < 0.02
    for tokens, fetched in bench.SMALL_REQUEST_FETCH["opt6.7b_tp2"].items():
        assert 1.0 <= fetched / 6667665408 < 1.25, tokens
