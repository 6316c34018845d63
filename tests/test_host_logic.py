"""Host-side pieces that need no GPU: the benchmark's refusal of more than one GPU, its reading of the committed
counter summary, and the shape of the committed profiler summaries."""
import glob
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_bench_reads_the_traffic_summary_and_its_commit():
    sys.path.insert(0, ROOT)
    import bench
    traffic, commit = bench.read_traffic()
    assert commit and re.fullmatch(r"[0-9a-f]{7,40}", commit)
    for kernel in ("k_mlp_mfma", "k_march_wave", "k_group_pass", "k_composite_wave", "k_render_init"):
        assert traffic[kernel] > 0
    # the dominant kernel moves tens of MB per launch, not bytes and not terabytes
    assert 1e7 < traffic["k_mlp_mfma"] < 1e9


def test_profiler_summaries_say_how_and_at_which_commit_they_were_made():
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt")))
    assert len(files) >= 4
    for f in files:
        text = open(f).read()
        assert len(text) < 16_000, f                                  # short summaries, not raw output
        assert re.search(r"^measured_at_commit [0-9a-f]{7,40}$", text, re.M), f
        assert "rocprofv3 " in text and "bench.py" in text, f        # the command that made it, on committed files
        assert "_work" not in text, f
