"""Host-side parts of the benchmark contract that need no GPU."""
import os
import subprocess
import sys

from conftest import ROOT


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_profile_traffic_figure_is_readable():
    """bench.py takes the counter-measured HBM traffic of the dominant kernel from the committed profile summary."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_stream_rows_gptj_block_k256_decode.md")
    lines = [ln for ln in open(path) if ln.startswith("traffic_bytes_per_fired_launch:")]
    assert len(lines) == 1 and int(lines[0].split(":")[1]) > 100_000_000
