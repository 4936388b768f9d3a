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
    """bench.py takes the counter-measured HBM traffic of the dominant kernel from the committed profile summary of
    its default workload; any other workload reports null."""
    sys.path.insert(0, ROOT)
    import bench

    tag = "opt_stack_32layers_k256_fire5_decode"
    assert os.path.exists(os.path.join(ROOT, "profiles", f"hbm_traffic_{tag}.md"))
    for kernel in ("table_rows", "table_partial", "stream_fired"):
        v = bench.counter_traffic(kernel, tag)
        assert isinstance(v, int) and v > 400_000_000, (kernel, v)
    assert bench.counter_traffic("table_rows", "opt_stack_32layers_k64_fire5_decode") is None
    assert bench.counter_traffic("no_such_kernel", tag) is None
