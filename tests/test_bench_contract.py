"""Parts of the benchmark's command-line contract that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert run.returncode != 0
    assert "one GPU" in (run.stdout + run.stderr)


def test_measured_traffic_constants_match_the_committed_profiles():
    """bench.py's `traffic` figures are FETCH_SIZE x 2 + WRITE_SIZE of the fused kernel in the committed
    rocprofv3 summaries (KiB per dispatch): the constants must not drift from the files they cite."""
    sys.path.insert(0, ROOT)
    import bench

    def per_dispatch(path):
        with open(path) as f:
            for line in f:
                if line.startswith("pod::fused_kernel"):
                    return float(line.split()[-2])
        raise AssertionError(f"no fused_kernel line in {path}")

    for (config, index), value in bench.MEASURED_TRAFFIC_BYTES.items():
        assert index == 0
        fetch = per_dispatch(os.path.join(ROOT, "profiles", f"fused_kernel_fetch_size_config{config}.txt"))
        write = per_dispatch(os.path.join(ROOT, "profiles", f"fused_kernel_write_size_config{config}.txt"))
        assert abs(value - (fetch * 2.0 + write) * 1024) <= 2048, (config, value, fetch, write)
