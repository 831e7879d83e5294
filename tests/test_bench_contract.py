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

    def per_dispatch(path, kernel):
        with open(path) as f:
            for line in f:
                if line.startswith("pod::" + kernel + "<"):
                    return float(line.split()[-2])
        raise AssertionError(f"no {kernel} line in {path}")

    for (config, index), kernels in bench.MEASURED_TRAFFIC_BYTES.items():
        assert index == 0
        for kernel, value in kernels.items():
            fetch = per_dispatch(os.path.join(ROOT, "profiles", f"fused_kernel_fetch_size_config{config}.txt"), kernel)
            write = per_dispatch(os.path.join(ROOT, "profiles", f"fused_kernel_write_size_config{config}.txt"), kernel)
            assert abs(value - (fetch * 2.0 + write) * 1024) <= 2048, (config, kernel, value, fetch, write)


def test_trace_report_on_synthetic_records():
    """The interval arithmetic of the co-location report, on records written by hand."""
    import numpy as np
    from paper_2410_18038_amd import pod, trace_report
    assert trace_report._union_length(np.array([0, 5, 20]), np.array([10, 8, 30])) == 20.0
    assert trace_report._overlap_length(np.array([0]), np.array([10]), np.array([5, 50]), np.array([7, 60])) == 2.0
    trace = np.zeros(4, dtype=pod.TRACE_DTYPE)
    trace["cu"] = [64, 64, 129, 129]
    trace["first_role"] = [0, 1, 1, 1]
    trace["t_begin"], trace["t_switch"], trace["t_end"] = 100, 200, 400
    ev = np.zeros(5, dtype=pod.EVENT_DTYPE)
    ev["kind"] = [0, 0, 1, 1, 1]
    ev["item"] = [0, 1, 0, 1, 2]
    ev["cu"] = [64, 129, 64, 129, 129]
    ev["t_begin"] = [100, 100, 150, 300, 320]
    ev["t_end"] = [200, 200, 400, 310, 400]
    rep = trace_report.colocation(trace, ev, 2, 3)
    assert rep["hardware_units"] == 2 and rep["units_with_both_first_roles"] == 1
    assert rep["units_with_exactly_one_of_each"] == 1
    assert rep["prefill_items_logged_once"] and rep["decode_units_logged_once"]
    assert rep["units_where_roles_overlap_in_time"] == 1
    assert abs(rep["share_of_prefill_time_with_decode_on_same_unit"] - 0.25) < 1e-9
    assert rep["prefill_items_per_xcd"][:3] == [0, 1, 1] and rep["decode_units_per_xcd"][:3] == [0, 1, 2]
    assert "hardware_units" in trace_report.as_text("x", rep)
