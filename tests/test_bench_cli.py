"""Host-side behaviour of bench.py that needs no GPU: the one-GPU rule and the guard of the
optional live traffic measurement."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode == 2 and "ONE GPU" in p.stderr and p.stdout == ""


def test_traffic_measurement_declines_under_a_profiler(monkeypatch):
    """The child runs of --measure-traffic must not be started from a process that a profiler
    has already attached to (its preloaded library has initialised the GPU)."""
    import bench

    monkeypatch.setattr(sys, "argv", ["bench.py", "--measure-traffic"])
    args = bench.parse_args()
    monkeypatch.setenv("ROCPROF_OUTPUT_PATH", "/tmp/x")
    traffic, why = bench.measure_traffic(args)
    assert traffic is None and "profiler" in why
    monkeypatch.delenv("ROCPROF_OUTPUT_PATH")
    monkeypatch.setenv("LD_PRELOAD", "/opt/rocm/lib/rocprofiler-sdk/librocprofiler-sdk-tool.so")
    traffic, why = bench.measure_traffic(args)
    assert traffic is None and "profiler" in why


def test_recorded_traffic_is_labelled_as_recorded():
    import bench

    traffic, source = bench.recorded_traffic("7b", [])
    assert traffic and traffic > 2.0e9 and "recorded" in source and "not this run" in source
    traffic, source = bench.recorded_traffic("7b", ["accum_threads=128"])
    assert traffic is None and "not measured" in source
    traffic, source = bench.recorded_traffic("tiny", [])
    assert traffic is None
