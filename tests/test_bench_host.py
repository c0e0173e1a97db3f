"""Host-side logic of bench.py that needs no GPU: the percentile used for the median of the timed regions, the
guard that ties roofline.traffic to the kernels that actually run, the clock reader, and the one-GPU rule."""
import importlib.util
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bench():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)   # defines functions only: main() runs under __main__
    return mod


def test_percentile_is_the_order_statistic_with_linear_interpolation(bench):
    nine = [float(v) for v in range(1, 10)]
    assert bench.percentile(nine, 0.5) == 5.0
    assert bench.percentile(nine, 0.0) == 1.0 and bench.percentile(nine, 1.0) == 9.0
    assert abs(bench.percentile(nine, 0.1) - 1.8) < 1e-12 and abs(bench.percentile(nine, 0.9) - 8.2) < 1e-12
    assert bench.percentile([3.0], 0.9) == 3.0


def test_traffic_figure_is_dropped_when_the_gemm_sources_change(bench, tmp_path, monkeypatch):
    got = bench.measured_traffic()
    if got is None:
        pytest.skip("the committed traffic summary predates the current GEMM sources: nothing to guard")
    assert set(got) == {"M1", "M8", "M64", "source"} and got["M1"] > 244_056_064 and got["M64"] > got["M1"]
    # the same files in a scratch tree, one source byte appended: the summary no longer describes what runs
    csrc = tmp_path / "paper_2505_22179_amd" / "csrc"
    csrc.mkdir(parents=True)
    for name in bench.GEMM_SOURCES:
        shutil.copy(os.path.join(ROOT, "paper_2505_22179_amd", "csrc", name), csrc / name)
    (tmp_path / "profiles").mkdir()
    shutil.copy(os.path.join(ROOT, bench.TRAFFIC_PROFILE), tmp_path / bench.TRAFFIC_PROFILE)
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.measured_traffic() == got
    with open(csrc / bench.GEMM_SOURCES[0], "a") as f:
        f.write("\n")
    assert bench.measured_traffic() is None
    os.remove(tmp_path / bench.TRAFFIC_PROFILE)
    assert bench.measured_traffic() is None


def test_clock_reader_never_raises(bench):
    clocks = bench.gpu_clocks()
    assert clocks is None or all(isinstance(v, int) and v > 0 for v in clocks.values())


def test_more_than_one_gpu_is_refused_with_a_message():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert run.returncode != 0 and "one GPU" in (run.stderr + run.stdout)
