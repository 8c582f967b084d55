"""Host-side checks of bench.py that need no GPU: the one-GPU contract, the figures it reads from the committed
profile summaries, and the published-peak lower bound it prints."""
import os
import subprocess
import sys
import types

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_recorded_figures_come_from_the_committed_summaries():
    traffic = bench.recorded(4, "gemm_config{config}_hbm_traffic.txt", "traffic_bytes_per_launch")
    clock = bench.recorded(4, "gemm_config{config}_mfma_counters.txt", "observed_clock_ghz")
    assert traffic is not None and 3e8 < traffic < 2e9        # operands + fp32 result of an average configuration-4 GEMM
    assert clock is not None and 1.0 < clock < 2.5
    assert bench.recorded(4, "no_such_file.txt", "x") is None
    assert bench.recorded(4, "gemm_config{config}_hbm_traffic.txt", "no_such_key") is None


def test_lower_bound_is_the_sum_of_the_two_rooflines():
    layer = types.SimpleNamespace(t=1024, i=2048, o=4096)
    flops = 6.0 * 1024 * 2048 * 4096
    mem = 2.65625 * (1024 * 2048 + 4096 * 2048) + 2.53125 * 2 * 1024 * 4096 + 1.0625 * (4096 * 2048 + 1024 * 2048)
    want_ms = (flops / (bench.PEAK_FP4_TFLOPS * 1e12) + mem / (bench.PEAK_HBM_GBS * 1e9)) * 1e3
    assert abs(bench.lower_bound_ms([layer]) - want_ms) < 1e-12
    assert abs(bench.lower_bound_ms([layer, layer]) - 2 * want_ms) < 1e-12
    assert bench.PEAK_FP4_TFLOPS == 10100.0 and bench.PEAK_HBM_GBS == 8000.0
