"""bench.py end to end on the GPU, on the smallest configuration: the one JSON line it must print, with the fields the
measurement contract names, and the oracle comparison it carries."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(480)
def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline():
    # --quant-sweep (now the default, still accepted) together with the CPU baseline: the combination that used to crash
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "1", "--steps", "3", "--warmup", "1",
                        "--quant-sweep"],
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=380, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["unit"] == "TFLOP/s"
    assert d["value"] > 0 and d["ms_per_step"] > 0 and d["vs_baseline"] is None and "workload" in d["config"]
    roof = d["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 10100.0
    assert roof["achieved"] > 0 and abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    assert roof["launches"] == 3 * 2                      # per layer pass: the forward product, and dW with dX under one event pair
    assert roof["mfma_ceiling"]["TFLOPs"] > 0 and 0.5 < roof["mfma_ceiling"]["clock_ghz"] < 3.0
    assert roof["traffic_source"].startswith("recorded")
    sweep = d["quantizer_sweep"]                          # configuration 5: 3 matrices x 5 modes
    assert len(sweep) == 15 and {r_["mode"] for r_ in sweep} == {"fwd_rtn_row", "bwd_sr_row", "bwd_rtn_row", "bwd_sr_transposed",
                                                                "bwd_rtn_transposed"}
    assert all(r_["GBps"] > 0 and abs(r_["frac_hbm"] - r_["GBps"] / 8000.0) < 1e-3 and r_["copy_GBps"] > 0 for r_ in sweep)
    others = d["other_configs"]                           # the configurations the main workload is not
    assert [o["config"] for o in others] == [2, 3] and all(o["value"] > 0 and o["ms_per_step"] > 0 for o in others)
    cpu = d["cpu_baseline"]
    assert cpu["quantizer"]["fwd_rtn_GBps"] > 0 and cpu["quantizer"]["bwd_sr_GBps"] > 0
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["single_thread"]["cores"] == 1
    par = cpu["parity_on_sample"]
    assert max(par["y"], par["dx"], par["dw"]) <= par["tolerance"] == 1e-5
