"""The benchmark's one JSON line has the fields its readers rely on (run in-process on a small call)."""
import io
import json
import os
import sys
from contextlib import redirect_stdout

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_bench(argv):
    sys.path.insert(0, ROOT)
    import bench

    old = sys.argv
    sys.argv = ["bench.py"] + argv
    try:
        buf = io.StringIO()
        with redirect_stdout(buf):
            bench.main()
    finally:
        sys.argv = old
    lines = [line for line in buf.getvalue().splitlines() if line.strip()]
    assert len(lines) == 1, "bench.py prints exactly one line"
    return json.loads(lines[0])


def test_layer_line_has_the_contract_fields():
    r = _run_bench(["--tokens", "2304", "--steps", "2", "--warmup", "1", "--decode-tokens", "1", "--cpu-sample", "4",
                    "--prefill-tokens", "512", "--other-model", "", "--no-stack"])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["steps"] == 2 and r["warmup"] == 1 and r["higher_is_better"] is True
    assert r["unit"] == "tokens/s" and r["dtype"] == "bf16" and r["data"] == "synthetic" and r["vs_baseline"] is None
    assert r["config"]["workload"].startswith("mixtral_layer_prefill_T2304")
    assert abs(r["value"] - 2304 / (r["ms_per_step"] * 1e-3)) <= 1e-6 * r["value"]
    roof = r["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 2500.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9 and 0.0 < roof["frac"] < 1.0
    assert "traffic" in roof and roof["traffic_source"]
    short = r["prefill"][0]   # 512 tokens: below the ridge, priced against the HBM bound, both fractions reported
    assert short["tokens"] == 512 and short["layer_bound"] == "hbm" and 0.0 < short["layer_frac_of_hbm_peak"] < 1.0
    assert 0.0 < short["layer_frac_of_mfma_peak"] < 1.0 and short["roofline"]["bound"] == "hbm"
    assert r["decode"][0]["rendezvous_gave_up"] is False
    cpu = r["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "tokens/s" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    dec = r["decode"][0]["roofline"]
    assert dec["bound"] == "hbm" and dec["unit"] == "GB/s" and dec["peak"] == 8000.0 and 0.0 < dec["frac"] < 1.0
    assert r["mfma_probe"]["random_operands"] > 0 and r["hbm_probe"]["read_stream"] > 0


def test_more_than_one_gpu_is_refused(capsys):
    with pytest.raises(SystemExit) as e:
        _run_bench(["--gpus", "2"])
    assert e.value.code != 0
