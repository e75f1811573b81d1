"""bench.py prints ONE JSON line with the agreed fields (a short run of the decode part only),
and refuses more than one GPU."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_contract_fields():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "6", "--warmup", "2", "--sets", "8",
                          "--skip", "group,variants,prefill,grad,stack,pack,patch"],
                         cwd=ROOT, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key, typ in (("metric", str), ("value", float), ("unit", str), ("n_gpus", int), ("steps", int), ("warmup", int),
                     ("ms_per_step", float), ("higher_is_better", bool), ("scaling", str), ("dtype", str),
                     ("data", str), ("config", dict), ("roofline", dict), ("cpu_baseline", dict)):
        assert isinstance(d[key], typ), key
    assert d["vs_baseline"] is None and d["n_gpus"] == 1 and d["steps"] == 6 and d["warmup"] == 2
    assert d["unit"] == "GB/s" and d["higher_is_better"] is True and "workload" in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and r["achieved"] == d["value"]
    assert abs(d["value"] - d["config"]["bytes_per_step"] / (d["ms_per_step"] * 1e-3) / 1e9) / d["value"] < 1e-2
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "GB/s" and c["cores"] >= 1 and c["value"] > 0 and "sample" in c
    assert c["one_thread"]["cores"] == 1 and c["one_thread"]["value"] > 0 and c["nproc"] >= 1 and "cpu_model" in c
    assert set(c["other_configs"]) == {"config2_prefill", "config3_stack", "config4_pack"}
    t = d["timed_replays"]
    assert t["count"] >= 5 and t["ms_per_step_min"] <= t["ms_per_step_median"] <= t["ms_per_step_max"]
    assert t["ms_per_step_median"] == d["ms_per_step"]
    ceil = d["achieved_ceiling"]
    assert 0.3 < ceil["read_only_stream_4GiB"]["frac_hbm"] <= 1.0
    assert ceil["read_only_stream_per_launch_of_decode_layer_size"]["us"] > 0
    m = d["mfma_ceiling"]
    assert 0 < m["2_waves_per_simd_random_operands_TFLOP/s"] <= 2600.0
    assert m["2_waves_per_simd_constant_operands_TFLOP/s"] <= 2600.0
    assert set(("sclk_MHz", "mclk_MHz", "compute_partition", "memory_partition")) <= set(d["device"])


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], cwd=ROOT,
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0 and "one GPU" in res.stderr
