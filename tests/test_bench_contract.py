"""Host-only checks of bench.py's command line contract (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    for extra_env, argv in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "2"}, [])):
        env = dict(os.environ, **extra_env)
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + argv, env=env,
                           capture_output=True, text=True, timeout=120)
        assert r.returncode == 2
        assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_workload_table_is_consistent():
    sys.path.insert(0, ROOT)
    import tess_workloads as wl
    names = [w.name for w in wl.WORKLOADS + wl.PAPER_TABLE_WORKLOADS]
    assert len(names) == len(set(names))
    for w in wl.WORKLOADS + wl.PAPER_TABLE_WORKLOADS:
        assert 1 <= w.d <= w.q
        for L in w.layers:
            assert L.a == L.m * w.q * w.d and L.b == L.kb * w.q and L.c == L.n * w.q
    assert wl.workload_by_name("cfg4_q4d4_bf16_attn_h8192").layers[0].m == 8192
    # Table 2 keeps the per-processor block fixed while the grid grows
    weak = [w for w in wl.PAPER_TABLE_WORKLOADS if w.name.startswith("weak")]
    assert {(L.m, L.kb, L.n) for w in weak for L in w.layers if L.name == "up"} == {(24576, 1024, 4096)}


import json

import pytest


@pytest.mark.gpu
def test_bench_line_carries_the_contract_fields():
    """One short run of bench.py on the GPU: a single JSON line with the metric, the roofline
    object of the dominant kernel and per-call figures (the CPU leg and the other workloads
    are skipped here; the default run carries them)."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "2", "--warmup", "1",
                        "--no-cpu", "--no-others", "--no-sustained"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "calls"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["unit"] == "TFLOP/s" and d["dtype"] == "bf16"
    assert d["config"]["workload"] == "cfg4_q4d4_bf16_attn_h8192"
    rf = d["roofline"]
    assert rf["bound"] == "mfma" and rf["peak"] == 2500.0 and rf["unit"] == "TFLOP/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and 0.2 < rf["frac"] < 1.0
    assert abs(d["value"] - d["config"]["flop_per_step"] / d["ms_per_step"] / 1e9) < 1.0
    assert set(d["calls"]) == {"qkv.fwd", "qkv.dx", "qkv.dw", "out.fwd", "out.dx", "out.dw"}
