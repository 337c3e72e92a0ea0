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
