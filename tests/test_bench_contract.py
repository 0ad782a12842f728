"""The command line contract of bench.py: one JSON line with the agreed fields, and a refusal of more than one GPU."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode == 2 and "one GPU" in p.stderr and p.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="4")
    p = subprocess.run([sys.executable, BENCH], capture_output=True, text=True, timeout=120, env=env)
    assert p.returncode == 2 and "one GPU" in p.stderr


@pytest.mark.gpu
def test_one_json_line_with_the_agreed_fields():
    p = subprocess.run([sys.executable, BENCH, "--workload", "tiny", "--steps", "6", "--warmup", "4", "--sample-workers", "2"],
                       capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, "bench.py prints exactly one line on stdout"
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
                "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 6 and d["warmup"] == 4 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "f32" and d["unit"] == "mini-batches/s"
    assert d["config"]["workload"] == "tiny" and "model" not in d["config"] and d["config"]["layer_type"] == "sage"
    assert d["value"] > 0 and abs(d["value"] * d["ms_per_step"] / 1e3 - 1.0) < 1e-6
    r = d["roofline"]
    assert set(("bound", "achieved", "peak", "unit", "frac", "traffic")) <= set(r)
    assert r["bound"] in ("hbm", "mfma", "alu", "host_link") and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1 and c["unit"] == d["unit"] and c["sample"]
    assert isinstance(c["cpu_model"], str) and c["cpu_model"]
    # the cache is brought to its steady state whatever --warmup says: t_stale + 1 = 11 untimed iterations, 4 of them warm-up
    assert d["prefill_steps"] == 7
    a = d["path_a1_a6"]
    assert a["bound"] == "hbm" and a["bytes"] > 0 and a["ms"] > 0 and abs(a["frac"] - a["achieved"] / a["peak"]) < 1e-9
    assert not any(k.startswith(("linear", "cache_update")) for k in a["calls"]) and any(k.startswith("top_down") for k in a["calls"])
    pp = d["policy_paper"]
    assert (pp["t_stale"], pp["p_grad"]) == (200, 0.9) and pp["prefill_steps"] + pp["warmup"] == 201 and pp["steps"] == 6
    assert pp["value"] > 0 and 0.0 <= pp["io_saving"] < 1.0 and pp["roofline"]["frac"] > 0
    assert pp["table_rows_read"] <= pp["table_rows_without_cache"]


@pytest.mark.gpu
def test_plain_c_caller():
    """tests/c/c_abi_example (built by __graft_entry__.build() with gcc): the library called from C without Python or torch."""
    exe = os.path.join(ROOT, "tests", "c", "c_abi_example")
    if not os.path.exists(exe):
        pytest.skip("tests/c/c_abi_example is not built: run __graft_entry__.build()")
    p = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert p.returncode == 0 and p.stdout.strip() == "ok", (p.returncode, p.stdout, p.stderr)
