"""bench.py's command-line contract, as far as it can be checked without a GPU; on a GPU, one short
run of the small configuration and the shape of its JSON line."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args, timeout=600):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=timeout, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr and not r.stdout.strip()


def test_no_product_module_imports_the_oracle():
    """The oracle is test infrastructure: nothing in the package may import it (bench.py's CPU-baseline
    leg and the smoke check are the only callers outside tests/)."""
    pkg = os.path.join(ROOT, "paper_2508_02124_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith(".py"):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f


@pytest.mark.gpu
def test_small_config_json_line(gpu):
    print("[case] bench.py --config cfg1", flush=True)
    r = run_bench("--config", "cfg1", "--steps", "3", "--warmup", "1")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["unit"] == "TFLOP/s" and d["value"] > 0 and d["higher_is_better"] is True
    assert "workload" in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "mfma" and rf["peak"] == 2500.0 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12
    # one record per kernel of the step: the three matrix-core kernels and the HBM-bound score kernel
    rfs = d["rooflines"]
    assert set(rfs) == {"fwd_kernel", "dq_kernel", "dkv_kernel<clean>", "z_kernel"} and rf["kernel"] in rfs
    for name, o in rfs.items():
        assert o["bound"] == ("hbm" if name == "z_kernel" else "mfma") and o["peak"] == (8000.0 if name == "z_kernel" else 2500.0)
        assert abs(o["frac"] - o["achieved"] / o["peak"]) < 1e-12
        assert 0 < o["launch_ms_min"] <= o["launch_ms_median"] and o["launch_ms"] > 0
    assert 0 < d["step_ms_min"] <= d["step_ms_median"]
    for st in ("z", "fwd", "bwd_dq", "bwd_dkv", "bwd_part"):
        assert d["stage_ms_min"][st] <= d["stage_ms_median"][st], st
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
