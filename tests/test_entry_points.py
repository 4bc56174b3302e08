"""The repository's entry points: package hygiene on the CPU, bench.py and smoke() on the GPU."""
import ast
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2509_01193_amd")


def _imports(path):
    mods = set()
    for node in ast.walk(ast.parse(open(path).read())):
        if isinstance(node, ast.Import):
            mods.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.module and node.level == 0:
            mods.add(node.module.split(".")[0])
    return mods


def test_product_and_oracle_do_not_import_each_other():
    for f in os.listdir(PKG):
        if f.endswith(".py"):
            assert "oracle" not in _imports(os.path.join(PKG, f)), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            assert "paper_2509_01193_amd" not in _imports(os.path.join(ROOT, "oracle", f)), f
    # the native sides share no file either
    csrc = set(os.listdir(os.path.join(PKG, "csrc")))
    assert not csrc & set(os.listdir(os.path.join(ROOT, "oracle")))
    for f in csrc:
        assert "oracle" not in open(os.path.join(PKG, "csrc", f)).read().lower(), f


def test_missing_library_raises_instead_of_falling_back(tmp_path):
    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_2509_01193_amd import binding as bd\n"
            "try:\n    bd.version()\nexcept FileNotFoundError as e:\n    print('raised', e)\n" % ROOT)
    env = dict(os.environ, LOBRA_MLORA_LIB=str(tmp_path / "absent.so"))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "raised" in r.stdout and "absent.so" in r.stdout, r.stdout + r.stderr


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr


def test_graft_entry_has_build_and_smoke():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as ge
    assert callable(ge.build) and callable(ge.smoke)


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_contract_keys():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "3", "--warmup", "1",
                        "--oracle-rows", "64"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
              "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["unit"] == "tokens/s"
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "bf16"
    assert d["config"]["workload"].startswith("cfg2") and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "mfma" and rf["unit"] == "TFLOP/s" and rf["peak"] == 2500.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9 and 0.05 < rf["frac"] < 1.0
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "tokens/s" and cb["value"] > 0 and cb["cores"] >= 1
    assert abs(d["value"] - d["config"]["T"] / (d["ms_per_step"] * 1e-3)) < 1e-6 * d["value"]


@pytest.mark.gpu
def test_bench_padded_layout_counts_real_tokens_only():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "2", "--warmup", "1",
                        "--layout", "padded", "--buckets", "8", "--no-cpu-baseline"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    d = json.loads([l for l in r.stdout.splitlines() if l.startswith("{")][0])
    c = d["config"]
    assert c["layout"] == "padded" and len(c["bucket_bounds"]) <= 8
    assert c["T"] == c["real_tokens"] + c["pad_tokens"] and c["real_tokens"] == 16384 and c["pad_tokens"] > 0
    assert abs(d["value"] - c["real_tokens"] / (d["ms_per_step"] * 1e-3)) < 1e-6 * d["value"]


@pytest.mark.gpu
def test_bench_vendor_gemm_context_line():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "2", "--warmup", "1", "--vendor-gemm"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    d = json.loads([l for l in r.stdout.splitlines() if l.startswith("{")][0])
    assert d["vendor_gemm_context"] and d["T"] == 16384
    for k in ("torch_matmul_x_W_tflops", "torch_matmul_dy_Wt_tflops", "this_library_base_only_tflops"):
        assert 100.0 < d[k] < 2500.0, (k, d[k])


@pytest.mark.gpu
def test_smoke_entry_point():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as ge
    ge.smoke()
