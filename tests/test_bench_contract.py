"""The benchmark's command-line contract that can be checked without a GPU, and -- on a GPU --
the shape of the JSON line it prints."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, cwd=ROOT)
    assert p.returncode != 0
    assert "one GPU" in p.stderr


def test_product_code_does_not_import_the_oracle():
    """The oracle is test infrastructure: nothing in the package may import it, and bench.py /
    __graft_entry__.py may do so only inside the baseline leg / smoke()."""
    pkg = os.path.join(ROOT, "paper_2307_03500_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            src = open(os.path.join(pkg, name)).read()
            assert "import oracle" not in src and "from oracle" not in src, name
    for name in os.listdir(os.path.join(pkg, "csrc")):
        assert "oracle" not in open(os.path.join(pkg, "csrc", name)).read(), name
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert "\nfrom oracle" not in bench and "\nimport oracle" not in bench  # no module-level import
    entry = open(os.path.join(ROOT, "__graft_entry__.py")).read()
    assert "\nfrom oracle" not in entry and "\nimport oracle" not in entry


def test_oracle_does_not_import_the_product():
    odir = os.path.join(ROOT, "oracle")
    for name in os.listdir(odir):
        if name.endswith(".py"):
            src = open(os.path.join(odir, name)).read()
            assert "paper_2307_03500_amd" not in src and "ctypes" not in src, name


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_agreed_fields():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "resnet18",
                        "--steps", "5", "--warmup", "2"], capture_output=True, text=True, cwd=ROOT,
                       timeout=300)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
                "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config", "roofline",
                "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["vs_baseline"] is None
    assert "workload" in d["config"] and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]
    assert d["oracle_match"] is True
