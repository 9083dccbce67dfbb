"""Host-side checks of bench.py and __graft_entry__ that need no GPU."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env=e, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    r = run_bench(env={"WORLD_SIZE": "4"})              # launched as one rank of several
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_the_product_path_never_imports_the_oracle():
    """Only tests, smoke() and the cpu_baseline leg of bench.py may touch oracle/."""
    pkg = os.path.join(ROOT, "paper_2602_13836_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f), encoding="utf-8").read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    text = open(os.path.join(ROOT, "workloads", "gen.py"), encoding="utf-8").read()
    assert "import oracle" not in text and "from oracle" not in text
    bench = open(os.path.join(ROOT, "bench.py"), encoding="utf-8").read()
    uses = [ln for ln in bench.splitlines() if "import oracle" in ln or "from oracle" in ln]
    assert len(uses) == 1, uses                         # the single import inside the cpu_baseline leg


def test_graft_entry_has_build_and_smoke():
    spec = importlib.util.spec_from_file_location("graft_entry", os.path.join(ROOT, "__graft_entry__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert callable(mod.build) and callable(mod.smoke)
