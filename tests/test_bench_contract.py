"""Host-side contract of bench.py and the entry module (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True,
                          text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0
    assert "--gpus 1" in r.stderr and not r.stdout.strip()


def test_without_a_gpu_the_benchmark_fails_loudly_instead_of_falling_back():
    import torch

    if torch.cuda.is_available():
        return  # on a GPU machine the real run is the test
    r = run("--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "no GPU" in r.stderr and "fallback" in r.stderr and not r.stdout.strip()


def test_entry_module_exposes_build_and_smoke():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as g

    assert callable(g.build) and callable(g.smoke)


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2603_16219_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "specsteer_oracle" not in text, f
