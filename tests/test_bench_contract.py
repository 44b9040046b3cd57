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


def test_tracked_profiles_were_taken_on_this_build_of_the_kernels():
    """Every rocprofv3 summary under profiles/ records the hash of the kernel sources it measured; it must be
    the hash of the sources in this tree, so that no figure quoted from them describes other code."""
    sys.path.insert(0, ROOT)
    import bench

    want = bench.kernel_source_hash()
    names = sorted(os.listdir(os.path.join(ROOT, "profiles")))
    assert any(n.startswith("verify_block_c4") for n in names)
    for n in names:
        text = open(os.path.join(ROOT, "profiles", n)).read()
        assert f"kernel_source_sha256: {want}" in text, f"profiles/{n} was taken on another build"
        assert "rocprofv3" in text and " -- python3 bench.py" in text, f"profiles/{n} does not give its command"


def test_traffic_is_only_quoted_from_a_summary_of_this_build(tmp_path, monkeypatch):
    sys.path.insert(0, ROOT)
    import bench

    got, src = bench.read_traffic("c4")
    assert got and got > 3e8 and src == "profiles/verify_block_c4_pmc.txt"
    assert bench.read_traffic("c9")[0] is None
    monkeypatch.setattr(bench, "kernel_source_hash", lambda: "0" * 16)
    got, why = bench.read_traffic("c4")
    assert got is None and "another build" in why
