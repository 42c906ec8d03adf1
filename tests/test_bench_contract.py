"""Host-side checks of bench.py's command line contract that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_flags_of_the_contract_exist():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup", "--workload"):
        assert flag in r.stdout


def test_bench_takes_nothing_from_the_test_tree():
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert "helpers" not in src and '"tests"' not in src and "'tests'" not in src


def test_kernel_source_digest_follows_the_sources(tmp_path, monkeypatch):
    sys.path.insert(0, ROOT)
    import bench
    d0 = bench.kernel_source_digest()
    assert len(d0) == 64 and d0 == bench.kernel_source_digest()
    # the same files under another root with one byte more give another digest
    import shutil
    dst = tmp_path / "paper_2105_04779_amd" / "csrc"
    shutil.copytree(os.path.join(ROOT, "paper_2105_04779_amd", "csrc"), dst)
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.kernel_source_digest() == d0
    with open(dst / "api.hip", "a") as f:
        f.write("\n")
    assert bench.kernel_source_digest() != d0
