"""Host-side behaviour of bench.py and of the product path when no GPU (or no library) is there: it
must say so and fail, never fall back to the CPU oracle."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, env=None):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, env=env,
                          capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
    assert not [l for l in r.stdout.splitlines() if l.startswith("{")]


def test_without_a_gpu_the_bench_fails_and_prints_no_result_line():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible here")
    r = _run("--steps", "2", "--warmup", "1")
    assert r.returncode != 0
    assert "no GPU" in (r.stdout + r.stderr)
    assert not [l for l in r.stdout.splitlines() if l.startswith("{")]


def test_missing_library_is_an_error_not_a_fallback(tmp_path):
    """The binding raises when libktanh.so is not where it is built; nothing else is tried."""
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import paper_1909_07729_amd.binding as b\n"
        "b.LIB_PATH = %r\n"
        "try:\n"
        "    b.load_library()\n"
        "except Exception as e:\n"
        "    print('raised', type(e).__name__); sys.exit(0)\n"
        "sys.exit(3)\n" % (ROOT, str(tmp_path / "libktanh.so")))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "raised" in r.stdout


def test_product_package_does_not_import_the_oracle():
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_1909_07729_amd")):
        for name in files:
            if name.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, name)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, name)
