"""Host-side behaviour of bench.py and of the package boundary that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode == 2 and r.stdout == ""
    assert "one GPU only" in r.stderr and "--gpus 1" in r.stderr


def test_without_a_gpu_the_benchmark_refuses_instead_of_falling_back():
    import torch
    if torch.cuda.is_available():
        return                      # on a GPU machine the benchmark itself is the test
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode == 2 and r.stdout == ""
    assert "no CPU path" in r.stderr


def test_the_product_package_never_touches_the_oracle():
    """The oracle is test infrastructure: nothing under the package imports, loads or names it."""
    pkg = os.path.join(ROOT, "paper_2510_00236_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath or "__pycache__" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f), errors="replace").read()
                for line in text.splitlines():
                    if "oracle" in line.lower():
                        # prose may name it; code may not import, load or call it
                        assert not any(k in line for k in ("import", "CDLL", "dlopen", "oracle.", "oracle/")), f"{f}: {line.strip()}"
    # and the other way round: the oracle shares nothing with the package
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2510_00236_amd" not in text and "libpex.so" not in text, f
