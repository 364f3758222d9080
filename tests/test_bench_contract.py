"""Host-side contract of bench.py and the entry module: what can be checked
without a GPU."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          cwd=ROOT, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line is printed


def test_without_a_gpu_the_bench_fails_loudly():
    import torch
    if torch.cuda.is_available():
        return
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode != 0 and "no GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_per_element():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2503_08154_amd import workloads as wl
    # 2e + 1/2 bytes per element and direction (x or dy in, y or dx out, one nibble of codes)
    assert bench.bytes_per_direction(1000, wl.BF16) == 4500
    assert bench.bytes_per_direction(1000, wl.F32) == 8500
    w = wl.WORKLOADS["vit_b16"]
    assert w.layers == 12 and w.dtype == wl.BF16
    x, dy = wl.layer_inputs(w, 0, 0, n=4096)
    assert x.dtype == np.uint16 and dy.shape == (4096,)


def test_entry_module_has_build_and_smoke():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as g
    assert callable(g.build) and callable(g.smoke)
