"""Host-side checks of bench.py that need no GPU: the one-GPU contract and the workload table."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args],
                          capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_help_lists_the_modes():
    r = _run("--help")
    assert r.returncode == 0
    for flag in ("--steps", "--warmup", "--gpus", "--sweep", "--backward", "--context", "--criteria"):
        assert flag in r.stdout


def test_default_workload_is_the_config_the_metric_is_quoted_on():
    sys.path.insert(0, ROOT)
    import bench
    wl = bench.make_workload("cfg2")
    assert (wl.M, wl.K, wl.N) == (4096, 4096, 11008)
    nb = (wl.M // 128) * (wl.K // 128)
    assert abs(len(wl.flagged_blocks) / nb - 0.05) < 0.005        # ~5 % of the X blocks hold outliers
    assert wl.X.dtype == np.uint16 and wl.W.dtype == np.uint16     # bf16 bit patterns
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert 'default="cfg2"' in src
    # the peaks the roofline figures are priced against: MI355X's published dense INT8 and HBM
    assert bench.INT8_PEAK_TOPS == 5000.0 and bench.HBM_PEAK_GBS == 8000.0
