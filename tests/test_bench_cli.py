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
    for flag in ("--steps", "--warmup", "--gpus", "--sweep", "--backward", "--context", "--criteria",
                 "--group-sweep", "--quantizer-sizes", "--pipeline-probe", "--gemm-ablation",
                 "--gemm-only", "--no-tolerance-variant", "--no-overhead-curve"):
        assert flag in r.stdout


def test_ablation_builds_are_declared_with_their_switches():
    """Every ablation build names a switch that the GEMM source really has."""
    sys.path.insert(0, ROOT)
    from paper_2503_08040_amd import build
    src = open(os.path.join(ROOT, "paper_2503_08040_amd", "csrc", "fq_gemm.hip")).read()
    assert build.ABLATIONS
    for name, flags in build.ABLATIONS.items():
        for f in flags:
            macro = f[2:].split("=")[0]
            assert f.startswith("-DFQ_ABLATE_") and macro in src, (name, f)
        assert build.ablation_lib(name).endswith(f"libfq_ablate_{name}.so")


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


def test_traffic_figure_is_tied_to_the_kernel_source(tmp_path, monkeypatch):
    """roofline.traffic comes from the committed profile summary and only while the GEMM source
    is the one it was measured on."""
    import hashlib
    sys.path.insert(0, ROOT)
    import bench
    src = tmp_path / "k.hip"
    src.write_text("kernel v1")
    sha = hashlib.sha256(src.read_bytes()).hexdigest()
    prof = tmp_path / "p.md"
    prof.write_text(f"# summary\n\ngemm_traffic: workload=wl_a bytes_per_launch=123456 fq_gemm_hip_sha256={sha}\n")
    monkeypatch.setattr(bench, "GEMM_SOURCE", str(src))
    monkeypatch.setattr(bench, "TRAFFIC_PROFILE", str(prof))
    assert bench.measured_gemm_traffic("wl_a") == 123456
    assert bench.measured_gemm_traffic("wl_b") is None          # another workload
    src.write_text("kernel v2")
    assert bench.measured_gemm_traffic("wl_a") is None          # the kernel changed since
    monkeypatch.setattr(bench, "TRAFFIC_PROFILE", str(tmp_path / "missing.md"))
    assert bench.measured_gemm_traffic("wl_a") is None
