"""The alternative k-loop schedule kept as a measurement build (the two wavefronts of a SIMD half an
item apart, FQ_ABLATE_TEAM_SKEW: see the header of csrc/fq_gemm.hip) computes the same products as
the library: the GEMM parity tests, which hold fq_gemm to the oracle of Alg. 1 bit for bit, are run
once more in a child process that loads that build instead of the library."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_parity_suite_with_the_team_skew_build():
    sys.path.insert(0, ROOT)
    from paper_2503_08040_amd import build
    lib = build.ablation_lib("team_skew")
    if not os.path.exists(lib):
        pytest.skip("measurement builds are not built (python -c 'import __graft_entry__ as g; g.build()')")
    env = dict(os.environ, FQ_LIBRARY=lib)
    print(f"child: GEMM parity tests with {os.path.basename(lib)}", flush=True)
    r = subprocess.run([sys.executable, "-u", "-m", "pytest", os.path.join(ROOT, "tests", "test_gpu_gemm.py"),
                        "-x", "-q", "-m", "gpu", "--timeout", "120", "--timeout-method", "thread",
                        "-k", "config1 or config4 or ragged or mixed or overflow or cfg3 or cfg5_random"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    print(r.stdout[-1500:], flush=True)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-2000:]
    assert " passed" in r.stdout and "failed" not in r.stdout
