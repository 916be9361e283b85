"""The CPU oracle against hand-worked examples (tests/golden/*.txt).

The expected values are fixed by the paper's definitions (Sec. 3.1, 4.3, 4.4,
Alg. 1) and were worked out by hand; see each fixture's header."""
import numpy as np
import pytest

from oracle import fqo
from paper_2503_08040_amd import synth
from tests import golden_io

CRIT = {"NONE": fqo.CRIT_NONE, "ABSMAX": fqo.CRIT_ABSMAX_GT, "ALL": fqo.CRIT_ALL}


def _bf16(m):
    b = synth.to_bf16_bits(m.astype(np.float32))
    # fixtures must be exactly representable in bf16
    assert np.array_equal(synth.bf16_bits_to_f32(b).astype(np.float64), m)
    return b


@pytest.mark.parametrize("name", ["example_A_underflow.txt", "example_B_ties.txt",
                                  "example_C_scale.txt"])
def test_two_step_quantization_examples(name):
    sc, m = golden_io.load(name)
    q = fqo.quantize(_bf16(m["X"]), int(sc["g"]), CRIT[sc["crit"]], float(sc["theta"]))
    assert np.array_equal(q.codes, m["codes"])
    assert np.array_equal(q.scales.view(np.uint32), m["scales"].view(np.uint32))
    assert np.array_equal(q.mask, m["mask"])
    assert np.array_equal(q.res_scales.view(np.uint32), m["res_scales"].view(np.uint32))
    assert np.array_equal(q.res_codes, m["res_codes"])
    assert q.fb_count[0] == 1 and q.fb_list[0] == 0


def test_example_B_distinguishes_tie_rule():
    # half-away-from-zero would give 3, 4, -1 where ties-to-even gives 2, 4, 0
    _, m = golden_io.load("example_B_ties.txt")
    half_away = np.sign(m["X"]) * np.floor(np.abs(m["X"]) + 0.5)
    assert not np.array_equal(half_away, m["codes"])


def test_fallback_gemm_example_D():
    sc, m = golden_io.load("example_D_gemm.txt")
    g, theta = int(sc["g"]), float(sc["theta"])
    X, W = _bf16(m["X"]), _bf16(m["W4096"] / 4096.0)
    qx = fqo.quantize(X, g, fqo.CRIT_ABSMAX_GT, theta)
    qw = fqo.quantize(W, g, fqo.CRIT_NONE, 0.0)
    assert np.array_equal(qx.codes, m["x_codes"])
    assert np.array_equal(qx.scales.astype(np.float64), m["x_scales"])
    assert np.array_equal(qx.mask, m["x_mask"])
    assert np.array_equal(qx.res_codes, m["x_res_codes"])
    assert np.array_equal(qx.res_scales.astype(np.float64), m["x_res_scales"])
    assert qx.fb_count[0] == 1 and qx.fb_list[0] == 0
    assert np.array_equal(qw.codes, m["w_codes"])
    assert np.all(qw.scales == np.float32(2.0 ** -12))
    assert not qw.mask.any()
    # INT32 block products of Alg. 1
    assert np.array_equal(fqo.gemm_partials(fqo.OP_NT, qx, qw, 0, False), m["P_k0"])
    assert np.array_equal(fqo.gemm_partials(fqo.OP_NT, qx, qw, 1, False), m["P_k1"])
    assert np.array_equal(fqo.gemm_partials(fqo.OP_NT, qx, qw, 0, True), m["Pres_k0"])
    assert not fqo.gemm_partials(fqo.OP_NT, qx, qw, 1, True).any()
    # with fallback the result is the exact product
    y, yb = fqo.gemm(fqo.OP_NT, qx, qw, want_bf16=True)
    assert np.array_equal(y.astype(np.float64) * 4096.0, m["Y4096_fallback"])
    exact = m["X"] @ (m["W4096"] / 4096.0).T
    assert np.array_equal(y.astype(np.float64), exact)
    assert np.array_equal(yb, synth.to_bf16_bits(y))
    # without fallback row 1 shows the underflow
    qn = fqo.quantize(X, g, fqo.CRIT_NONE, 0.0)
    yn = fqo.gemm(fqo.OP_NT, qn, qw)
    assert np.array_equal(yn.astype(np.float64) * 4096.0, m["Y4096_none"])
    # the mask alone decides: same quantizer output, fallback term switched off
    yoff = fqo.gemm(fqo.OP_NT, qx, qw, a_fallback=False)
    assert np.array_equal(yoff, yn)
