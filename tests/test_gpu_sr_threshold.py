"""GPU parity for the widened path: stochastic-rounding quantizer (bit-exact against the
oracle, same counter-based generator on both sides), the paper's backward recipe built
from it (Sec. 5.1, 5.3: dX = Q_s(dY) W, dW = Q_s(dY)^T Q_s(X)), and the delay-threshold
loop (App. D) driven by the quantizer's own fallback count."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2503_08040_amd as fq
from oracle import fqo
from paper_2503_08040_amd import synth
from tests import gpu_util as gu

F32 = np.float32


def _sr_pair(bits, seed, label):
    gu.announce(f"quantize_sr {label} shape={bits.shape} seed={seed}")
    gq = fq.fq_quantize_sr(gu.to_device_bf16(bits), seed, want_transposed=True)
    oq = fqo.quantize_sr(bits, 128, seed)
    gu.compare_quantized(gq, oq, label)
    return gq, oq


@pytest.mark.parametrize("shape", [(256, 512), (130, 203), (1, 1), (257, 384), (64, 1001)])
def test_sr_codes_bit_exact(shape):
    rng = np.random.default_rng(shape[0] + shape[1])
    x = (rng.standard_t(3.0, size=shape) * 1e-3).astype(F32)
    bits = synth.to_bf16_bits(x)
    for seed in (0, 0x1234567890ABCDEF):
        gq, oq = _sr_pair(bits, seed, f"sr {shape}")
    assert fq.fq_qtensor_check(gq) == 0
    assert gq.c.criterion == fq.FQ_CRIT_NONE


def test_sr_differs_from_nearest_and_across_seeds():
    wl = synth.config4()
    g0 = fq.fq_quantize_sr(gu.to_device_bf16(wl.dY), 1)
    g1 = fq.fq_quantize_sr(gu.to_device_bf16(wl.dY), 2)
    gn = fq.fq_quantize(gu.to_device_bf16(wl.dY), fq.FQ_CRIT_NONE, 0.0)
    c0, c1, cn = (t.view("codes").cpu().numpy() for t in (g0, g1, gn))
    assert (c0 != c1).mean() > 0.1 and (c0 != cn).mean() > 0.1
    assert np.abs(c0.astype(int) - cn.astype(int)).max() <= 1


def test_backward_recipe_of_the_paper():
    """Config 4's tensors with the paper's own backward: stochastic dY and stochastic X context,
    two plain block GEMMs."""
    wl = synth.config4()
    gdy, ody = _sr_pair(wl.dY, 11, "dY")
    gx, ox = _sr_pair(wl.X, 12, "X context")
    gw = fq.fq_quantize(gu.to_device_bf16(wl.W), fq.FQ_CRIT_NONE, 0.0, want_transposed=True)
    ow = fqo.quantize(wl.W, 128, fqo.CRIT_NONE, 0.0)
    for op, gb, ob, name in ((fq.FQ_OP_NN, gw, ow, "dX"), (fq.FQ_OP_TN, gx, ox, "dW")):
        gu.announce(f"backward gemm {name}")
        ref = fqo.gemm(op, ody, ob)
        got = fq.fq_gemm(op, gdy, gb).cpu().numpy()
        assert gu.rel_err(got, ref) <= 1e-3
        assert np.array_equal(got, ref)
    f64 = lambda b: synth.bf16_bits_to_f32(b).astype(np.float64)
    dw = fq.fq_gemm(fq.FQ_OP_TN, gdy, gx).cpu().numpy()
    assert gu.rel_err(dw, f64(wl.dY).T @ f64(wl.X)) < 0.1


def test_delay_threshold_loop_on_gpu():
    """theta starts at 1 and is updated from the count the quantizer reports (read after the
    step, as the paper delays it); it settles with the rate inside [0.1, 0.3]."""
    wl = synth.config2(M=1024, K=2048, N=128, frac=0.2)
    x = gu.to_device_bf16(wl.X)
    q = fq.QTensor(1024, 2048)
    theta, rates = 1.0, []
    for step in range(30):
        gu.announce(f"threshold loop step {step} theta={theta:.4f}")
        fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, theta, out=q)
        n = fq.fq_qtensor_check(q)
        rates.append(n / (q.nbr * q.nbc))
        new = fq.fq_threshold_update(theta, n, q.nbr * q.nbc)
        assert new == fqo.threshold_update(theta, n, q.nbr * q.nbc)
        theta = new
    assert rates[0] == 1.0                       # theta = 1: every N(0,1) block exceeds it
    assert 0.1 <= rates[-1] <= 0.3 and rates[-1] == rates[-2]
    oq = fqo.quantize(wl.X, 128, fqo.CRIT_ABSMAX_GT, theta)
    gu.compare_quantized(q, oq, "threshold loop final")
