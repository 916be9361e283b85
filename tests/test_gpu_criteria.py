"""GPU parity for the error-based fallback selectors of Sec. 4.4 (L1, L1-Rel): masks, slots,
residual codes and the GEMM built on them match the oracle bit for bit.  The metric sums are
binary64 accumulations whose order differs between the two sides, so thresholds are placed in
gaps between the blocks' metric values (computed by numpy from the oracle's codes)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2503_08040_amd as fq
from oracle import fqo
from paper_2503_08040_amd import synth
from tests import gpu_util as gu

F32 = np.float32
CRITS = {"l1": (fq.FQ_CRIT_L1_GT, fqo.CRIT_L1_GT), "l1rel": (fq.FQ_CRIT_L1REL_GT, fqo.CRIT_L1REL_GT)}


def _metric(bits, which):
    base = fqo.quantize(bits, 128, fqo.CRIT_NONE, 0.0)
    x = synth.bf16_bits_to_f32(bits).astype(np.float64)
    out = np.zeros((base.nbr, base.nbc))
    for bi in range(base.nbr):
        for bk in range(base.nbc):
            rs, cs = slice(bi * 128, (bi + 1) * 128), slice(bk * 128, (bk + 1) * 128)
            r = (x[rs, cs] - float(base.scales[bi, bk]) * base.codes[rs, cs].astype(np.float64)).astype(F32)
            l1 = np.abs(r.astype(np.float64)).sum()
            sx = np.abs(x[rs, cs]).sum()
            out[bi, bk] = l1 if which == "l1" else (l1 / sx if sx > 0 else 0.0)
    return out


def _thresholds(metric, count=3):
    """Thresholds in the `count` widest relative gaps between distinct positive metric values."""
    v = np.unique(metric[metric > 0])
    ratio = v[1:] / v[:-1]
    picks = np.argsort(ratio)[::-1][:count]
    assert np.all(ratio[picks] > 1 + 1e-6)
    return [float(F32(np.sqrt(v[i] * v[i + 1]))) for i in picks]


def _workload(seed, rows, cols):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols)).astype(F32) * np.exp(rng.standard_normal((1, cols))).astype(F32)
    x[:128, :128] *= 3000.0
    x[rng.integers(0, rows, 20), rng.integers(0, cols, 20)] = 700.0
    if rows > 256 and cols > 384:
        x[256:, 384:] = 0.0
    return synth.to_bf16_bits(x)


@pytest.mark.parametrize("which", ["l1", "l1rel"])
@pytest.mark.parametrize("shape", [(384, 512), (300, 520), (128, 128)])
def test_error_selectors_match_oracle(which, shape):
    bits = _workload(shape[0] + shape[1], *shape)
    gcrit, ocrit = CRITS[which]
    metric = _metric(bits, which)
    thetas = _thresholds(metric) if np.unique(metric[metric > 0]).size >= 2 else []
    thetas += [0.0, -1.0, float("inf")]
    xd = gu.to_device_bf16(bits)
    for theta in thetas:
        gu.announce(f"criterion {which} shape={shape} theta={theta}")
        gq = fq.fq_quantize(xd, gcrit, theta, want_transposed=True)
        oq = fqo.quantize(bits, 128, ocrit, theta)
        gu.compare_quantized(gq, oq, f"{which} theta={theta}")


@pytest.mark.parametrize("which", ["l1", "l1rel"])
def test_gemm_on_error_selected_blocks(which):
    wl = synth.config1()
    gcrit, ocrit = CRITS[which]
    theta = _thresholds(_metric(wl.X, which), count=1)[0]
    gu.announce(f"gemm with criterion {which} theta={theta}")
    gx = fq.fq_quantize(gu.to_device_bf16(wl.X), gcrit, theta, want_transposed=True)
    gw = fq.fq_quantize(gu.to_device_bf16(wl.W), fq.FQ_CRIT_NONE, 0.0, want_transposed=True)
    ox = fqo.quantize(wl.X, 128, ocrit, theta)
    ow = fqo.quantize(wl.W, 128, fqo.CRIT_NONE, 0.0)
    gu.compare_quantized(gx, ox, which)
    assert 0 < int(ox.fb_count[0]) < ox.mask.size
    ref = fqo.gemm(fqo.OP_NT, ox, ow)
    got = fq.fq_gemm(fq.FQ_OP_NT, gx, gw).cpu().numpy()
    assert gu.rel_err(got, ref) <= 1e-3
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def test_error_selectors_reuse_and_errors():
    """Switching criteria on one tensor re-points the live counter correctly; an unknown
    criterion is rejected on the host."""
    bits = _workload(5, 256, 256)
    xd = gu.to_device_bf16(bits)
    qt = fq.QTensor(256, 256)
    for crit, ocrit, theta in ((fq.FQ_CRIT_L1_GT, fqo.CRIT_L1_GT, 0.0),
                               (fq.FQ_CRIT_ABSMAX_GT, fqo.CRIT_ABSMAX_GT, 10.0),
                               (fq.FQ_CRIT_L1REL_GT, fqo.CRIT_L1REL_GT, 0.0),
                               (fq.FQ_CRIT_NONE, fqo.CRIT_NONE, 0.0)):
        gu.announce(f"reuse crit={crit}")
        fq.fq_quantize(xd, crit, theta, out=qt)
        gu.compare_quantized(qt, fqo.quantize(bits, 128, ocrit, theta), f"reuse crit={crit}")
    with pytest.raises(fq.FqError) as e:
        fq.fq_quantize(xd, 5, 0.0, out=qt)
    assert e.value.status == fq.FQ_ERR_ENUM
