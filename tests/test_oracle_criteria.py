"""Oracle pins for the error-based fallback selectors of Sec. 4.4: L1 = sum|G - Q(G)| and
L1-Rel = L1 / sum|G|, each compared with theta.  The metric is recomputed here with numpy from
the oracle's codes and scales (not from its metric code), and thresholds sit in gaps between
the blocks' metric values so that the decision does not hinge on the last bits of a sum."""
import numpy as np
import pytest

from oracle import fqo
from paper_2503_08040_amd import synth

F32 = np.float32


def _blocks(rows, cols, g=128):
    for bi in range(-(-rows // g)):
        for bk in range(-(-cols // g)):
            yield bi, bk, slice(bi * g, min(rows, bi * g + g)), slice(bk * g, min(cols, bk * g + g))


def _metrics(bits, q):
    """Per-block (L1, sum|x|) in float64 from codes and scales: the residual x - a*q is exact in
    binary64 (a*q has at most 31 significant bits), rounded once to binary32 like fmaf."""
    x = synth.bf16_bits_to_f32(bits).astype(np.float64)
    rows, cols = x.shape
    l1 = np.zeros((q.nbr, q.nbc))
    l1x = np.zeros((q.nbr, q.nbc))
    for bi, bk, rs, cs in _blocks(rows, cols):
        r = (x[rs, cs] - float(q.scales[bi, bk]) * q.codes[rs, cs].astype(np.float64)).astype(F32)
        l1[bi, bk] = np.abs(r.astype(np.float64)).sum()
        l1x[bi, bk] = np.abs(x[rs, cs]).sum()
    return l1, l1x


def _gap_threshold(values, widest=True):
    """A threshold inside a relative gap between sorted distinct positive metric values: the
    widest gap, or the narrowest one that is still wider than 1e-3."""
    v = np.unique(values[values > 0])
    assert v.size >= 2
    ratio = v[1:] / v[:-1]
    i = int(np.argmax(ratio)) if widest else int(np.argmin(np.where(ratio > 1.001, ratio, np.inf)))
    return F32(np.sqrt(v[i] * v[i + 1])), v[i], v[i + 1]


def _input(seed=0, rows=300, cols=520):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols)).astype(F32)
    x[:128, :128] *= 4000.0                 # a uniformly large block: largest L1, ordinary L1-Rel
    x[130:140, 300] = 900.0                 # a few outliers: the bulk rounds to 0, largest L1-Rel
    x[260:, 384:] = 0.0                     # an all-zero (ragged) block
    return synth.to_bf16_bits(x)


@pytest.mark.parametrize("crit", [fqo.CRIT_L1_GT, fqo.CRIT_L1REL_GT])
def test_mask_is_metric_above_threshold(crit):
    bits = _input()
    base = fqo.quantize(bits, 128, fqo.CRIT_NONE, 0.0)
    l1, l1x = _metrics(bits, base)
    metric = l1 if crit == fqo.CRIT_L1_GT else np.where(l1x > 0, l1 / np.maximum(l1x, 1e-300), 0.0)
    theta, lo, hi = _gap_threshold(metric)
    assert hi / lo > 1.0001                 # the threshold is well inside a gap
    q = fqo.quantize(bits, 128, crit, float(theta))
    want = metric > float(theta)
    assert np.array_equal(q.mask.astype(bool), want)
    assert 0 < want.sum() < want.size
    assert int(q.fb_count[0]) == int(want.sum())
    # everything but the decision is the same two-step quantization as with any other selector
    ref = fqo.quantize(bits, 128, fqo.CRIT_ALL, 0.0)
    assert np.array_equal(q.codes, ref.codes) and np.array_equal(q.scales, ref.scales)
    for bi, bk, rs, cs in _blocks(*bits.shape):
        if want[bi, bk]:
            assert np.array_equal(q.res_codes[rs, cs], ref.res_codes[rs, cs])
            assert q.res_scales[bi, bk] == ref.res_scales[bi, bk]
        else:
            assert not q.res_codes[rs, cs].any() and q.res_scales[bi, bk] == 0.0


def test_selectors_rank_blocks_differently():
    """The uniformly large block has the largest abs-max and L1 but an ordinary L1-Rel; the block
    with a few outliers, whose bulk rounds to zero, has the largest L1-Rel."""
    bits = _input()
    base = fqo.quantize(bits, 128, fqo.CRIT_NONE, 0.0)
    l1, l1x = _metrics(bits, base)
    rel = l1 / np.maximum(l1x, 1e-300)
    assert np.unravel_index(np.argmax(l1), l1.shape) == (0, 0)
    assert np.unravel_index(np.argmax(rel), rel.shape) == (1, 2)
    assert np.unravel_index(np.argmax(base.scales), rel.shape) == (0, 0)
    assert rel[1, 2] > 0.5 and rel[0, 0] < 0.05


def test_exactly_representable_block_has_zero_error():
    """x = a*q exactly (integers with abs-max 127): L1 = 0, so no threshold >= 0 flags the block
    however large its abs-max is, while the abs-max selector does."""
    rng = np.random.default_rng(1)
    x = rng.integers(-127, 128, size=(128, 256)).astype(F32)
    x[0, 0] = 127.0
    x[0, 128] = -127.0
    x *= 64.0
    bits = synth.to_bf16_bits(x)
    assert np.array_equal(synth.bf16_bits_to_f32(bits), x)
    for crit in (fqo.CRIT_L1_GT, fqo.CRIT_L1REL_GT):
        assert not fqo.quantize(bits, 128, crit, 0.0).mask.any()
        assert fqo.quantize(bits, 128, crit, -1.0).mask.all()      # 0 > -1
    assert fqo.quantize(bits, 128, fqo.CRIT_ABSMAX_GT, 100.0).mask.all()


def test_scaling_by_a_power_of_two():
    """Multiplying the input by 2^k multiplies L1 by 2^k and leaves L1-Rel unchanged."""
    bits = _input(seed=2)
    x = synth.bf16_bits_to_f32(bits)
    bits4 = synth.to_bf16_bits((x * F32(4.0)).astype(F32))
    base = fqo.quantize(bits, 128, fqo.CRIT_NONE, 0.0)
    l1, l1x = _metrics(bits, base)
    rel = np.where(l1x > 0, l1 / np.maximum(l1x, 1e-300), 0.0)
    t1, lo, hi = _gap_threshold(l1, widest=False)
    assert hi / lo < 4.0
    tr, _, _ = _gap_threshold(rel)
    m1 = fqo.quantize(bits, 128, fqo.CRIT_L1_GT, float(t1)).mask
    assert np.array_equal(fqo.quantize(bits4, 128, fqo.CRIT_L1_GT, float(t1) * 4).mask, m1)
    assert not np.array_equal(fqo.quantize(bits4, 128, fqo.CRIT_L1_GT, float(t1)).mask, m1)
    mr = fqo.quantize(bits, 128, fqo.CRIT_L1REL_GT, float(tr)).mask
    assert np.array_equal(fqo.quantize(bits4, 128, fqo.CRIT_L1REL_GT, float(tr)).mask, mr)


def test_all_zero_block_is_never_flagged_by_the_relative_selector():
    bits = synth.to_bf16_bits(np.zeros((128, 128), F32))
    assert not fqo.quantize(bits, 128, fqo.CRIT_L1REL_GT, -1.0).mask.any()
    assert fqo.quantize(bits, 128, fqo.CRIT_L1_GT, -1.0).mask.all()
