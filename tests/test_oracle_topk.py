"""Pins for the oracle's TopK AbsMax selection (Sec. 4.4 of the paper: the k blocks with the
largest abs-max fall back).  Checked against things other than the oracle's own loop: a numpy
ordering of abs-max values computed from the input, the threshold criterion with a threshold
placed between the k-th and (k+1)-th value, and the degenerate k."""
import numpy as np
import pytest

from oracle import fqo
from paper_2503_08040_amd import synth

F32 = np.float32


def _same(a, b):
    for f in ("codes", "scales", "mask", "res_codes", "res_scales", "fb_count"):
        x, y = getattr(a, f), getattr(b, f)
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8)), f
    n = int(a.fb_count[0])
    assert np.array_equal(a.fb_list[:n], b.fb_list[:n])


def _block_amax(bits, g):
    x = np.abs(synth.bf16_bits_to_f32(bits))
    rows, cols = x.shape
    nbr, nbc = -(-rows // g), -(-cols // g)
    pad = np.zeros((nbr * g, nbc * g), F32)
    pad[:rows, :cols] = x
    return pad.reshape(nbr, g, nbc, g).max(axis=(1, 3))


def _input(rng, shape, g):
    x = rng.standard_normal(shape).astype(F32)
    # distinct block maxima: one spike per block, all different
    nbr, nbc = -(-shape[0] // g), -(-shape[1] // g)
    spikes = rng.permutation(nbr * nbc).astype(F32) * 3.0 + 8.0
    for b in range(nbr * nbc):
        x[(b // nbc) * g, (b % nbc) * g] = spikes[b]
    return synth.to_bf16_bits(x)


@pytest.mark.parametrize("shape,g", [((64, 96), 16), ((70, 50), 16), ((256, 384), 128)])
def test_topk_is_the_numpy_ordering_and_a_threshold(shape, g):
    rng = np.random.default_rng(shape[0] + g)
    bits = _input(rng, shape, g)
    amax = _block_amax(bits, g)
    nb = amax.size
    order = np.lexsort((np.arange(nb), -amax.ravel()))     # descending, lower index first
    vals = np.sort(amax.ravel())[::-1]
    assert len(np.unique(vals)) == nb                      # no ties in this input
    for k in (1, 2, nb // 3, nb - 1):
        q = fqo.quantize_topk(bits, g, k)
        assert int(q.fb_count[0]) == k == int(q.mask.sum())
        assert np.array_equal(np.flatnonzero(q.mask.ravel()), np.sort(order[:k]))
        assert amax[q.mask.astype(bool)].min() > amax[~q.mask.astype(bool)].max()
        # the same decision as a threshold between the k-th and the (k+1)-th largest value
        theta = float(0.5 * (vals[k - 1] + vals[k]))
        _same(q, fqo.quantize(bits, g, fqo.CRIT_ABSMAX_GT, theta))


def test_topk_degenerate_k():
    rng = np.random.default_rng(3)
    bits = _input(rng, (48, 80), 16)
    nb = 3 * 5
    _same(fqo.quantize_topk(bits, 16, 0), fqo.quantize(bits, 16, fqo.CRIT_NONE, 0.0))
    _same(fqo.quantize_topk(bits, 16, -4), fqo.quantize(bits, 16, fqo.CRIT_NONE, 0.0))
    _same(fqo.quantize_topk(bits, 16, nb), fqo.quantize(bits, 16, fqo.CRIT_ALL, 0.0))
    _same(fqo.quantize_topk(bits, 16, nb + 7), fqo.quantize(bits, 16, fqo.CRIT_ALL, 0.0))
    assert int(fqo.quantize_topk(bits[:0], 16, 3).fb_count[0]) == 0


def test_topk_takes_equal_values_in_block_order():
    """Six blocks share the largest abs-max; k = 4 takes the four with the lowest block ids,
    and an all-zero block is taken only when k reaches it."""
    g = 8
    x = np.zeros((3 * g, 4 * g), F32)
    rng = np.random.default_rng(5)
    x[:] = rng.uniform(-1, 1, x.shape)
    tied = [1, 4, 5, 7, 10, 11]
    for b in tied:
        x[(b // 4) * g + 3, (b % 4) * g + 2] = -9.0
    x[0:g, 0:g] = 0.0                                       # block 0: all zero
    x[2 * g, 0] = 20.0                                      # block 8: the single largest
    bits = synth.to_bf16_bits(x)
    q = fqo.quantize_topk(bits, g, 5)
    assert np.flatnonzero(q.mask.ravel()).tolist() == [1, 4, 5, 7, 8]
    q = fqo.quantize_topk(bits, g, 7)
    assert np.flatnonzero(q.mask.ravel()).tolist() == [1, 4, 5, 7, 8, 10, 11]
    q = fqo.quantize_topk(bits, g, 11)
    assert 0 not in np.flatnonzero(q.mask.ravel()).tolist()
    q = fqo.quantize_topk(bits, g, 12)
    assert q.mask.all() and q.res_scales[0, 0] == 0.0 and not q.res_codes[0:g, 0:g].any()


def test_topk_residual_payload_is_the_two_step_quantization():
    """Flagged blocks carry the residual of Sec. 4.3: |x - (a q + a~ q~)| <= amax / 64516."""
    rng = np.random.default_rng(9)
    g = 16
    bits = _input(rng, (64, 64), g)
    q = fqo.quantize_topk(bits, g, 5)
    x = synth.bf16_bits_to_f32(bits).astype(np.float64)
    a = np.kron(q.scales.astype(np.float64), np.ones((g, g)))
    ra = np.kron(q.res_scales.astype(np.float64), np.ones((g, g)))
    m = np.kron(q.mask, np.ones((g, g), np.uint8)).astype(bool)
    amax = np.kron(_block_amax(bits, g).astype(np.float64), np.ones((g, g)))
    err = np.abs(x - (a * q.codes + ra * q.res_codes))
    assert np.all(err[m] <= amax[m] / 64516 * (1 + 1e-6))
    assert np.all(err[~m] <= amax[~m] / 254 * (1 + 1e-6))
    assert not q.res_codes[~m].any()
