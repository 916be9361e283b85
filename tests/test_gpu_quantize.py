"""GPU parity: fq_quantize against the CPU oracle, bit-exact on every output
(codes, scales, mask, count, list, residual codes and scales through fb_slot,
transposed copies)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2503_08040_amd as fq
from oracle import fqo
from paper_2503_08040_amd import synth
from tests import gpu_util as gu

F32 = np.float32


def _run(bits, crit, theta, want_t=True, capacity=None, label=""):
    gu.announce(f"quantize {label} shape={bits.shape} crit={crit} theta={theta}")
    x = gu.to_device_bf16(bits)
    gq = fq.fq_quantize(x, crit, theta, capacity=capacity, want_transposed=want_t)
    oq = fqo.quantize(bits, 128, crit, theta)
    gu.compare_quantized(gq, oq, label)
    return gq, oq


def test_config1_quantize():
    wl = synth.config1()
    gq, oq = _run(wl.X, fq.FQ_CRIT_ABSMAX_GT, wl.theta, label="cfg1 X")
    assert int(oq.fb_count[0]) == 1 and oq.fb_list[0] == wl.flagged_blocks[0]
    _run(wl.W, fq.FQ_CRIT_NONE, 0.0, label="cfg1 W")
    _run(wl.X, fq.FQ_CRIT_ALL, 0.0, label="cfg1 X all")
    _run(wl.X, fq.FQ_CRIT_NONE, 0.0, want_t=False, label="cfg1 X none")


def test_config4_gradient_quantize():
    wl = synth.config4()
    gq, oq = _run(wl.dY, fq.FQ_CRIT_ABSMAX_GT, wl.theta, label="cfg4 dY")
    assert int(oq.fb_count[0]) == 2


@pytest.mark.parametrize("shape", [(1, 1), (127, 129), (130, 200), (257, 384), (128, 1000), (300, 128)])
@pytest.mark.parametrize("crit", [fq.FQ_CRIT_ABSMAX_GT, fq.FQ_CRIT_ALL])
def test_ragged_shapes(shape, crit):
    rng = np.random.default_rng(shape[0] * 1000 + shape[1])
    x = rng.standard_normal(shape).astype(F32)
    for _ in range(3):
        x[rng.integers(shape[0]), rng.integers(shape[1])] *= 150.0
    _run(synth.to_bf16_bits(x), crit, 8.0, label=f"ragged {shape}")


def test_strided_and_misaligned_input():
    rng = np.random.default_rng(5)
    full = synth.to_bf16_bits(rng.standard_normal((260, 397)).astype(F32) * 3)
    xd = gu.to_device_bf16(full)
    for (r0, c0, rows, cols) in [(0, 0, 256, 384), (3, 5, 200, 300), (1, 8, 256, 256)]:
        gu.announce(f"quantize strided window {(r0, c0, rows, cols)}")
        sub = xd[r0:r0 + rows, c0:c0 + cols]
        gq = fq.fq_quantize(sub, fq.FQ_CRIT_ABSMAX_GT, 9.0, want_transposed=True)
        oq = fqo.quantize(full[r0:r0 + rows, c0:c0 + cols], 128, fqo.CRIT_ABSMAX_GT, 9.0)
        gu.compare_quantized(gq, oq, "strided")


def test_threshold_edge_cases_and_special_values():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((256, 256)).astype(F32)
    x[:128, 128:] = 0.0                       # an all-zero block
    x[128:, 128:] = np.clip(x[128:, 128:], -6, 6)
    x[130, 131] = 6.0                         # amax == theta exactly
    x[128:, :128] *= 1e-37                    # tiny scales
    bits = synth.to_bf16_bits(x)
    sub = rng.integers(0, 128, size=(128, 128)).astype(np.uint16)   # bf16 subnormals m * 2^-133
    sub[5, 7] = 127
    bits[:128, :128] = sub | (rng.integers(0, 2, size=(128, 128)).astype(np.uint16) << 15)
    for theta in (6.0, float(np.nextafter(F32(6.0), F32(0))), -1.0, 0.0, float("inf")):
        gq, oq = _run(bits, fq.FQ_CRIT_ABSMAX_GT, theta, label=f"edge theta={theta}")
    assert oq.scales[0, 0] == F32(2.0 ** -133)


def test_subnormal_scales_need_the_clamp():
    """bf16 subnormals m * 2^-133: scales and residual scales are subnormal binary32 numbers, whole
    multiples of 2^-149 and therefore far from max/127, so quotients leave the code range and are
    clamped (the hand-worked oracle pin, tiled over blocks, plus random subnormal blocks)."""
    rng = np.random.default_rng(12)
    pat = np.array([[3, 1], [1 | 0x8000, 0]], dtype=np.uint16)          # bit patterns: m, sign
    bits = np.tile(pat, (128, 128)).astype(np.uint16)                   # 256 x 256
    rnd = rng.integers(0, 128, size=(128, 256)).astype(np.uint16)
    bits[128:, :] = rnd | (rng.integers(0, 2, size=(128, 256)).astype(np.uint16) << 15)
    gq, oq = _run(bits, fq.FQ_CRIT_ALL, 0.0, label="subnormal clamp")
    assert oq.res_codes.min() == -127 and oq.res_codes.max() == 127
    assert oq.res_scales[0, 0] == F32(4 * 2.0 ** -149)
    # the INT10 context quantizer meets the same situation (a = max / 511)
    packed, scales = fq.fq_ctx_quantize(gu.to_device_bf16(bits))
    o_packed, o_scales = fqo.ctx_quantize(bits)
    assert np.array_equal(packed.cpu().numpy(), o_packed)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), o_scales.view(np.uint32))


def test_extreme_magnitudes():
    """Blocks scaled by 2^k from the subnormal range up to just below the largest finite bf16:
    every code path that treats small and large scales differently (the reciprocal shortcut is
    only taken for scales in [2^-100, 2^100]) must still agree with the oracle bit for bit, for
    nearest and stochastic rounding and for the INT10 contexts."""
    rng = np.random.default_rng(33)
    ks = [-140, -133, -127, -126, -110, -101, -100, -99, -90, -20, 0, 60, 99, 100, 101, 110, 120, 126]
    x = np.zeros((3 * 128, 6 * 128), np.float64)
    for b, k in enumerate(ks):
        bi, bk = divmod(b, 6)
        blk = rng.standard_normal((128, 128)) * 2.0 ** k
        blk[rng.integers(128), rng.integers(128)] = 1.9 * 2.0 ** k
        x[bi * 128:(bi + 1) * 128, bk * 128:(bk + 1) * 128] = blk
    x = np.clip(x, -3.0e38, 3.0e38)
    with np.errstate(under="ignore"):
        bits = synth.to_bf16_bits(x.astype(F32))
    _run(bits, fq.FQ_CRIT_ALL, 0.0, label="extreme magnitudes")
    gq = fq.fq_quantize_sr(gu.to_device_bf16(bits), 99, want_transposed=True)
    gu.compare_quantized(gq, fqo.quantize_sr(bits, 128, 99), "extreme magnitudes, stochastic")
    packed, scales = fq.fq_ctx_quantize(gu.to_device_bf16(bits))
    o_packed, o_scales = fqo.ctx_quantize(bits)
    assert np.array_equal(packed.cpu().numpy(), o_packed)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), o_scales.view(np.uint32))


def test_rounding_ties_on_gpu():
    """Every block holds exact ties k + 0.5 (a = 1): the GPU must round to even."""
    x = np.zeros((128, 256), F32)
    vals = np.arange(-126, 127, dtype=F32) + 0.5
    x[:, :] = np.resize(vals, (128, 256))
    x[0, 0] = 127.0
    x[0, 128] = -127.0
    gq, oq = _run(synth.to_bf16_bits(x), fq.FQ_CRIT_ALL, 0.0, label="ties")
    assert np.array_equal(oq.codes[1, :4], np.rint(x[1, :4]).astype(np.int8))


def test_capacity_overflow_is_reported():
    wl = synth.config1()
    x = gu.to_device_bf16(wl.X)
    gu.announce("quantize with capacity 3 < flagged 8")
    gq = fq.fq_quantize(x, fq.FQ_CRIT_ALL, 0.0, capacity=3)
    with pytest.raises(fq.FqError) as e:
        fq.fq_qtensor_check(gq)
    assert e.value.status == fq.FQ_ERR_CAPACITY
    slot = gq.view("fb_slot").cpu().numpy().ravel()
    assert sorted(slot[slot >= 0].tolist()) == [0, 1, 2] and np.sum(slot == -2) == 5
    assert int(gq.view("fb_count").cpu()[0]) == 8
    assert fq.fq_qtensor_check(fq.fq_quantize(x, fq.FQ_CRIT_ALL, 0.0)) == 8


def test_empty_input():
    x = torch.empty((0, 256), dtype=torch.bfloat16, device="cuda")
    gu.announce("quantize empty")
    gq = fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, 1.0, capacity=0)
    assert fq.fq_qtensor_check(gq) == 0


def test_quantizer_is_deterministic_and_reusable():
    wl = synth.config1()
    x = gu.to_device_bf16(wl.X)
    q = fq.QTensor(256, 512, want_transposed=True)
    gu.announce("quantize twice into the same buffers")
    fq.fq_quantize(x, fq.FQ_CRIT_ALL, 0.0, out=q)
    fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, wl.theta, out=q)
    gu.compare_quantized(q, fqo.quantize(wl.X, 128, fqo.CRIT_ABSMAX_GT, wl.theta), "reuse")


def test_untile_matches_documented_layout():
    wl = synth.config1()
    gq = fq.fq_quantize(gu.to_device_bf16(wl.X[:200, :300].copy()), fq.FQ_CRIT_NONE, 0.0)
    gu.announce("untile kernel")
    dense = fq.fq_codes_to_rowmajor(gq.view("codes"), 200, 300).cpu().numpy()
    want, _ = gu.untile(gq.view("codes").cpu().numpy(), 200, 300)
    assert np.array_equal(dense, want)
