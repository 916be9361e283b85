"""Oracle pins for the 1 x 128 group INT10 activation-context compression (Sec. 5.2, 5.3)."""
import numpy as np

from oracle import fqo
from paper_2503_08040_amd import synth

F32 = np.float32


def _unpack(packed):
    """Independent unpacking with numpy bit operations: [rows, ng, 160] bytes -> [rows, ng, 128] ints."""
    bits = np.unpackbits(packed, axis=-1, bitorder="little")          # [rows, ng, 1280]
    vals = bits.reshape(*packed.shape[:2], 128, 10).astype(np.int64)
    q = (vals << np.arange(10)).sum(axis=-1)
    return np.where(q >= 512, q - 1024, q)


def test_size_is_five_eighths_of_bf16():
    rows, cols = 7, 512
    packed, scales = fqo.ctx_quantize(synth.to_bf16_bits(np.ones((rows, cols), F32)))
    assert packed.size * 8 == rows * cols * 2 * 5          # 5/8 of the bf16 bytes (Sec. 5.2)
    assert scales.shape == (rows, cols // 128)


def test_codes_error_bound_and_round_trip():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((33, 300)).astype(F32) * np.exp(rng.standard_normal((33, 1))).astype(F32)
    x[5, 130] = 80.0
    xb = synth.to_bf16_bits(x)
    xf = synth.bf16_bits_to_f32(xb).astype(np.float64)
    packed, scales = fqo.ctx_quantize(xb)
    q = _unpack(packed)
    assert np.abs(q).max() <= 511
    qq = q.reshape(33, -1)[:, :300]
    assert not q.reshape(33, -1)[:, 300:].any()              # ragged tail is zero
    a = np.repeat(scales.astype(np.float64), 128, axis=1)[:, :300]
    amax = np.zeros((33, 3))
    for j in range(3):
        amax[:, j] = np.abs(xf[:, j * 128:(j + 1) * 128]).max(axis=1)
    assert np.array_equal(scales, (amax.astype(F32) / F32(511)).astype(F32))
    err = np.abs(xf - a * qq)
    # |x - a q| <= a/2 with a = amax/511 (slack: x/a is rounded to binary32 before rounding to an integer)
    assert np.all(err <= 0.5 * a * (1 + 2e-4))
    # every group's largest element maps to +-511
    for j in range(3):
        g = np.abs(qq[:, j * 128:(j + 1) * 128]).max(axis=1)
        assert np.all(g[amax[:, j] > 0] == 511)
    # dequantization = a*q rounded to bf16 (numpy rounding as the independent check)
    back = fqo.ctx_dequantize(packed, scales, 33, 300)
    want = synth.to_bf16_bits((scales.repeat(128, axis=1)[:, :300] * qq.astype(F32)).astype(F32))
    assert np.array_equal(back, want)
    rel = np.abs(synth.bf16_bits_to_f32(back) - xf).max() / np.abs(xf).max()
    assert rel < 2.0 ** -8                                    # 10 bits + bf16 rounding


def test_codes_are_nearest_integers_and_special_groups():
    """Away from ties the code is the integer nearest to x/a evaluated in fp64.  (511 is not a
    bf16 number, so a scale is never a power of two and exact ties cannot be constructed.)"""
    rng = np.random.default_rng(2)
    xb = synth.to_bf16_bits(rng.standard_normal((16, 256)).astype(F32))
    xf = synth.bf16_bits_to_f32(xb).astype(np.float64)
    packed, scales = fqo.ctx_quantize(xb)
    q = _unpack(packed).reshape(16, 256)
    t = xf / np.repeat(scales.astype(np.float64), 128, axis=1)
    clear = np.abs(t - np.floor(t) - 0.5) > 1e-3
    assert clear.mean() > 0.99
    assert np.array_equal(q[clear], np.rint(t[clear]).astype(np.int64))
    # a group holding one non-zero value: that value maps to +-511 and comes back exactly
    one = np.zeros((2, 128), F32)
    one[0, 17], one[1, 99] = 3.0, -0.0625
    p1, s1 = fqo.ctx_quantize(synth.to_bf16_bits(one))
    u = _unpack(p1)
    assert u[0, 0, 17] == 511 and u[1, 0, 99] == -511 and np.count_nonzero(u) == 2
    back = synth.bf16_bits_to_f32(fqo.ctx_dequantize(p1, s1, 2, 128))
    assert np.array_equal(back, one)
    z, zs = fqo.ctx_quantize(synth.to_bf16_bits(np.zeros((3, 128), F32)))
    assert not z.any() and not zs.any()
    assert not fqo.ctx_dequantize(z, zs, 3, 128).any()


def test_ten_bits_beat_eight_bits_by_four():
    """The point of INT10 (Sec. 5.2): 4x finer grid than INT8 at the same group size."""
    rng = np.random.default_rng(1)
    xb = synth.to_bf16_bits(rng.standard_normal((64, 256)).astype(F32))
    xf = synth.bf16_bits_to_f32(xb).astype(np.float64)
    packed, scales = fqo.ctx_quantize(xb)
    e10 = np.abs(xf - np.repeat(scales.astype(np.float64), 128, axis=1) * _unpack(packed).reshape(64, -1)).mean()
    amax = np.abs(xf.reshape(64, 2, 128)).max(axis=2, keepdims=True)
    e8 = np.abs(xf.reshape(64, 2, 128) - np.rint(xf.reshape(64, 2, 128) / (amax / 127)) * (amax / 127)).mean()
    assert 3.5 < e8 / e10 < 4.5
