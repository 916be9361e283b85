"""GPU parity for the 1 x 128 group INT10 context compression (Sec. 5.2, 5.3): packed bytes,
scales and dequantized bf16 values are compared bit for bit with the oracle's, through the C ABI."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2503_08040_amd as fq
from oracle import fqo
from paper_2503_08040_amd import synth
from tests import gpu_util as gu

F32 = np.float32


def _roundtrip(bits, label, x_dev=None):
    rows, cols = bits.shape
    gu.announce(f"ctx {label} shape={bits.shape}")
    x = gu.to_device_bf16(bits) if x_dev is None else x_dev
    packed, scales = fq.fq_ctx_quantize(x)
    back = fq.fq_ctx_dequantize(packed, scales, rows, cols)
    torch.cuda.synchronize()
    o_packed, o_scales = fqo.ctx_quantize(bits)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), o_scales.view(np.uint32)), \
        f"{label}: scales differ"
    assert np.array_equal(packed.cpu().numpy(), o_packed), f"{label}: packed bytes differ"
    o_back = fqo.ctx_dequantize(o_packed, o_scales, rows, cols)
    got = back.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, o_back), f"{label}: dequantized values differ"
    return packed, scales, back


@pytest.mark.parametrize("shape", [(256, 512), (33, 300), (1, 1), (5, 127), (3, 129), (64, 1001),
                                   (17, 2048), (2, 16), (300, 8)])
def test_ctx_bit_exact(shape):
    rng = np.random.default_rng(shape[0] * 7 + shape[1])
    x = rng.standard_normal(shape).astype(F32) * np.exp(rng.standard_normal((shape[0], 1))).astype(F32)
    x.flat[rng.integers(0, x.size, size=max(1, x.size // 500))] *= 100.0
    _roundtrip(synth.to_bf16_bits(x), f"normal+outliers {shape}")


def test_ctx_ties_zero_groups_and_subnormals():
    rows, cols = 8, 384
    x = np.zeros((rows, cols), F32)
    x[0, :128] = np.arange(128, dtype=F32) * 1.0 - 64.0      # small integers next to one large value
    x[0, 5] = 1024.0
    x[1, 128:256] = 3.0                                      # one constant group, neighbours all zero
    x[2, :] = 1e-40                                          # bf16 subnormal
    x[3, 256:] = -np.linspace(0, 7, 128, dtype=F32)
    x[4, ::2] = 2.5
    x[4, 1] = 5.0
    bits = synth.to_bf16_bits(x)
    packed, scales, back = _roundtrip(bits, "ties/zeros/subnormals")
    s = scales.cpu().numpy()
    assert s[1, 0] == 0.0 and s[1, 2] == 0.0 and s[5, 1] == 0.0
    assert not packed.cpu().numpy()[5:].any()


def test_ctx_strided_input_and_output():
    rng = np.random.default_rng(3)
    rows, cols, ld = 70, 200, 264
    x = rng.standard_normal((rows, ld)).astype(F32)
    bits = synth.to_bf16_bits(x)
    xd = gu.to_device_bf16(bits)
    # 16-byte aligned pitch and an unaligned one (column offset 3)
    for off in (0, 3):
        view = xd[:, off:off + cols]
        sub = np.ascontiguousarray(bits[:, off:off + cols])
        packed, scales, _ = _roundtrip(sub, f"strided off={off}", x_dev=view)
        out = torch.full((rows, ld), -1.0, dtype=torch.bfloat16, device="cuda")
        fq.fq_ctx_dequantize(packed, scales, rows, cols, out=out[:, off:off + cols])
        torch.cuda.synchronize()
        full = out.view(torch.int16).cpu().numpy().view(np.uint16)
        want = fqo.ctx_dequantize(*fqo.ctx_quantize(sub), rows, cols)
        assert np.array_equal(full[:, off:off + cols], want)
        rest = np.delete(full, np.s_[off:off + cols], axis=1)
        assert np.all(rest == 0xBF80), "dequantize wrote outside its window"


def test_ctx_glu_activation_shape():
    """The up/gate activation of workload config 3 (what a SiLU-GLU layer would keep), a slice the
    oracle finishes quickly, plus the 5/8 size claim of Sec. 5.2 on the full shape."""
    wl = synth.config3()
    bits = np.ascontiguousarray(wl.X[:192])
    _roundtrip(bits, "cfg3 activation rows 0..191")
    rows, cols = wl.X.shape
    assert (fq.fq_ctx_packed_bytes(rows, cols)) * 8 == rows * (-(-cols // 128)) * 128 * 2 * 5


def test_ctx_empty_and_errors():
    L = fq.lib()
    z = torch.empty((0, 256), dtype=torch.bfloat16, device="cuda")
    p, s = fq.fq_ctx_quantize(z)
    assert p.numel() == 0 and s.numel() == 0
    assert fq.fq_ctx_packed_bytes(-1, 4) == 0 and fq.fq_ctx_packed_bytes(4, 129) == 4 * 2 * 160
    x = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    pk = torch.zeros(4 * 160 + 4, dtype=torch.uint8, device="cuda")
    sc = torch.zeros(4, dtype=torch.float32, device="cuda")
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    xp, pp, sp = C.c_void_p(x.data_ptr()), C.c_void_p(pk.data_ptr()), C.c_void_p(sc.data_ptr())
    assert L.fq_ctx_quantize(None, 4, 128, 128, pp, sp, st) == fq.FQ_ERR_NULL
    assert L.fq_ctx_quantize(xp, 4, 128, 128, None, sp, st) == fq.FQ_ERR_NULL
    assert L.fq_ctx_quantize(xp, 4, 128, 127, pp, sp, st) == fq.FQ_ERR_SHAPE
    assert L.fq_ctx_quantize(xp, -4, 128, 128, pp, sp, st) == fq.FQ_ERR_SHAPE
    assert L.fq_ctx_quantize(xp, 4, 128, 128, C.c_void_p(pk.data_ptr() + 1), sp, st) == fq.FQ_ERR_SHAPE
    assert L.fq_ctx_dequantize(pp, sp, 4, 128, None, 128, st) == fq.FQ_ERR_NULL
    assert L.fq_ctx_dequantize(pp, sp, 4, 128, xp, 100, st) == fq.FQ_ERR_SHAPE
    assert L.fq_ctx_quantize(xp, 4, 128, 128, pp, sp, st) == fq.FQ_OK
    torch.cuda.synchronize()
