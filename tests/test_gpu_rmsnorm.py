"""GPU parity for RMS normalization with a fused INT10 context (Sec. 5.2, 5.3).

The context is pure quantization of x and must match the oracle bit for bit.  rstd, y, dx and dw
are binary32 arithmetic on the GPU and binary64 in the oracle; the tolerances below are what that
arithmetic gives: rstd within a few binary32 ulps, bf16 outputs at most one bf16 step apart and
equal almost everywhere (with an absolute floor for dx, whose bracket g - xh*mean cancels), dw
within 1e-5 of the sum of the magnitudes it adds up.  The backward pass is checked with the GPU's
own rstd handed to the oracle, so that only the arithmetic differs."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2503_08040_amd as fq
from oracle import fqo
from paper_2503_08040_amd import synth
from tests import gpu_util as gu

F32 = np.float32


def _f(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def _bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _steps(a_bits, b_bits):
    def key(h):
        h = h.astype(np.int64)
        return np.where(h & 0x8000, -(h & 0x7FFF), h & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def _close(got_bits, ref_bits, abs_floor, label, min_exact=0.99):
    d = _steps(got_bits, ref_bits)
    bad = (d > 1) & (np.abs(_f(got_bits) - _f(ref_bits)) > abs_floor)
    assert not bad.any(), f"{label}: {int(bad.sum())} elements beyond one bf16 step"
    exact = ((d == 0) | (np.abs(_f(got_bits) - _f(ref_bits)) <= abs_floor)).mean()
    assert exact > min_exact, f"{label}: only {exact:.4f} of the elements equal the oracle's"


def _case(rows, cols, seed):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((rows, cols)) * np.exp(rng.standard_normal((rows, 1)))).astype(F32)
    x.flat[rng.integers(0, x.size, size=max(1, x.size // 400))] *= 40.0
    w = (1.0 + 0.2 * rng.standard_normal(cols)).astype(F32)
    dy = (rng.standard_t(3.0, size=(rows, cols)) * 1e-2).astype(F32)
    return tuple(synth.to_bf16_bits(v) for v in (x, w, dy))


@pytest.mark.parametrize("shape,parts", [((64, 512), 16), ((33, 300), 7), ((1, 1), 1), ((5, 4097), 3),
                                          ((300, 136), 256), ((9, 11008), 4), ((2, 16384), 5), ((3, 20000), 2),
                                          # 16-byte rows whose last group is ragged; one, two and three
                                          # 4096-column chunks; fewer rows than parts
                                          ((37, 4112), 5), ((21, 11024), 4), ((12, 12288), 3), ((3, 2048), 8),
                                          ((70, 8192), 8), ((1, 4096), 1)])
def test_rmsnorm_forward_backward(shape, parts):
    rows, cols = shape
    bx, bw, bdy = _case(rows, cols, seed=rows + cols)
    eps = 1e-5
    gu.announce(f"rmsnorm forward shape={shape}")
    wd = gu.to_device_bf16(bw.reshape(1, -1)).reshape(-1)
    y, rstd, ctx = fq.fq_rmsnorm_forward(gu.to_device_bf16(bx), wd, eps)
    torch.cuda.synchronize()
    oy, orstd, octx = fqo.rmsnorm_forward(bx, bw, eps)
    assert np.array_equal(ctx[0].cpu().numpy(), octx[0]), "context: packed bytes"
    assert np.array_equal(ctx[1].cpu().numpy().view(np.uint32), octx[1].view(np.uint32)), "context: scales"
    grstd = rstd.cpu().numpy()
    assert np.allclose(grstd, orstd, rtol=2e-6, atol=0), "rstd"
    _close(_bits(y), oy, 0.0, "y")
    gu.announce(f"rmsnorm backward shape={shape} parts={parts}")
    dx, dw = fq.fq_rmsnorm_backward(gu.to_device_bf16(bdy), ctx, rstd, wd, n_parts=parts)
    torch.cuda.synchronize()
    odx, odw = fqo.rmsnorm_backward(bdy, octx, grstd, bw)
    xq = _f(fqo.ctx_dequantize(octx[0], octx[1], rows, cols))
    # floor for dx: the bracket g - xh * m is formed in binary32
    xh = np.abs(xq) * grstd.astype(np.float64)[:, None]
    g = np.abs(_f(bdy) * _f(bw))
    m = np.abs((_f(bdy) * _f(bw) * xq * grstd.astype(np.float64)[:, None]).mean(axis=1, keepdims=True))
    floor = 2.0 ** -18 * grstd.astype(np.float64)[:, None] * (g + xh * m + np.abs(g * xh).mean(axis=1, keepdims=True))
    _close(_bits(dx), odx, floor, "dx", min_exact=0.98)
    mag = (np.abs(_f(bdy)) * xh).sum(axis=0)
    assert np.all(np.abs(dw.cpu().numpy().astype(np.float64) - odw) <= 1e-5 * mag + 1e-30), "dw"
    # end to end: the oracle's backward on the oracle's own forward outputs (its rstd, not the
    # GPU's).  The two rstd agree to 2e-6, which the floor of the bracket is widened by.
    odx2, odw2 = fqo.rmsnorm_backward(bdy, octx, orstd, bw)
    _close(_bits(dx), odx2, 4.0 * floor, "dx (oracle rstd)", min_exact=0.98)
    assert np.all(np.abs(dw.cpu().numpy().astype(np.float64) - odw2) <= 1.2e-5 * mag + 1e-30), "dw (oracle rstd)"


def test_rmsnorm_strides_determinism_and_errors():
    rows, cols, ld = 40, 384, 400
    rng = np.random.default_rng(9)
    bx = synth.to_bf16_bits(rng.standard_normal((rows, ld)).astype(F32))
    bw = synth.to_bf16_bits(np.ones(cols, F32))
    xd = gu.to_device_bf16(bx)
    wd = gu.to_device_bf16(bw.reshape(1, -1)).reshape(-1)
    for off in (0, 5):                     # aligned and unaligned views, pitch > cols
        gu.announce(f"rmsnorm strided off={off}")
        sub = np.ascontiguousarray(bx[:, off:off + cols])
        y, rstd, ctx = fq.fq_rmsnorm_forward(xd[:, off:off + cols], wd, 1e-6)
        torch.cuda.synchronize()
        oy, orstd, octx = fqo.rmsnorm_forward(sub, bw, 1e-6)
        assert np.array_equal(ctx[0].cpu().numpy(), octx[0])
        assert np.allclose(rstd.cpu().numpy(), orstd, rtol=2e-6)
        _close(_bits(y), oy, 0.0, f"y off={off}")
    dy = gu.to_device_bf16(synth.to_bf16_bits(rng.standard_normal((rows, cols)).astype(F32)))
    a = fq.fq_rmsnorm_backward(dy, ctx, rstd, wd, n_parts=8)
    b = fq.fq_rmsnorm_backward(dy, ctx, rstd, wd, n_parts=8)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])      # deterministic
    c = fq.fq_rmsnorm_backward(dy, ctx, rstd, wd, n_parts=3)
    assert torch.equal(a[0], c[0]) and torch.allclose(a[1], c[1], rtol=1e-5, atol=1e-6)
    import ctypes as C
    L = fq.lib()
    p = C.c_void_p(y.data_ptr())
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.fq_rmsnorm_forward(None, p, 4, 128, 128, C.c_float(0), p, 128, p, p, p, st) == fq.FQ_ERR_NULL
    assert L.fq_rmsnorm_forward(p, p, 4, 0, 128, C.c_float(0), p, 128, p, p, p, st) == fq.FQ_ERR_SHAPE
    assert L.fq_rmsnorm_forward(p, p, 4, 128, 64, C.c_float(0), p, 128, p, p, p, st) == fq.FQ_ERR_SHAPE
    assert L.fq_rmsnorm_backward(p, 128, p, p, p, p, 4, 128, p, 128, p, p, 0, st) == fq.FQ_ERR_SHAPE
    assert L.fq_rmsnorm_backward(p, 128, p, p, p, p, 4, 128, p, 128, None, p, 4, st) == fq.FQ_ERR_NULL
    # no rows: dw is written as zeros
    dw = torch.full((128,), 7.0, dtype=torch.float32, device="cuda")
    parts = torch.empty((2 * 128,), dtype=torch.float32, device="cuda")
    assert L.fq_rmsnorm_backward(None, 128, None, None, None, None, 0, 128, None, 128,
                                 C.c_void_p(dw.data_ptr()), C.c_void_p(parts.data_ptr()), 2, st) == fq.FQ_OK
    torch.cuda.synchronize()
    assert torch.all(dw == 0).item()


@pytest.mark.parametrize("cols,ld,off", [(4112, 4224, 0), (4112, 4224, 8), (4112, 4224, 3), (8192, 8196, 0)])
def test_rmsnorm_backward_pitched(cols, ld, off):
    """dy and dx as column windows of wider matrices: 16-byte pitch and offset (the two-team
    kernel), a pitch or offset that is not (the general kernel); both against the contiguous call."""
    rows = 45
    bx, bw, bdy = _case(rows, cols, seed=cols + off)
    wd = gu.to_device_bf16(bw.reshape(1, -1)).reshape(-1)
    y, rstd, ctx = fq.fq_rmsnorm_forward(gu.to_device_bf16(bx), wd, 1e-5)
    dy = gu.to_device_bf16(bdy)
    gu.announce(f"rmsnorm backward pitched cols={cols} ld={ld} off={off}")
    ref_dx, ref_dw = fq.fq_rmsnorm_backward(dy, ctx, rstd, wd, n_parts=6)
    wide = torch.zeros((rows, ld), dtype=torch.bfloat16, device="cuda")
    wide[:, off:off + cols] = dy
    out = torch.full((rows, ld), 7.0, dtype=torch.bfloat16, device="cuda")
    dw = torch.empty((cols,), dtype=torch.float32, device="cuda")
    fq.fq_rmsnorm_backward_static(wide[:, off:off + cols], ctx, rstd, wd, out[:, off:off + cols], dw, n_parts=6)
    torch.cuda.synchronize()
    got = out[:, off:off + cols]
    assert (out[:, :off] == 7.0).all().item() and (out[:, off + cols:] == 7.0).all().item()
    if off % 8 == 0 and ld % 8 == 0:
        assert torch.equal(got, ref_dx)          # the same kernel: the same bits
    else:
        # the general kernel sums a row's mean in another order: a last-place difference in the
        # mean moves few dx values by one bf16 step
        differ = (got != ref_dx)
        assert differ.float().mean().item() < 0.01
        assert ((got.float() - ref_dx.float()).abs() <= 2.0 ** -7 * ref_dx.float().abs() + 1e-30).all().item()
    assert torch.allclose(dw, ref_dw, rtol=1e-5, atol=1e-6)
