"""Oracle pins for RMS normalization as a non-linear layer with an INT10 context (Sec. 5.2, 5.3).
Checked against numpy formulas written independently, closed forms, and central differences of
the forward map."""
import numpy as np

from oracle import fqo
from paper_2503_08040_amd import synth

F32 = np.float32


def _f(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def _steps(a_bits, b_bits):
    def key(h):
        h = h.astype(np.int64)
        return np.where(h & 0x8000, -(h & 0x7FFF), h & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def _deq(ctx, rows, cols):
    bits = np.unpackbits(ctx[0], axis=-1, bitorder="little").reshape(rows, -1, 128, 10).astype(np.int64)
    q = (bits << np.arange(10)).sum(axis=-1)
    q = np.where(q >= 512, q - 1024, q).astype(F32)
    return (ctx[1][:, :, None] * q).astype(F32).reshape(rows, -1)[:, :cols].astype(np.float64)


def _case(rows=7, cols=300, seed=0):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((rows, cols)) * np.exp(rng.standard_normal((rows, 1)))).astype(F32)
    w = (1.0 + 0.1 * rng.standard_normal(cols)).astype(F32)
    dy = rng.standard_normal((rows, cols)).astype(F32)
    return synth.to_bf16_bits(x), synth.to_bf16_bits(w), synth.to_bf16_bits(dy)


def test_forward_against_numpy_and_closed_forms():
    bx, bw, _ = _case()
    eps = 1e-6
    y, rstd, ctx = fqo.rmsnorm_forward(bx, bw, eps)
    x, w = _f(bx), _f(bw)
    rs = 1.0 / np.sqrt((x * x).mean(axis=1) + eps)
    assert np.array_equal(rstd, rs.astype(F32))
    d = _steps(y, synth.to_bf16_bits((x * rs[:, None] * w).astype(F32)))
    assert d.max() <= 1 and (d == 0).mean() > 0.99
    p, s = fqo.ctx_quantize(bx)
    assert np.array_equal(ctx[0], p) and np.array_equal(ctx[1], s)
    # a constant row of value v with unit gain normalizes to sign(v) (eps = 0), rstd = 1/|v|
    c = synth.to_bf16_bits(np.full((2, 256), -4.0, F32))
    one = synth.to_bf16_bits(np.ones(256, F32))
    y2, rstd2, _ = fqo.rmsnorm_forward(c, one, 0.0)
    assert np.all(_f(y2) == -1.0) and np.all(rstd2 == 0.25)
    # an all-zero row: rstd = 1/sqrt(eps), y = 0
    z = synth.to_bf16_bits(np.zeros((1, 128), F32))
    y3, rstd3, _ = fqo.rmsnorm_forward(z, synth.to_bf16_bits(np.ones(128, F32)), 1e-4)
    assert np.all(_f(y3) == 0.0) and np.isclose(rstd3[0], 100.0, rtol=1e-6)
    # the output of a row has unit mean square (gain 1, eps -> 0) up to bf16 rounding
    y4, _, _ = fqo.rmsnorm_forward(bx, synth.to_bf16_bits(np.ones(300, F32)), 0.0)
    assert np.allclose((_f(y4) ** 2).mean(axis=1), 1.0, rtol=5e-3)


def test_backward_is_the_gradient_of_the_forward_map():
    """dx and dw against central differences of L = sum(dy * y(x~, w)) taken at the dequantized
    context x~ with rstd recomputed from x~ (the stored rstd is passed as rstd(x~) for this check)."""
    bx, bw, bdy = _case(rows=3, cols=200, seed=1)
    eps = 1e-5
    _, _, ctx = fqo.rmsnorm_forward(bx, bw, eps)
    xq = _deq(ctx, 3, 200)
    w, dy = _f(bw), _f(bdy)
    rs = (1.0 / np.sqrt((xq * xq).mean(axis=1) + eps))
    dx, dw = fqo.rmsnorm_backward(bdy, ctx, rs.astype(F32), bw)
    rs32 = rs.astype(F32).astype(np.float64)

    def loss(xv, wv):
        r = 1.0 / np.sqrt((xv * xv).mean(axis=1, keepdims=True) + eps)
        return (dy * xv * r * wv).sum()

    h = 1e-6
    gx = np.zeros_like(xq)
    for i in range(3):
        for j in range(0, 200, 7):           # a sample of the columns
            e = np.zeros_like(xq); e[i, j] = h
            gx[i, j] = (loss(xq + e, w) - loss(xq - e, w)) / (2 * h)
    got = _f(dx)
    cols = np.arange(0, 200, 7)
    assert np.allclose(got[:, cols], gx[:, cols], rtol=2.0 ** -7, atol=2e-3 * np.abs(gx).max())
    gw = np.zeros(200)
    for j in range(0, 200, 5):
        e = np.zeros(200); e[j] = h
        gw[j] = (loss(xq, w + e) - loss(xq, w - e)) / (2 * h)
    cw = np.arange(0, 200, 5)
    assert np.allclose(dw[cw], gw[cw], rtol=1e-4, atol=1e-5 * np.abs(gw).max())
    # closed form written with numpy
    xh = xq * rs32[:, None]
    g = dy * w
    want_dx = rs32[:, None] * (g - xh * (g * xh).mean(axis=1, keepdims=True))
    d = _steps(dx, synth.to_bf16_bits(want_dx.astype(F32)))
    assert d.max() <= 1 and (d == 0).mean() > 0.98
    assert np.allclose(dw, (dy * xh).sum(axis=0), rtol=1e-6, atol=1e-6)


def test_backward_properties():
    """dx of every row is orthogonal to xh (the normalization removes the radial direction), and
    dw sums over rows."""
    bx, bw, bdy = _case(rows=6, cols=384, seed=2)
    _, rstd, ctx = fqo.rmsnorm_forward(bx, bw, 0.0)
    dx, dw = fqo.rmsnorm_backward(bdy, ctx, rstd, bw)
    xh = _deq(ctx, 6, 384) * rstd.astype(np.float64)[:, None]
    # with eps = 0 and rstd taken at x (not x~) orthogonality holds up to the context error
    dots = (_f(dx) * xh).sum(axis=1) / (np.abs(_f(dx)) * np.abs(xh)).sum(axis=1)
    assert np.all(np.abs(dots) < 2e-2)
    dx1, dw1 = fqo.rmsnorm_backward(bdy[:3], (ctx[0][:3], ctx[1][:3]), rstd[:3], bw)
    dx2, dw2 = fqo.rmsnorm_backward(bdy[3:], (ctx[0][3:], ctx[1][3:]), rstd[3:], bw)
    assert np.array_equal(np.vstack([dx1, dx2]), dx)
    assert np.allclose(dw1 + dw2, dw, rtol=1e-6, atol=1e-7)
