"""Oracle pins for the SiLU-gated linear unit as a non-linear layer with INT10 contexts
(Sec. 4.1: y = sigma(x1) x2; Sec. 5.2 / 5.3: bf16 in and out, 1 x 128 INT10 contexts, dequantized
in the backward pass).  The checks use formulas written differently from the oracle's (tanh form
of the logistic function, central differences of the forward map, numpy rounding to bf16)."""
import numpy as np

from oracle import fqo
from paper_2503_08040_amd import synth

F32 = np.float32


def _f(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def _silu(x):
    return x * 0.5 * (1.0 + np.tanh(0.5 * x))          # x * logistic(x), tanh form


def _ulp_distance(a_bits, b_bits):
    """Distance in bf16 steps between two arrays of bf16 bit patterns (sign-magnitude aware)."""
    def key(h):
        h = h.astype(np.int64)
        return np.where(h & 0x8000, -(h & 0x7FFF), h & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def _inputs(rows=9, cols=300, seed=0):
    rng = np.random.default_rng(seed)
    x1 = (rng.standard_normal((rows, cols)) * 3).astype(F32)
    x2 = (rng.standard_normal((rows, cols)) * 2).astype(F32)
    x1[0, :6] = [0.0, -0.0, 40.0, -40.0, 1e-3, -1.278]
    return synth.to_bf16_bits(x1), synth.to_bf16_bits(x2)


def test_forward_values_and_contexts():
    b1, b2 = _inputs()
    y, c1, c2 = fqo.glu_forward(b1, b2)
    want = synth.to_bf16_bits((_silu(_f(b1)) * _f(b2)).astype(F32))   # double rounding: <= 1 step off
    ok = np.abs(_f(b1)) < 15            # the tanh form loses its accuracy far in the negative tail
    d = _ulp_distance(y, want)[ok]
    assert d.max() <= 1 and (d == 0).mean() > 0.99
    # closed forms: silu(0) = 0, silu(x) -> x for large x, -> 0 for very negative x
    x2 = _f(b2)
    assert y[0, 0] in (0x0000, 0x8000) and y[0, 1] in (0x0000, 0x8000)
    assert y[0, 2] == synth.to_bf16_bits(np.array([40.0 * x2[0, 2]], F32))[0]
    assert abs(synth.bf16_bits_to_f32(y[0:1, 3:4])[0, 0]) < 1e-14
    # the contexts are exactly the INT10 compression of the two inputs
    for got, src in ((c1, b1), (c2, b2)):
        p, s = fqo.ctx_quantize(src)
        assert np.array_equal(got[0], p) and np.array_equal(got[1], s)


def test_direct_rounding_to_bf16():
    """The forward value is rounded once from binary64: it is never farther than half a bf16
    step from the exact value."""
    b1, b2 = _inputs(seed=3)
    y, _, _ = fqo.glu_forward(b1, b2)
    exact = _silu(_f(b1)) * _f(b2)
    got = _f(y)
    step = np.maximum(np.abs(exact), 2.0 ** -126) * 2.0 ** -7       # bf16 spacing is <= |v| * 2^-7
    ok = np.abs(_f(b1)) < 15            # where the tanh form is accurate to ~1e-16 relative
    assert np.all((np.abs(got - exact) <= 0.5 * step * (1 + 1e-9))[ok])


def _deq(ctx, rows, cols):
    """scale * code in binary32, the codes unpacked with numpy bit operations."""
    bits = np.unpackbits(ctx[0], axis=-1, bitorder="little").reshape(rows, -1, 128, 10).astype(np.int64)
    q = (bits << np.arange(10)).sum(axis=-1)
    q = np.where(q >= 512, q - 1024, q).astype(F32)
    return (ctx[1][:, :, None] * q).astype(F32).reshape(rows, -1)[:, :cols].astype(np.float64)


def test_backward_is_the_derivative_of_forward():
    """dx1 and dx2 are dy times the partial derivatives of y = silu(x1) x2, taken at the values
    the INT10 contexts hold; the derivative of silu is checked by central differences."""
    rng = np.random.default_rng(1)
    rows, cols = 6, 256
    b1 = synth.to_bf16_bits((rng.standard_normal((rows, cols)) * 3).astype(F32))
    b2 = synth.to_bf16_bits((rng.standard_normal((rows, cols)) * 2).astype(F32))
    bdy = synth.to_bf16_bits(rng.standard_normal((rows, cols)).astype(F32))
    _, c1, c2 = fqo.glu_forward(b1, b2)
    dx1, dx2 = fqo.glu_backward(bdy, c1, c2)
    X1, X2, DY = _deq(c1, rows, cols), _deq(c2, rows, cols), _f(bdy)
    h = 1e-5
    d1 = (_silu(X1 + h) - _silu(X1 - h)) / (2 * h) * X2 * DY
    d2 = _silu(X1) * DY
    for got, want in ((dx1, d1), (dx2, d2)):
        tol = np.abs(want) * 2.0 ** -8 * 1.01 + 1e-7 * np.abs(DY) * (1 + np.abs(X2))
        assert np.all(np.abs(_f(got) - want) <= tol)


def test_backward_uses_the_dequantized_context_not_the_input():
    """Inputs that INT10 cannot hold exactly: the gradients follow the dequantized values."""
    b1, b2 = _inputs(rows=5, cols=260, seed=4)
    rng = np.random.default_rng(5)
    bdy = synth.to_bf16_bits(rng.standard_normal((5, 260)).astype(F32))
    _, c1, c2 = fqo.glu_forward(b1, b2)
    dx1, dx2 = fqo.glu_backward(bdy, c1, c2)
    x1q, x2q, DY = _deq(c1, 5, 260), _deq(c2, 5, 260), _f(bdy)
    assert np.abs(x1q - _f(b1)).max() > 0          # the context really is lossy here
    s = 0.5 * (1.0 + np.tanh(0.5 * x1q))
    want1 = DY * x2q * s * (1.0 + x1q * (1.0 - s))
    want2 = DY * x1q * s
    for got, want in ((dx1, want1), (dx2, want2)):
        d = _ulp_distance(got, synth.to_bf16_bits(want.astype(F32)))[np.abs(x1q) < 15]
        assert d.max() <= 1 and (d == 0).mean() > 0.99
    # and they differ from the gradients at the unquantized inputs somewhere
    s0 = 0.5 * (1.0 + np.tanh(0.5 * _f(b1)))
    assert (synth.to_bf16_bits((DY * _f(b1) * s0).astype(F32)) != dx2).any()
