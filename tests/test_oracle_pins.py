"""The CPU oracle against what the mathematics fixes: closed-form error bounds,
invariants, special cases that reduce to a library routine, brute force in
fp64 on tiny inputs.  None of these re-uses the oracle's own formulas."""
import numpy as np
import pytest

from oracle import fqo
from paper_2503_08040_amd import synth

F32 = np.float32


def _rand_bf16(rng, shape, std=1.0, outliers=0):
    x = rng.standard_normal(shape).astype(F32) * F32(std)
    for _ in range(outliers):
        i, j = rng.integers(shape[0]), rng.integers(shape[1])
        x[i, j] *= F32(rng.uniform(50, 400))
    return synth.to_bf16_bits(x)


def _f64(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def _expand(grid, g, rows, cols):
    """block grid -> per-element array"""
    return np.kron(grid, np.ones((g, g), grid.dtype))[:rows, :cols]


def _dequant(q, with_res):
    a = _expand(q.scales.astype(np.float64), q.g, q.rows, q.cols)
    d = a * q.codes
    if with_res:
        ra = _expand(q.res_scales.astype(np.float64), q.g, q.rows, q.cols)
        d = d + ra * q.res_codes
    return d


@pytest.mark.parametrize("g,shape", [(4, (8, 12)), (16, (40, 50)), (128, (256, 384)), (128, (130, 200))])
def test_error_bounds_and_code_range(g, shape):
    """Sec. 3.1: |x - a q| <= a/2.  Sec. 4.3: the residual has max <= a/2, so
    |x - (a q + a~ q~)| <= a~/2 <= amax / (2*127*254) = amax/64516."""
    rng = np.random.default_rng(1)
    xb = _rand_bf16(rng, shape, outliers=6)
    x = _f64(xb)
    q = fqo.quantize(xb, g, fqo.CRIT_ALL, 0.0)
    amax = np.zeros((q.nbr, q.nbc))
    for bi in range(q.nbr):
        for bk in range(q.nbc):
            amax[bi, bk] = np.abs(x[bi * g:(bi + 1) * g, bk * g:(bk + 1) * g]).max()
    # scale is the correctly rounded quotient amax/127
    assert np.array_equal(q.scales, (amax.astype(F32) / F32(127)).astype(F32))
    assert np.abs(q.codes.astype(int)).max() <= 127 and np.abs(q.res_codes.astype(int)).max() <= 127
    a = _expand(q.scales.astype(np.float64), g, *shape)
    ra = _expand(q.res_scales.astype(np.float64), g, *shape)
    am = _expand(amax, g, *shape)
    e1 = np.abs(x - _dequant(q, False))
    assert np.all(e1 <= 0.5 * a * (1 + 1e-6))
    e2 = np.abs(x - _dequant(q, True))
    assert np.all(e2 <= 0.5 * ra * (1 + 1e-6) + am * 2.0 ** -30)
    assert np.all(e2 <= am / 64516.0 * (1 + 1e-5))
    # the block's largest element gets code +-127; residual likewise where it is not zero
    for bi in range(q.nbr):
        for bk in range(q.nbc):
            blk = (slice(bi * g, (bi + 1) * g), slice(bk * g, (bk + 1) * g))
            if amax[bi, bk] > 0:
                assert np.abs(q.codes[blk].astype(int)).max() == 127
                idx = np.unravel_index(np.abs(x[blk]).argmax(), x[blk].shape)
                assert q.codes[blk][idx] == 127 * np.sign(x[blk][idx])
            if q.res_scales[bi, bk] > 0:
                assert np.abs(q.res_codes[blk].astype(int)).max() == 127
    assert q.mask.all() and q.fb_count[0] == q.nbr * q.nbc
    assert np.array_equal(q.fb_list[:q.fb_count[0]], np.arange(q.nbr * q.nbc))


def test_codes_are_nearest_integers_in_high_precision():
    """round(G/a): away from ties, the code is the integer nearest to x/a (fp64)."""
    rng = np.random.default_rng(2)
    xb = _rand_bf16(rng, (64, 64), outliers=3)
    q = fqo.quantize(xb, 32, fqo.CRIT_NONE, 0.0)
    x = _f64(xb)
    t = x / _expand(q.scales.astype(np.float64), 32, 64, 64)
    frac = np.abs(t - np.floor(t) - 0.5)
    clear = frac > 1e-4
    assert clear.mean() > 0.99
    assert np.array_equal(q.codes[clear], np.rint(t[clear]).astype(np.int8))
    assert np.all(np.abs(q.codes - t) <= 0.5 + 1e-4)


def test_block_size_one_is_exact_gemm():
    """g = 1: every element is its own block, q = +-127, a = |x|/127, so the
    method is the exact GEMM up to fp32 rounding -> compare with fp64 matmul."""
    rng = np.random.default_rng(3)
    M, K, N = 7, 9, 5
    xb, wb = _rand_bf16(rng, (M, K)), _rand_bf16(rng, (N, K), 0.02)
    qx = fqo.quantize(xb, 1, fqo.CRIT_NONE, 0.0)
    qw = fqo.quantize(wb, 1, fqo.CRIT_NONE, 0.0)
    nz = _f64(xb) != 0
    assert np.all(np.abs(qx.codes[nz].astype(int)) == 127)
    c = fqo.gemm(fqo.OP_NT, qx, qw).astype(np.float64)
    ref = _f64(xb) @ _f64(wb).T
    bound = (np.abs(_f64(xb)) @ np.abs(_f64(wb)).T) * (K + 8) * 2.0 ** -23
    assert np.all(np.abs(c - ref) <= bound)
    assert np.abs(c - ref).max() > 0 or True


def test_threshold_semantics():
    """Sec. 4.4: u = [max|G| > theta], strict.  theta = +inf is plain block INT8;
    a negative theta flags every block, even an all-zero one."""
    rng = np.random.default_rng(4)
    x = rng.standard_normal((8, 8)).astype(F32)
    x[0:4, 4:8] = 0.0
    x[4, 5] = 6.0      # block (1,1) has amax exactly 6 (representable in bf16)
    x[4:8, 4:8] = np.clip(x[4:8, 4:8], -6, 6)
    xb = synth.to_bf16_bits(x)
    q_eq = fqo.quantize(xb, 4, fqo.CRIT_ABSMAX_GT, 6.0)
    assert q_eq.mask[1, 1] == 0           # amax == theta is not "greater than"
    q_lt = fqo.quantize(xb, 4, fqo.CRIT_ABSMAX_GT, float(np.nextafter(F32(6.0), F32(0))))
    assert q_lt.mask[1, 1] == 1
    q_inf = fqo.quantize(xb, 4, fqo.CRIT_ABSMAX_GT, float("inf"))
    q_none = fqo.quantize(xb, 4, fqo.CRIT_NONE, 0.0)
    for f in ("codes", "scales", "mask", "res_codes", "res_scales", "fb_count"):
        assert np.array_equal(getattr(q_inf, f), getattr(q_none, f))
    assert not q_none.mask.any() and not q_none.res_codes.any() and q_none.fb_count[0] == 0
    q_neg = fqo.quantize(xb, 4, fqo.CRIT_ABSMAX_GT, -1.0)
    q_all = fqo.quantize(xb, 4, fqo.CRIT_ALL, 0.0)
    for f in ("codes", "scales", "mask", "res_codes", "res_scales", "fb_count", "fb_list"):
        assert np.array_equal(getattr(q_neg, f), getattr(q_all, f))
    q_zero = fqo.quantize(xb, 4, fqo.CRIT_ABSMAX_GT, 0.0)
    assert q_zero.mask.tolist() == [[1, 0], [1, 1]]     # the all-zero block is not > 0
    assert q_all.scales[0, 1] == 0 and not q_all.codes[0:4, 4:8].any()
    # mask is monotone in theta, count and list follow the mask
    prev = None
    for th in [0.5, 1.0, 2.0, 3.0, 6.0]:
        q = fqo.quantize(xb, 4, fqo.CRIT_ABSMAX_GT, th)
        assert q.fb_count[0] == q.mask.sum()
        assert np.array_equal(q.fb_list[:q.fb_count[0]], np.nonzero(q.mask.ravel())[0])
        if prev is not None:
            assert np.all(q.mask <= prev)
        prev = q.mask.copy()


def test_transpose_and_power_of_two_scaling_invariance():
    rng = np.random.default_rng(5)
    xb = _rand_bf16(rng, (48, 80), outliers=4)
    q = fqo.quantize(xb, 16, fqo.CRIT_ABSMAX_GT, 8.0)
    qt = fqo.quantize(np.ascontiguousarray(xb.T), 16, fqo.CRIT_ABSMAX_GT, 8.0)
    assert 0 < q.fb_count[0] < q.nbr * q.nbc
    assert np.array_equal(qt.codes, q.codes.T) and np.array_equal(qt.res_codes, q.res_codes.T)
    assert np.array_equal(qt.scales, q.scales.T) and np.array_equal(qt.res_scales, q.res_scales.T)
    assert np.array_equal(qt.mask, q.mask.T)
    # x * 2^e: same codes, scales * 2^e (bf16 exponent shift is exact away from the range ends)
    for e in (-20, 7):
        xs = synth.to_bf16_bits(synth.bf16_bits_to_f32(xb) * F32(2.0 ** e))
        qs = fqo.quantize(xs, 16, fqo.CRIT_ABSMAX_GT, 8.0 * 2.0 ** e)
        assert np.array_equal(qs.codes, q.codes) and np.array_equal(qs.res_codes, q.res_codes)
        assert np.array_equal(qs.scales, q.scales * F32(2.0 ** e))
        assert np.array_equal(qs.res_scales, q.res_scales * F32(2.0 ** e))
        assert np.array_equal(qs.mask, q.mask)


def test_subnormal_scales_are_not_flushed():
    """bf16 subnormals m * 2^-133 (m <= 127) with block max m = 127: a = 2^-133
    exactly (an fp32 subnormal) and the codes are the integers m."""
    rng = np.random.default_rng(6)
    m = rng.integers(-127, 128, size=(4, 4))
    m[1, 2] = 127
    bits = (np.abs(m).astype(np.uint16)) | np.where(m < 0, np.uint16(0x8000), np.uint16(0))
    q = fqo.quantize(bits.astype(np.uint16), 4, fqo.CRIT_ALL, 0.0)
    assert q.scales[0, 0] == F32(2.0 ** -133) and q.scales[0, 0] > 0
    assert np.array_equal(q.codes, m)
    assert q.res_scales[0, 0] == 0 and not q.res_codes.any()
    # small normal range too
    xb = synth.to_bf16_bits((rng.standard_normal((8, 8)) * 1e-37).astype(F32))
    q = fqo.quantize(xb, 8, fqo.CRIT_ALL, 0.0)
    assert np.abs(q.codes.astype(int)).max() == 127 and np.isfinite(q.scales).all()


def _int_blocks(rng, rows, cols, g):
    """integer matrix whose every g x g block has abs-max exactly 127"""
    x = rng.integers(-127, 128, size=(rows, cols))
    for bi in range(0, rows, g):
        for bk in range(0, cols, g):
            x[bi + rng.integers(min(g, rows - bi)), bk + rng.integers(min(g, cols - bk))] = 127
    return x


def test_clamp_matters_for_subnormal_scales():
    """Worked by hand in units of u = 2^-149 (Sec. 3.1, 4.3): the block [[3, 1], [-1, 0]] * 2^-133
    has a = RN(196608 u / 127) = 1548 u, codes [[127, 42], [-42, 0]], residuals
    [[12, 520], [-520, 0]] u and a~ = RN(520 u / 127) = 4 u: a subnormal scale is an integer number
    of u, far from 520/127, so r / a~ = +-130 lies outside the code range and is clamped to +-127."""
    u = 2.0 ** -149
    x = np.array([[3.0, 1.0], [-1.0, 0.0]]) * 2.0 ** -133
    q = fqo.quantize(synth.to_bf16_bits(x.astype(F32)), 2, fqo.CRIT_ALL, 0.0)
    assert float(q.scales[0, 0]) == 1548 * u
    assert q.codes.tolist() == [[127, 42], [-42, 0]]
    assert float(q.res_scales[0, 0]) == 4 * u
    assert q.res_codes.tolist() == [[3, 127], [-127, 0]]


@pytest.mark.parametrize("op", [fqo.OP_NT, fqo.OP_NN, fqo.OP_TN])
def test_integer_inputs_reduce_to_integer_matmul(op):
    """All scales 1 -> Eq. (1) is an exact integer matrix product (numpy int64)."""
    rng = np.random.default_rng(7)
    g = 4
    if op == fqo.OP_NT:
        a, b = _int_blocks(rng, 12, 20, g), _int_blocks(rng, 8, 20, g)
        ref = a @ b.T
    elif op == fqo.OP_NN:
        a, b = _int_blocks(rng, 12, 20, g), _int_blocks(rng, 20, 8, g)
        ref = a @ b
    else:
        a, b = _int_blocks(rng, 20, 12, g), _int_blocks(rng, 20, 8, g)
        ref = a.T @ b
    qa = fqo.quantize(synth.to_bf16_bits(a.astype(F32)), g, fqo.CRIT_NONE, 0.0)
    qb = fqo.quantize(synth.to_bf16_bits(b.astype(F32)), g, fqo.CRIT_NONE, 0.0)
    assert np.all(qa.scales == 1) and np.array_equal(qa.codes, a)
    c = fqo.gemm(op, qa, qb)
    assert np.array_equal(c.astype(np.int64), ref)
    nkb = 5
    tot = sum(fqo.gemm_partials(op, qa, qb, kb, False).astype(np.int64) for kb in range(nkb))
    assert np.array_equal(tot, ref)


def _brute_force(op, xa, qa, qb, use_res):
    """fp64 evaluation of sum_k (a q + u a~ q~)(b q_B), element by element."""
    da = _dequant(qa, False)
    if use_res:
        u = _expand(qa.mask.astype(np.float64), qa.g, qa.rows, qa.cols)
        ra = _expand(qa.res_scales.astype(np.float64), qa.g, qa.rows, qa.cols)
        da = da + u * ra * qa.res_codes
    db = _dequant(qb, False)
    Mo, No = fqo.out_shape(op, qa, qb)
    out = np.zeros((Mo, No))
    for i in range(Mo):
        for j in range(No):
            if op == fqo.OP_NT:
                out[i, j] = sum(da[i, t] * db[j, t] for t in range(qa.cols))
            elif op == fqo.OP_NN:
                out[i, j] = sum(da[i, t] * db[t, j] for t in range(qa.cols))
            else:
                out[i, j] = sum(da[t, i] * db[t, j] for t in range(qa.rows))
    return out


@pytest.mark.parametrize("op", [fqo.OP_NT, fqo.OP_NN, fqo.OP_TN])
@pytest.mark.parametrize("g", [2, 4])
def test_brute_force_tiny(op, g):
    """Sec. 4.3's sum evaluated directly in fp64 on tiny, ragged inputs."""
    rng = np.random.default_rng(8 + g)
    shapes = {fqo.OP_NT: ((7, 9), (6, 9)), fqo.OP_NN: ((7, 9), (9, 6)), fqo.OP_TN: ((9, 7), (9, 6))}
    sa, sb = shapes[op]
    ab, bb = _rand_bf16(rng, sa, outliers=3), _rand_bf16(rng, sb, 0.02)
    qa = fqo.quantize(ab, g, fqo.CRIT_ABSMAX_GT, 4.0)
    qb = fqo.quantize(bb, g, fqo.CRIT_NONE, 0.0)
    assert 0 < qa.fb_count[0] < qa.nbr * qa.nbc
    c = fqo.gemm(op, qa, qb).astype(np.float64)
    ref = _brute_force(op, ab, qa, qb, True)
    scale = np.abs(ref).max()
    assert np.abs(c - ref).max() <= 1e-5 * scale
    # dropping the residual term must be visible at this tolerance
    ref_nores = _brute_force(op, ab, qa, qb, False)
    assert np.abs(ref_nores - ref).max() > 1e-4 * scale
    c_off = fqo.gemm(op, qa, qb, a_fallback=False).astype(np.float64)
    assert np.abs(c_off - ref_nores).max() <= 1e-5 * scale


def test_backward_forms_equal_forward_on_transposed_inputs():
    """dX = dY W equals the NT product of dY with W^T, dW = dY^T X equals the NT
    product of dY^T with X^T (square blocks: transposing commutes with quantizing)."""
    rng = np.random.default_rng(10)
    M, N, K, g = 24, 40, 16, 8
    dyb = _rand_bf16(rng, (M, N), 1e-3, outliers=3)
    wb, xb = _rand_bf16(rng, (N, K), 0.02), _rand_bf16(rng, (M, K))
    th = 4e-3
    qdy = fqo.quantize(dyb, g, fqo.CRIT_ABSMAX_GT, th)
    assert 0 < qdy.fb_count[0] < qdy.nbr * qdy.nbc
    qw = fqo.quantize(wb, g, fqo.CRIT_NONE, 0.0)
    qx = fqo.quantize(xb, g, fqo.CRIT_NONE, 0.0)
    qwt = fqo.quantize(np.ascontiguousarray(wb.T), g, fqo.CRIT_NONE, 0.0)
    qxt = fqo.quantize(np.ascontiguousarray(xb.T), g, fqo.CRIT_NONE, 0.0)
    qdyt = fqo.quantize(np.ascontiguousarray(dyb.T), g, fqo.CRIT_ABSMAX_GT, th)
    dx = fqo.gemm(fqo.OP_NN, qdy, qw)
    assert dx.shape == (M, K)
    assert np.array_equal(dx, fqo.gemm(fqo.OP_NT, qdy, qwt))
    dw = fqo.gemm(fqo.OP_TN, qdy, qx)
    assert dw.shape == (N, K)
    assert np.array_equal(dw, fqo.gemm(fqo.OP_NT, qdyt, qxt))
    for kb in range(2):
        for res in (False, True):
            assert np.array_equal(fqo.gemm_partials(fqo.OP_TN, qdy, qx, kb, res),
                                  fqo.gemm_partials(fqo.OP_NT, qdyt, qxt, kb, res))
    # and both are close to the exact fp64 products
    exact_dx = _f64(dyb) @ _f64(wb)
    exact_dw = _f64(dyb).T @ _f64(xb)
    assert np.abs(dx - exact_dx).max() <= 2e-2 * np.abs(exact_dx).max()
    assert np.abs(dw - exact_dw).max() <= 2e-2 * np.abs(exact_dw).max()


def test_full_fallback_is_16_bit_on_the_A_side():
    """u == 1: C equals A * deq(Q(B)) to within sum_k amax^A_ik/64516 * sum_t |deq(B)_t|
    plus fp32 accumulation error; with u == 0 the error is two orders larger."""
    rng = np.random.default_rng(11)
    M, K, N, g = 32, 64, 24, 16
    xb, wb = _rand_bf16(rng, (M, K), outliers=5), _rand_bf16(rng, (N, K), 0.02)
    qa = fqo.quantize(xb, g, fqo.CRIT_ALL, 0.0)
    qn = fqo.quantize(xb, g, fqo.CRIT_NONE, 0.0)
    qw = fqo.quantize(wb, g, fqo.CRIT_NONE, 0.0)
    dw = _dequant(qw, False)
    ref = _f64(xb) @ dw.T
    amax = np.abs(_f64(xb)).reshape(M // g, g, K // g, g).max(axis=(1, 3))
    bound = (_expand(amax, g, M, K) / 64516.0) @ np.abs(dw).T
    bound = bound * (1 + 1e-5) + (np.abs(_f64(xb)) @ np.abs(dw).T) * (K // g + 4) * 2.0 ** -23
    c_all = fqo.gemm(fqo.OP_NT, qa, qw).astype(np.float64)
    assert np.all(np.abs(c_all - ref) <= bound)
    c_none = fqo.gemm(fqo.OP_NT, qn, qw).astype(np.float64)
    assert np.abs(c_none - ref).max() > 30 * np.abs(c_all - ref).max()


def test_window_and_bf16_output():
    rng = np.random.default_rng(12)
    xb, wb = _rand_bf16(rng, (20, 24), outliers=2), _rand_bf16(rng, (12, 24), 0.02)
    qa = fqo.quantize(xb, 8, fqo.CRIT_ABSMAX_GT, 5.0)
    qw = fqo.quantize(wb, 8, fqo.CRIT_NONE, 0.0)
    full, fullb = fqo.gemm(fqo.OP_NT, qa, qw, want_bf16=True)
    win = fqo.gemm(fqo.OP_NT, qa, qw, window=(3, 11, 2, 9))
    assert np.array_equal(win[3:11, 2:9], full[3:11, 2:9])
    assert not win[:3].any() and not win[:, 9:].any()
    assert np.array_equal(fullb, synth.to_bf16_bits(full))      # RNE, checked by numpy's rounding
    back = synth.bf16_bits_to_f32(fullb)
    assert np.all(np.abs(back - full) <= np.abs(full) * 2.0 ** -8)


def test_bf16_output_ties_round_to_even():
    """257 = 1.00000001b * 2^8 lies midway between the bf16 values 256 and 258:
    nearest-even gives 256 (0x4380); 259 lies midway between 258 and 260 -> 260."""
    a = np.array([[127, 3], [127, 5]], F32)
    b = np.array([[2, 1], [127, 0]], F32)
    qa = fqo.quantize(synth.to_bf16_bits(a), 2, fqo.CRIT_NONE, 0.0)
    qb = fqo.quantize(synth.to_bf16_bits(b), 2, fqo.CRIT_NONE, 0.0)
    c, cb = fqo.gemm(fqo.OP_NT, qa, qb, want_bf16=True)
    assert c[0, 0] == 257 and c[1, 0] == 259
    assert cb[0, 0] == 0x4380 and synth.bf16_bits_to_f32(cb)[1, 0] == 260


def test_gemm_window_returns_the_same_values_as_the_full_call():
    """fqo.gemm_window (only the window's rows are materialized) against fqo.gemm."""
    rng = np.random.default_rng(11)
    a = synth.to_bf16_bits(rng.standard_normal((70, 40)).astype(np.float32))
    b = synth.to_bf16_bits(rng.standard_normal((50, 40)).astype(np.float32))
    qa = fqo.quantize(a, 16, fqo.CRIT_ABSMAX_GT, 2.5)
    qb = fqo.quantize(b, 16, fqo.CRIT_NONE, 0.0)
    full, fullb = fqo.gemm(fqo.OP_NT, qa, qb, want_bf16=True)
    for win in ((0, 70, 0, 50), (16, 48, 5, 37), (69, 70, 49, 50), (10, 10, 0, 50)):
        i0, i1, j0, j1 = win
        w32, wb = fqo.gemm_window(fqo.OP_NT, qa, qb, win, want_bf16=True)
        assert w32.shape == (i1 - i0, 50)
        assert np.array_equal(w32[:, j0:j1], full[i0:i1, j0:j1])
        assert np.array_equal(wb[:, j0:j1], fullb[i0:i1, j0:j1])
        assert not w32[:, :j0].any() and not w32[:, j1:].any()
