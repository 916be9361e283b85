"""Oracle pins for the widened path: stochastic-rounding block quantization
(Sec. 3.1, 5.1) and the delay-threshold controller (App. D, Alg. 2)."""
import numpy as np

from oracle import fqo
from paper_2503_08040_amd import synth
from tests import golden_io

F32 = np.float32


def test_philox_known_answers():
    _, m = golden_io.load("philox4x32_10_kat.txt")
    for c, k, o in zip(m["ctr"], m["key"], m["out"]):
        assert np.array_equal(fqo.philox4x32_10(c, k), o.astype(np.uint32))


def _bf16(x):
    return synth.to_bf16_bits(np.asarray(x, F32))


def test_sr_rounds_to_a_neighbour_and_keeps_integers():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((64, 96)).astype(F32)
    x[3, 5] = 40.0
    xb = _bf16(x)
    q = fqo.quantize_sr(xb, 32, seed=7)
    ref = fqo.quantize(xb, 32, fqo.CRIT_NONE, 0.0)
    assert np.array_equal(q.scales, ref.scales)            # same scale as round-to-nearest
    t = synth.bf16_bits_to_f32(xb).astype(np.float64) / np.kron(q.scales.astype(np.float64),
                                                                 np.ones((32, 32)))
    assert np.all(q.codes >= np.floor(t) - 1e-9) and np.all(q.codes <= np.ceil(t) + 1e-9)
    assert np.abs(q.codes.astype(int)).max() <= 127
    assert (q.codes != ref.codes).mean() > 0.2               # it is not round-to-nearest
    # a block of integers with abs-max 127 has scale 1 and is reproduced exactly, any seed
    ints = rng.integers(-127, 128, size=(32, 32))
    ints[0, 0] = 127
    for seed in (0, 1, 12345678901234):
        qi = fqo.quantize_sr(_bf16(ints), 32, seed)
        assert np.array_equal(qi.codes, ints)
    # deterministic in the seed, different across seeds
    assert np.array_equal(fqo.quantize_sr(xb, 32, 7).codes, q.codes)
    assert not np.array_equal(fqo.quantize_sr(xb, 32, 8).codes, q.codes)
    # all-zero block
    z = fqo.quantize_sr(_bf16(np.zeros((32, 32))), 32, 3)
    assert not z.codes.any() and z.scales[0, 0] == 0


def test_sr_is_unbiased():
    """E[Q_s(x)] = x: the mean code over many seeds approaches x/a (binomial confidence bound),
    and the up-rounding frequency of one value matches its fraction."""
    vals = np.array([[127.0, 0.25, -0.75, 10.5], [63.3, -20.1, 0.0, 1e-3]], F32)
    xb = _bf16(np.tile(vals, (1, 1)))
    t = synth.bf16_bits_to_f32(xb).astype(np.float64)      # scale is 1 (abs-max 127)
    n = 4000
    acc = np.zeros_like(t)
    for seed in range(n):
        acc += fqo.quantize_sr(xb, 4, seed).codes[:2, :4]
    mean = acc / n
    sigma = np.sqrt(0.25 / n)
    assert np.all(np.abs(mean - t) < 5 * sigma + 1e-6)
    # many elements, one seed: element index enters the generator
    big = np.full((128, 128), 0.3, F32)
    big[0, 0] = 127.0
    qb = fqo.quantize_sr(_bf16(big), 128, 99)
    frac = synth.bf16_bits_to_f32(_bf16([[0.3]]))[0, 0]
    up = (qb.codes == 1).mean()
    assert abs(up - frac) < 5 * np.sqrt(0.21 / 16384)


def test_sr_gradient_gemm_is_unbiased_in_expectation():
    """Sec. 5.1: E[dY_q^T] X = dW.  Averaging the block GEMM over seeds approaches the GEMM of
    the unquantized gradient with the quantized X much closer than any single draw."""
    rng = np.random.default_rng(1)
    dy = (rng.standard_t(3.0, size=(32, 16)) * 1e-3).astype(F32)
    x = rng.standard_normal((32, 24)).astype(F32)
    dyb, xb = _bf16(dy), _bf16(x)
    qx = fqo.quantize(xb, 8, fqo.CRIT_NONE, 0.0)
    dxq = np.kron(qx.scales.astype(np.float64), np.ones((8, 8))) * qx.codes
    exact = synth.bf16_bits_to_f32(dyb).astype(np.float64).T @ dxq
    draws = [fqo.gemm(fqo.OP_TN, fqo.quantize_sr(dyb, 8, s), qx).astype(np.float64)
             for s in range(200)]
    single = np.abs(draws[0] - exact).max()
    mean = np.abs(np.mean(draws, axis=0) - exact).max()
    assert mean < 0.25 * single


def test_delay_threshold_controller():
    """Alg. 2: divide by alpha below r_min, multiply above r_max, keep inside the range."""
    th = fqo.threshold_update
    assert th(1.0, 5, 100) == np.float32(1.0) / np.float32(1.3)        # 5 % < 10 %
    assert th(1.0, 31, 100) == np.float32(1.0) * np.float32(1.3)       # 31 % > 30 %
    assert th(2.0, 10, 100) == 2.0 and th(2.0, 30, 100) == 2.0         # bounds are inside
    assert th(2.0, 20, 100) == 2.0
    assert th(3.0, 0, 0) == 3.0                                        # no blocks: unchanged
    assert th(1.0, 1, 100, r_min=0.0, r_max=0.0, alpha=2.0) == 2.0
    # closed loop on a fixed tensor: theta starts at 1 (Alg. 2) and settles where the rate is
    # inside [0.1, 0.3]; from then on it does not move
    rng = np.random.default_rng(2)
    x = rng.standard_normal((256, 256)).astype(F32) * np.exp(rng.standard_normal((256, 1))).astype(F32)
    xb = _bf16(x)
    theta, hist = 1.0, []
    for _ in range(40):
        q = fqo.quantize(xb, 32, fqo.CRIT_ABSMAX_GT, theta)
        rate = q.fb_count[0] / q.mask.size
        hist.append(rate)
        theta = th(theta, int(q.fb_count[0]), q.mask.size)
    assert 0.1 <= hist[-1] <= 0.3 and hist[-1] == hist[-2]
    assert hist[0] > 0.3                                               # it had to move
