"""Quantization groups of 64 x 64 and 32 x 32 (Sec. 4.5, Fig. 1b): plain block INT8 through the
library's plain kernel against the oracle with the same group size: codes, scales, the INT32
product of single k-groups and the outputs of all three products, bit for bit; fq_gemm_plain
at block 128 against fq_gemm; what block sizes below 128 do not support is refused."""
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


def _bits(shape, seed, std=1.0, spikes=0):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal(shape) * std).astype(F32)
    for _ in range(spikes):
        x[rng.integers(shape[0]), rng.integers(shape[1])] *= 60.0
    return synth.to_bf16_bits(x)


@pytest.mark.parametrize("g", [32, 64])
@pytest.mark.parametrize("shape", [(256, 384), (130, 200), (1, 1), (97, 33), (300, 700)])
def test_quantize_small_groups(g, shape):
    bits = _bits(shape, seed=g + shape[0], spikes=5)
    gu.announce(f"quantize block={g} shape={shape}")
    gq = fq.fq_quantize(gu.to_device_bf16(bits), fq.FQ_CRIT_NONE, 0.0, want_transposed=True, block=g)
    oq = fqo.quantize(bits, g, fqo.CRIT_NONE, 0.0)
    assert (gq.nbr, gq.nbc) == (oq.nbr, oq.nbc)
    gu.compare_quantized(gq, oq, f"block {g} {shape}")


@pytest.mark.parametrize("g", [32, 64])
@pytest.mark.parametrize("op,sa,sb", [
    (fq.FQ_OP_NT, (256, 384), (128, 384)),
    (fq.FQ_OP_NT, (130, 200), (70, 200)),
    (fq.FQ_OP_NN, (200, 130), (130, 310)),
    (fq.FQ_OP_TN, (260, 150), (260, 90)),
    (fq.FQ_OP_NT, (33, 1000), (257, 1000)),
])
def test_gemm_small_groups(g, op, sa, sb):
    a_bits = _bits(sa, seed=g + sa[0], spikes=6)
    b_bits = _bits(sb, seed=g + sb[0] + 1, std=0.05)
    ga = fq.fq_quantize(gu.to_device_bf16(a_bits), fq.FQ_CRIT_NONE, 0.0, want_transposed=True, block=g)
    gb = fq.fq_quantize(gu.to_device_bf16(b_bits), fq.FQ_CRIT_NONE, 0.0, want_transposed=True, block=g)
    oa = fqo.quantize(a_bits, g, fqo.CRIT_NONE, 0.0)
    ob = fqo.quantize(b_bits, g, fqo.CRIT_NONE, 0.0)
    gu.announce(f"gemm block={g} op={op} {sa} x {sb}")
    c32 = fq.fq_gemm(op, ga, gb)
    cb = fq.fq_gemm(op, ga, gb, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    ref, refb = fqo.gemm(op, oa, ob, want_bf16=True)
    assert gu.rel_err(c32.cpu().numpy(), ref) <= 1e-3
    assert np.array_equal(c32.cpu().numpy(), ref)
    assert np.array_equal(cb.view(torch.int16).cpu().numpy().view(np.uint16), refb)
    # the INT32 product of every k-group
    Kc = sa[1] if op != fq.FQ_OP_TN else sa[0]
    for kg in range(-(-Kc // g)):
        got = fq.fq_gemm_debug_partials(op, ga, gb, kg, False).cpu().numpy()
        assert np.array_equal(got, fqo.gemm_partials(op, oa, ob, kg, False)), f"k-group {kg}"


def test_plain_kernel_at_128_matches_the_tuned_one():
    a_bits = _bits((384, 640), 1, spikes=4)
    b_bits = _bits((520, 640), 2, std=0.02)
    ga = fq.fq_quantize(gu.to_device_bf16(a_bits), fq.FQ_CRIT_NONE, 0.0, capacity=0)
    gb = fq.fq_quantize(gu.to_device_bf16(b_bits), fq.FQ_CRIT_NONE, 0.0, capacity=0)
    gu.announce("plain kernel at block 128")
    assert torch.equal(fq.fq_gemm_plain(fq.FQ_OP_NT, ga, gb), fq.fq_gemm(fq.FQ_OP_NT, ga, gb))
    gf = fq.fq_quantize(gu.to_device_bf16(a_bits), fq.FQ_CRIT_ABSMAX_GT, 8.0)
    with pytest.raises(fq.FqError) as e:
        fq.fq_gemm_plain(fq.FQ_OP_NT, gf, gb)
    assert e.value.status == fq.FQ_ERR_ENUM


def test_small_groups_refuse_fallback_and_mixed_sizes():
    x = gu.to_device_bf16(_bits((128, 128), 3))
    for call in (lambda: fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, 1.0, block=64, capacity=0),
                 lambda: fq.QTensor(128, 128, capacity=4, block=32)):
        with pytest.raises(fq.FqError) as e:
            call()
        assert e.value.status in (fq.FQ_ERR_BLOCK, fq.FQ_ERR_SHAPE)
    q64 = fq.fq_quantize(x, fq.FQ_CRIT_NONE, 0.0, block=64)
    q128 = fq.fq_quantize(x, fq.FQ_CRIT_NONE, 0.0, capacity=0)
    with pytest.raises(fq.FqError) as e:
        fq.fq_gemm(fq.FQ_OP_NT, q64, q128)
    assert e.value.status == fq.FQ_ERR_BLOCK
    with pytest.raises(fq.FqError) as e:
        fq.fq_quantize(x, fq.FQ_CRIT_NONE, 0.0, block=16)
    assert e.value.status in (fq.FQ_ERR_BLOCK, fq.FQ_ERR_SHAPE)
