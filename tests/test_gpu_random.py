"""Randomized GPU parity: seeded random shapes, products, thresholds, selectors, rounding modes
and tile plans; every quantizer output and every GEMM output is compared with the oracle bit for
bit.  The seeds are fixed, so the cases are the same on every run."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2503_08040_amd as fq
from oracle import fqo
from paper_2503_08040_amd import synth
from tests import gpu_util as gu

F32 = np.float32


def _matrix(rng, shape, heavy):
    x = rng.standard_normal(shape).astype(F32) * F32(np.exp(rng.normal(0, 2)))
    if heavy:
        n = max(1, x.size // 2000)
        x.flat[rng.integers(0, x.size, size=n)] *= F32(rng.uniform(30, 300))
    if rng.random() < 0.3:
        x[:, rng.integers(0, shape[1])] = 0.0
    if rng.random() < 0.15:          # down into the subnormal range: scales far from max/127
        x = x * F32(2.0 ** -126) / max(F32(1.0), np.abs(x).max() / F32(64.0))
    with np.errstate(under="ignore"):
        return synth.to_bf16_bits(x)


import os

N_SEEDS = int(os.environ.get("FQ_TEST_RANDOM_SEEDS", "12"))     # more seeds for an occasional longer run


@pytest.mark.parametrize("seed", list(range(N_SEEDS)))
def test_random_case(seed, monkeypatch):
    rng = np.random.default_rng(1000 + seed)
    op = int(rng.integers(0, 3))
    m, n, k = (int(rng.integers(1, 700)) for _ in range(3))
    sa = {0: (m, k), 1: (m, k), 2: (k, m)}[op]          # NT: A[M,K]  NN: A[M,K]  TN: A[K,M]
    sb = {0: (n, k), 1: (k, n), 2: (k, n)}[op]          # NT: B[N,K]  NN: B[K,N]  TN: B[K,N]
    a_bits, b_bits = _matrix(rng, sa, True), _matrix(rng, sb, False)
    mode = ["absmax", "all", "none", "l1", "sr", "topk"][int(rng.integers(0, 6))]
    monkeypatch.setenv("FQ_GEMM_CUS", str(int(rng.choice([1, 2, 3, 5, 7, 256]))))
    label = f"seed={seed} op={op} A{sa} B{sb} mode={mode}"
    gu.announce(label)
    ad, bd = gu.to_device_bf16(a_bits), gu.to_device_bf16(b_bits)
    if mode == "sr":
        s = int(rng.integers(0, 2 ** 62))
        ga = fq.fq_quantize_sr(ad, s, want_transposed=True)
        oa = fqo.quantize_sr(a_bits, 128, s)
    elif mode == "topk":
        nb = (-(-sa[0] // 128)) * (-(-sa[1] // 128))
        kk = int(rng.integers(0, nb + 2))
        ga = fq.fq_quantize_topk(ad, kk, want_transposed=True)
        oa = fqo.quantize_topk(a_bits, 128, kk)
    else:
        amax = np.abs(synth.bf16_bits_to_f32(a_bits)).max()
        crit, ocrit, theta = {
            "absmax": (fq.FQ_CRIT_ABSMAX_GT, fqo.CRIT_ABSMAX_GT, float(amax) * float(rng.uniform(0.05, 0.9))),
            "all": (fq.FQ_CRIT_ALL, fqo.CRIT_ALL, 0.0),
            "none": (fq.FQ_CRIT_NONE, fqo.CRIT_NONE, 0.0),
            "l1": (fq.FQ_CRIT_L1_GT, fqo.CRIT_L1_GT, -1.0),          # flags every block: no ties with theta
        }[mode]
        ga = fq.fq_quantize(ad, crit, theta, want_transposed=True)
        oa = fqo.quantize(a_bits, 128, ocrit, theta)
    gb = fq.fq_quantize(bd, fq.FQ_CRIT_NONE, 0.0, want_transposed=True)
    ob = fqo.quantize(b_bits, 128, fqo.CRIT_NONE, 0.0)
    gu.compare_quantized(ga, oa, label + " A")
    gu.compare_quantized(gb, ob, label + " B")
    ref, refb = fqo.gemm(op, oa, ob, want_bf16=True)
    got = fq.fq_gemm(op, ga, gb).cpu().numpy()
    assert gu.rel_err(got, ref) <= 1e-3, label
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), label
    gotb = fq.fq_gemm(op, ga, gb, out_dtype=torch.bfloat16).view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(gotb, refb), label
