"""GPU parity of fq_gemm_biased, the tolerance variant of fq_gemm, against the CPU oracle.

The variant keeps Alg. 1's operands and order of terms but folds the INT32 block products into the
FP32 accumulators through a biased bit pattern instead of a conversion (see fq.h), so its FP32
additions round at a larger magnitude.  The bar is the one stated for FP32 outputs,
max |diff| / max |ref| <= 1e-3 against the oracle; it is not bit-identical (fq_gemm is, and stays
the reference path).  A bf16 output is the rounding of an FP32 value within that tolerance, so it
may differ from the oracle's by that tolerance plus its own rounding step.
The error does not grow with the contraction length: checked on K = 128 ... 11008."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2503_08040_amd as fq
from oracle import fqo
from paper_2503_08040_amd import synth
from tests import gpu_util as gu
from tests.test_gpu_gemm import _quant_pair, _tile_windows

F32 = np.float32
TOL = 1e-3


def _check(op, ga, gb, oa, ob, label):
    ref, refb = fqo.gemm(op, oa, ob, want_bf16=True)
    gu.announce(f"{label}: biased gemm op={op} fp32")
    c = fq.fq_gemm_biased(op, ga, gb).cpu().numpy()
    assert c.shape == ref.shape and np.isfinite(c).all()
    err = gu.rel_err(c, ref)
    print(f"{label}: max |diff| / max |ref| = {err:.3e}", flush=True)
    assert err <= TOL, f"{label}: rel err {err}"
    gu.announce(f"{label}: biased gemm op={op} bf16")
    cb = fq.fq_gemm_biased(op, ga, gb, out_dtype=torch.bfloat16)
    assert torch.equal(cb, torch.from_numpy(c).cuda().to(torch.bfloat16)), "bf16 output is not the rounding of fp32"
    # the bf16 value is the fp32 value (within TOL of the oracle) rounded: half a bf16 step more
    cbf = synth.bf16_bits_to_f32(cb.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    bound = TOL * np.abs(ref).max() + 2.0 ** -8 * np.abs(ref)
    assert (np.abs(cbf - ref) <= bound).all(), f"{label}: bf16 output outside tolerance + rounding"
    same = (cb.view(torch.int16).cpu().numpy().view(np.uint16) == refb).mean() if refb.size else 1.0
    print(f"{label}: bf16 outputs equal to the oracle's: {100 * same:.2f} %", flush=True)
    return err


def test_config1():
    wl = synth.config1()
    ga, gb, oa, ob = _quant_pair(wl.X, wl.W, fq.FQ_CRIT_ABSMAX_GT, wl.theta)
    _check(fq.FQ_OP_NT, ga, gb, oa, ob, "cfg1")
    # every block flagged: a residual item behind every main item
    ga, gb, oa, ob = _quant_pair(wl.X, wl.W, fq.FQ_CRIT_ALL, 0.0)
    _check(fq.FQ_OP_NT, ga, gb, oa, ob, "cfg1 all flagged")


@pytest.mark.parametrize("op,sa,sb", [
    (fq.FQ_OP_NT, (130, 200), (77, 200)),
    (fq.FQ_OP_NT, (300, 1300), (260, 1300)),      # 11 k-blocks: bias windows of 4, 4 and 3 items
    (fq.FQ_OP_NT, (1, 1), (1, 1)),
    (fq.FQ_OP_NN, (257, 384), (384, 300)),
    (fq.FQ_OP_TN, (384, 257), (384, 300)),
    (fq.FQ_OP_NT, (640, 128), (768, 128)),        # one k-block: a window that never fills
])
def test_ragged_and_multi_tile_shapes(op, sa, sb):
    rng = np.random.default_rng(sa[0] + 7 * sb[1] + op)
    a = rng.standard_normal(sa).astype(F32)
    for _ in range(6):
        a[rng.integers(sa[0]), rng.integers(sa[1])] *= 120.0
    b = rng.standard_normal(sb).astype(F32) * F32(0.02)
    ga, gb, oa, ob = _quant_pair(synth.to_bf16_bits(a), synth.to_bf16_bits(b),
                                 fq.FQ_CRIT_ABSMAX_GT, 8.0)
    _check(op, ga, gb, oa, ob, f"ragged op={op} {sa}x{sb}")


@pytest.mark.parametrize("op,sa,sb,cus", [
    (fq.FQ_OP_NT, (700, 300), (1100, 300), 10),
    (fq.FQ_OP_NN, (300, 200), (200, 1300), 7),
])
def test_mixed_tile_geometries(op, sa, sb, cus, monkeypatch):
    monkeypatch.setenv("FQ_GEMM_CUS", str(cus))
    rng = np.random.default_rng(sa[0] + 3 * sb[1] + op + cus)
    a = rng.standard_normal(sa).astype(F32)
    for _ in range(12):
        a[rng.integers(sa[0]), rng.integers(sa[1])] *= 120.0
    b = rng.standard_normal(sb).astype(F32) * F32(0.02)
    ga, gb, oa, ob = _quant_pair(synth.to_bf16_bits(a), synth.to_bf16_bits(b),
                                 fq.FQ_CRIT_ABSMAX_GT, 8.0)
    Mo, No = fqo.out_shape(op, oa, ob)
    plan = fq.fq_gemm_tile_plan(Mo, No)
    assert plan[2] > 0 and plan[0] > 0
    _check(op, ga, gb, oa, ob, f"mixed op={op} {sa}x{sb} cus={cus}")


def test_scale_range():
    """The bias is proportional to the scales: tiny and huge scale products in one contraction."""
    rng = np.random.default_rng(5)
    a = rng.standard_normal((256, 1024)).astype(F32)
    a[:, :128] *= F32(1e-12)
    a[:, 512:640] *= F32(1e12)
    b = rng.standard_normal((256, 1024)).astype(F32)
    ga, gb, oa, ob = _quant_pair(synth.to_bf16_bits(a), synth.to_bf16_bits(b), fq.FQ_CRIT_NONE, 0.0)
    _check(fq.FQ_OP_NT, ga, gb, oa, ob, "scale range")


def test_rejects_small_groups_and_empty_cases():
    x = torch.randn((256, 256), device="cuda").to(torch.bfloat16)
    q64 = fq.fq_quantize(x, fq.FQ_CRIT_NONE, 0.0, capacity=0, block=64)
    with pytest.raises(fq.FqError) as e:
        fq.fq_gemm_biased(fq.FQ_OP_NT, q64, q64)
    assert e.value.status == fq.FQ_ERR_BLOCK
    a = fq.QTensor(256, 0)
    b = fq.QTensor(128, 0, capacity=0)
    fq.fq_quantize(torch.empty((256, 0), dtype=torch.bfloat16, device="cuda"), fq.FQ_CRIT_NONE, 0.0, out=a)
    fq.fq_quantize(torch.empty((128, 0), dtype=torch.bfloat16, device="cuda"), fq.FQ_CRIT_NONE, 0.0, out=b)
    c = fq.fq_gemm_biased(fq.FQ_OP_NT, a, b, out=torch.full((256, 128), 3.0, device="cuda"))
    assert (c == 0).all().item()


@pytest.mark.parametrize("cfg", ["cfg2", "cfg3"])
def test_full_size(cfg):
    """Configs 2 and 3 at full size in the launch configuration the benchmark times: the oracle on
    at least 64 whole 128 x 128 tiles including one in every block-row that holds a flagged block,
    and the whole output against fq_gemm (which the other tests hold to the oracle bit for bit)."""
    wl = synth.config2() if cfg == "cfg2" else synth.config3()
    ga = fq.fq_quantize(gu.to_device_bf16(wl.X), fq.FQ_CRIT_ABSMAX_GT, wl.theta)
    gb = fq.fq_quantize(gu.to_device_bf16(wl.W), fq.FQ_CRIT_NONE, 0.0, capacity=0)
    oa = fqo.quantize(wl.X, 128, fqo.CRIT_ABSMAX_GT, wl.theta)
    ob = fqo.quantize(wl.W, 128, fqo.CRIT_NONE, 0.0)
    gu.announce(f"{cfg}: biased gemm")
    c32 = fq.fq_gemm_biased(fq.FQ_OP_NT, ga, gb)
    exact = fq.fq_gemm(fq.FQ_OP_NT, ga, gb)
    torch.cuda.synchronize()
    assert torch.isfinite(c32).all().item()
    whole = ((c32.double() - exact.double()).abs().max() / exact.double().abs().max()).item()
    print(f"{cfg}: whole output against fq_gemm: max |diff| / max |ref| = {whole:.3e}", flush=True)
    assert whole <= TOL
    rng = np.random.default_rng(1)
    windows = _tile_windows(rng, wl.M, wl.N, sorted({int(b) // oa.nbc for b in wl.flagged_blocks}))
    assert len(windows) >= 64
    ref_max = exact.abs().max().item()
    worst = 0.0
    for (i0, i1, j0, j1) in windows:
        ref, _ = fqo.gemm_window(fqo.OP_NT, oa, ob, (i0, i1, j0, j1), want_bf16=True)
        got = c32[i0:i1, j0:j1].cpu().numpy()
        worst = max(worst, float(np.abs(got.astype(np.float64) - ref[:, j0:j1]).max() / ref_max))
        del ref
    print(f"{cfg}: {len(windows)} oracle tiles: max |diff| / max |ref| = {worst:.3e}", flush=True)
    assert worst <= TOL
