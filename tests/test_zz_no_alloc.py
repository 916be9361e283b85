"""fq_rmsnorm_backward_static (the entry point for callers that cannot allocate device memory)
against fq_rmsnorm_backward: same kernels, the library's built-in scratch buffer instead of a
caller workspace.  Two calls in a row, the second on a smaller input, each bit-identical to the
allocating entry point; sizes beyond the built-in buffer are refused."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2503_08040_amd as fq
from paper_2503_08040_amd import synth
from tests import gpu_util as gu

F32 = np.float32


def _case(rows, cols, seed):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((rows, cols)) * np.exp(rng.standard_normal((rows, 1)))).astype(F32)
    w = (1.0 + 0.2 * rng.standard_normal(cols)).astype(F32)
    dy = (rng.standard_t(3.0, size=(rows, cols)) * 1e-2).astype(F32)
    return tuple(gu.to_device_bf16(synth.to_bf16_bits(v)) for v in (x, w.reshape(1, -1), dy))


def test_static_scratch_entry_point_matches_the_allocating_one():
    for rows, cols, parts in ((96, 1536, 48), (33, 300, 7)):      # the second call is smaller
        x, w, dy = _case(rows, cols, rows)
        w = w.reshape(-1)
        y, rstd, ctx = fq.fq_rmsnorm_forward(x, w, 1e-5)
        gu.announce(f"rmsnorm backward, caller workspace, shape=({rows}, {cols}) parts={parts}")
        dx_ref, dw_ref = fq.fq_rmsnorm_backward(dy, ctx, rstd, w, n_parts=parts)
        dx = torch.full((rows, cols), 7.0, dtype=torch.bfloat16, device="cuda")
        dw = torch.full((cols,), 7.0, dtype=torch.float32, device="cuda")
        gu.announce(f"rmsnorm backward, built-in scratch, shape=({rows}, {cols}) parts={parts}")
        fq.fq_rmsnorm_backward_static(dy, ctx, rstd, w, dx, dw, n_parts=parts)
        torch.cuda.synchronize()
        assert torch.equal(dx.view(torch.int16), dx_ref.view(torch.int16)), (rows, cols)
        assert torch.equal(dw.view(torch.int32), dw_ref.view(torch.int32)), (rows, cols)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    L = fq.lib()
    p = C.c_void_p(0x1000)
    too_many = fq.FQ_STATIC_SCRATCH_FLOATS // 4096 + 1
    assert L.fq_rmsnorm_backward_static(p, 4096, p, p, p, p, 8, 4096, p, 4096, p, too_many, None) \
        == fq.FQ_ERR_SCRATCH
    assert L.fq_rmsnorm_backward_static(p, 4096, p, p, p, p, 8, 4096, p, 4096, p, 0, None) == fq.FQ_ERR_SHAPE
    assert "scratch" in fq.status_string(fq.FQ_ERR_SCRATCH)
