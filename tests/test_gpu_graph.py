"""The quantize + GEMM step recorded into a HIP graph and replayed: every replay, with new
contents in the captured input buffer and the program's own eager work in between, gives the
result of the eager calls bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2503_08040_amd as fq
from paper_2503_08040_amd import synth
from tests import gpu_util as gu

F32 = np.float32


def _inputs(seed, shape):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(shape).astype(F32)
    for _ in range(1 + seed % 5):
        x[rng.integers(shape[0]), rng.integers(shape[1])] = 90.0      # a few flagged blocks
    return gu.to_device_bf16(synth.to_bf16_bits(x))


def test_step_replays_from_a_graph():
    M, K, N = 512, 640, 768
    w = _inputs(100, (N, K)) * 0.02
    qw = fq.fq_quantize(w, fq.FQ_CRIT_NONE, 0.0, capacity=0)
    x_static = _inputs(0, (M, K)).clone()
    qx = fq.QTensor(M, K)
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):           # warm-up on the capture stream, as torch asks for
        fq.fq_quantize(x_static, fq.FQ_CRIT_ABSMAX_GT, 8.0, out=qx)
        fq.fq_gemm(fq.FQ_OP_NT, qx, qw, out=y)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    gu.announce("capturing quantize + gemm")
    with torch.cuda.graph(graph):
        fq.fq_quantize(x_static, fq.FQ_CRIT_ABSMAX_GT, 8.0, out=qx)
        fq.fq_gemm(fq.FQ_OP_NT, qx, qw, out=y)

    counts = []
    for rep in range(5):
        x_new = _inputs(rep + 1, (M, K))
        # eager reference through a tensor of its own
        q_ref = fq.fq_quantize(x_new, fq.FQ_CRIT_ABSMAX_GT, 8.0)
        y_ref = fq.fq_gemm(fq.FQ_OP_NT, q_ref, qw)
        n_ref = fq.fq_qtensor_check(q_ref)
        x_static.copy_(x_new)
        gu.announce(f"replay {rep}")
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref), f"replay {rep}"
        assert torch.equal(qx.view("codes"), q_ref.view("codes"))
        assert torch.equal(qx.view("mask"), q_ref.view("mask"))
        assert int(qx.view("fb_count").cpu()[0]) == n_ref
        counts.append(n_ref)
    assert len(set(counts)) > 1          # the replays really saw different inputs

    # eager calls into the captured tensor between replays: counts and slots stay right
    for rep in range(3):
        for j in range(rep + 1):         # one, two, three eager calls in a row
            x_new = _inputs(20 + 3 * rep + j, (M, K))
            q_ref = fq.fq_quantize(x_new, fq.FQ_CRIT_ABSMAX_GT, 8.0)
            n_ref = fq.fq_qtensor_check(q_ref)
            gu.announce(f"eager call {j} into the captured tensor after replay round {rep}")
            fq.fq_quantize(x_new, fq.FQ_CRIT_ABSMAX_GT, 8.0, out=qx)
            assert fq.fq_qtensor_check(qx) == n_ref
            slot = qx.view("fb_slot").cpu().numpy()
            assert sorted(slot[slot >= 0].tolist()) == list(range(n_ref))
            assert torch.equal(qx.view("fb_list")[:n_ref], q_ref.view("fb_list")[:n_ref])
            assert torch.equal(fq.fq_gemm(fq.FQ_OP_NT, qx, qw), fq.fq_gemm(fq.FQ_OP_NT, q_ref, qw))
        x_new = _inputs(40 + rep, (M, K))
        q_ref = fq.fq_quantize(x_new, fq.FQ_CRIT_ABSMAX_GT, 8.0)
        y_ref = fq.fq_gemm(fq.FQ_OP_NT, q_ref, qw)
        x_static.copy_(x_new)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref), f"replay after eager calls, round {rep}"
        assert int(qx.view("fb_count").cpu()[0]) == fq.fq_qtensor_check(q_ref)
