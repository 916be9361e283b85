"""Helpers for the GPU parity tests: move synthetic inputs to the device, bring
library outputs back, undo the documented tile order with plain index
arithmetic, and compare with the CPU oracle's outputs."""
import sys

import numpy as np

import paper_2503_08040_amd as fq
from oracle import fqo

B = fq.FQ_BLOCK


def announce(msg):
    print(f"[gpu-step] {msg}", flush=True)
    sys.stdout.flush()


def to_device_bf16(bits: np.ndarray):
    import torch
    return torch.from_numpy(bits.view(np.int16).copy()).cuda().view(torch.bfloat16)


def tile_index_map():
    """dense (r, c) -> byte offset inside a 16 KiB block, from the formula in fq.h."""
    r = np.arange(B)[:, None]
    c = np.arange(B)[None, :]
    return ((r // 32) * 4 + c // 32) * 1024 + ((r % 32) + 32 * ((c % 32) // 16)) * 16 + c % 16


_MAP = tile_index_map()


def untile_block(blk16k: np.ndarray) -> np.ndarray:
    return blk16k[_MAP]


def untile(tiled: np.ndarray, rows, cols):
    """tiled: [nbr*nbc, 16384] -> (dense [rows, cols], padded [nbr*128, nbc*128])."""
    nbr, nbc = -(-rows // B), -(-cols // B)
    full = tiled.reshape(nbr, nbc, B * B)[:, :, _MAP]          # [nbr, nbc, 128, 128]
    full = full.transpose(0, 2, 1, 3).reshape(nbr * B, nbc * B)
    return full[:rows, :cols], full


def compare_quantized(gq: fq.QTensor, oq: fqo.QTensor, label=""):
    """Bit-exact comparison of every quantizer output with the oracle's."""
    import torch
    torch.cuda.synchronize()
    rows, cols, nbr, nbc = oq.rows, oq.cols, oq.nbr, oq.nbc
    codes, padded = untile(gq.view("codes").cpu().numpy(), rows, cols)
    assert np.array_equal(codes, oq.codes), f"{label}: codes differ"
    pad = padded.copy()
    pad[:rows, :cols] = 0
    assert not pad.any(), f"{label}: padding of edge blocks is not zero"
    assert np.array_equal(gq.view("scales").cpu().numpy().view(np.uint32),
                          oq.scales.view(np.uint32)), f"{label}: scales differ"
    assert np.array_equal(gq.view("mask").cpu().numpy(), oq.mask), f"{label}: mask differs"
    n = int(gq.view("fb_count").cpu().numpy()[0])
    assert n == int(oq.fb_count[0]), f"{label}: fb_count {n} != {int(oq.fb_count[0])}"
    slot = gq.view("fb_slot").cpu().numpy()
    if gq.capacity > 0:
        # the ascending list of flagged block ids, bit for bit (the lowest `capacity` ids when
        # more blocks are flagged than there are slots)
        keep = min(n, gq.capacity)
        lst = gq.view("fb_list").cpu().numpy()[:keep]
        assert np.array_equal(lst, oq.fb_list[:keep]), f"{label}: fb_list differs"

    flagged = oq.mask.astype(bool)
    assert np.all(slot[~flagged] == -1), f"{label}: unflagged block has a slot"
    if n <= gq.capacity:
        assert sorted(slot[flagged].tolist()) == list(range(n)), f"{label}: slots not a bijection"
    if gq.c.codes_t:
        ct, _ = untile(gq.view("codes_t").cpu().numpy(), cols, rows)
        assert np.array_equal(ct, oq.codes.T), f"{label}: transposed codes differ"
    if n == 0 or n > gq.capacity:
        return
    res = gq.view("res_codes").cpu().numpy()
    rsc = gq.view("res_scales").cpu().numpy()
    res_t = gq.view("res_codes_t").cpu().numpy() if gq.c.res_codes_t else None
    for b in oq.fb_list[:n]:
        bi, bk = int(b) // nbc, int(b) % nbc
        s = int(slot[bi, bk])
        want = np.zeros((B, B), np.int8)
        blk = oq.res_codes[bi * B:(bi + 1) * B, bk * B:(bk + 1) * B]
        want[:blk.shape[0], :blk.shape[1]] = blk
        assert np.array_equal(untile_block(res[s]), want), f"{label}: residual codes of block {b}"
        assert rsc[s].view(np.uint32) == oq.res_scales[bi, bk].view(np.uint32), \
            f"{label}: residual scale of block {b}"
        if res_t is not None:
            assert np.array_equal(untile_block(res_t[s]), want.T), \
                f"{label}: transposed residual codes of block {b}"


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref| (the output-level error measure of the tests)."""
    d = np.abs(got.astype(np.float64) - ref.astype(np.float64)).max() if got.size else 0.0
    s = np.abs(ref.astype(np.float64)).max() if ref.size else 0.0
    return float(d / s) if s > 0 else float(d)
