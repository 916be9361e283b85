"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/fq.h declares, and rejects bad arguments before touching
the device."""
import ctypes as C
import os
import re

import pytest

import paper_2503_08040_amd as fq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "fq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = fq.lib()
    names = _declared_symbols()
    assert set(names) == set(fq.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_qtensor_bytes_and_bind():
    assert fq.fq_qtensor_bytes(0, 0, 0) > 0
    nb = 2 * 4
    small = fq.fq_qtensor_bytes(256, 512, 0)
    big = fq.fq_qtensor_bytes(256, 512, nb)
    assert big - small >= nb * fq.FQ_BLOCK_BYTES - 512
    assert fq.fq_qtensor_bytes(256, 512, nb, True) - big >= 2 * nb * fq.FQ_BLOCK_BYTES - 512
    assert fq.fq_qtensor_bytes(256, 512, nb + 1) == 0          # capacity beyond nbr*nbc
    assert fq.fq_qtensor_bytes(-1, 5, 0) == 0
    assert fq.fq_qtensor_bytes(256, 512, 1, block=64) == 0
    t = fq.fq_qtensor()
    base = 0x10000
    assert fq.lib().fq_qtensor_bind(C.c_void_p(base), 130, 200, 128, 3, 1, C.byref(t)) == fq.FQ_OK
    assert (t.rows, t.cols, t.block, t.capacity) == (130, 200, 128, 3)
    ptrs = [t.codes, t.codes_t, t.scales, t.mask, t.fb_counters, t.fb_list, t.fb_slot, t.res_codes,
            t.res_codes_t, t.res_scales]
    assert all(p and p % 256 == 0 for p in ptrs) and len(set(ptrs)) == len(ptrs)
    assert t.fb_count == t.fb_counters and t.epoch == 0
    assert max(ptrs) < base + fq.fq_qtensor_bytes(130, 200, 3, True)
    assert fq.lib().fq_qtensor_bind(C.c_void_p(base + 8), 130, 200, 128, 3, 1, C.byref(t)) == fq.FQ_ERR_SHAPE
    assert fq.lib().fq_qtensor_bind(None, 130, 200, 128, 3, 1, C.byref(t)) == fq.FQ_ERR_NULL
    assert fq.lib().fq_qtensor_bind(C.c_void_p(base), 130, 200, 64, 3, 1, C.byref(t)) == fq.FQ_ERR_BLOCK


def _fake(rows, cols, cap=1, want_t=True, crit=fq.FQ_CRIT_NONE):
    """A struct with non-NULL fake pointers: valid for host-side validation only."""
    t = fq.fq_qtensor()
    assert fq.lib().fq_qtensor_bind(C.c_void_p(0x100000), rows, cols, 128, cap, int(want_t),
                                    C.byref(t)) == fq.FQ_OK
    t.criterion = crit
    return t


def test_quantize_rejects_bad_arguments_on_the_host():
    L = fq.lib()
    t = _fake(256, 256)
    x = C.c_void_p(0x2000)
    q = lambda *a: L.fq_quantize(*a)
    assert q(x, 256, 256, 256, 128, 0, 0.0, None, None) == fq.FQ_ERR_NULL
    assert q(None, 256, 256, 256, 128, 0, 0.0, C.byref(t), None) == fq.FQ_ERR_NULL
    assert q(x, 256, 256, 256, 64, 0, 0.0, C.byref(t), None) == fq.FQ_ERR_BLOCK
    assert q(x, 256, 256, 255, 128, 0, 0.0, C.byref(t), None) == fq.FQ_ERR_SHAPE     # ld < cols
    assert q(x, -1, 256, 256, 128, 0, 0.0, C.byref(t), None) == fq.FQ_ERR_SHAPE
    assert q(x, 128, 256, 256, 128, 0, 0.0, C.byref(t), None) == fq.FQ_ERR_SHAPE     # shape != out
    assert q(x, 256, 256, 256, 128, 7, 0.0, C.byref(t), None) == fq.FQ_ERR_ENUM
    t0 = _fake(256, 256, cap=0)
    assert q(x, 256, 256, 256, 128, 1, 0.0, C.byref(t0), None) == fq.FQ_ERR_CAPACITY
    t.codes = None
    assert q(x, 256, 256, 256, 128, 0, 0.0, C.byref(t), None) == fq.FQ_ERR_NULL


def test_gemm_rejects_bad_arguments_on_the_host():
    L = fq.lib()
    out = C.c_void_p(0x3000)
    A, Bm = _fake(256, 512, crit=fq.FQ_CRIT_ABSMAX_GT), _fake(384, 512)
    g = lambda *a: L.fq_gemm(*a)
    assert g(0, None, C.byref(Bm), out, 0, 384, None) == fq.FQ_ERR_NULL
    assert g(0, C.byref(A), C.byref(Bm), None, 0, 384, None) == fq.FQ_ERR_NULL
    assert g(5, C.byref(A), C.byref(Bm), out, 0, 384, None) == fq.FQ_ERR_ENUM
    assert g(0, C.byref(A), C.byref(Bm), out, 9, 384, None) == fq.FQ_ERR_ENUM
    assert g(0, C.byref(A), C.byref(Bm), out, 0, 383, None) == fq.FQ_ERR_SHAPE        # ldc < N
    assert g(0, C.byref(A), C.byref(_fake(384, 640)), out, 0, 384, None) == fq.FQ_ERR_SHAPE
    # NN needs A.cols == B.rows, TN needs A.rows == B.rows
    assert g(1, C.byref(A), C.byref(Bm), out, 0, 512, None) == fq.FQ_ERR_SHAPE
    assert g(2, C.byref(A), C.byref(Bm), out, 0, 512, None) == fq.FQ_ERR_SHAPE
    # the B operand must be plain block INT8 (Alg. 1 defines fallback for A only)
    Bf = _fake(384, 512, crit=fq.FQ_CRIT_ABSMAX_GT)
    assert g(0, C.byref(A), C.byref(Bf), out, 0, 384, None) == fq.FQ_ERR_ENUM
    # backward forms need the transposed copies
    Bnt = _fake(512, 384, want_t=False)
    assert g(1, C.byref(A), C.byref(Bnt), out, 0, 384, None) == fq.FQ_ERR_NULL
    Ant = _fake(256, 512, want_t=False, crit=fq.FQ_CRIT_ABSMAX_GT)
    assert g(2, C.byref(Ant), C.byref(_fake(256, 384)), out, 0, 384, None) == fq.FQ_ERR_NULL
    A.block = 64
    assert g(0, C.byref(A), C.byref(Bm), out, 0, 384, None) == fq.FQ_ERR_BLOCK
    A.block = 128
    p = lambda *a: L.fq_gemm_debug_partials(*a)
    assert p(0, C.byref(A), C.byref(Bm), 4, 0, out, None) == fq.FQ_ERR_SHAPE          # nkb = 4
    assert p(0, C.byref(A), C.byref(Bm), -1, 0, out, None) == fq.FQ_ERR_SHAPE
    assert p(0, C.byref(A), C.byref(Bm), 0, 0, None, None) == fq.FQ_ERR_NULL


def test_status_strings():
    for s in range(0, -8, -1):
        assert fq.status_string(s) and "unknown" not in fq.status_string(s)
    assert "unknown" in fq.status_string(-99)


def test_untile_rejects_bad_arguments():
    L = fq.lib()
    assert L.fq_codes_to_rowmajor(None, 4, 4, C.c_void_p(0x10), None) == fq.FQ_ERR_NULL
    assert L.fq_codes_to_rowmajor(C.c_void_p(0x10), -4, 4, C.c_void_p(0x10), None) == fq.FQ_ERR_SHAPE
    assert L.fq_codes_to_rowmajor(None, 0, 4, None, None) == fq.FQ_OK


def test_tile_plan_covers_the_output_and_never_costs_more():
    """fq_gemm_tile_plan (host-only): 256x256 tiles over the first block columns, 128x384 tiles
    over the rest; every block column is covered exactly once, and the plan is only split when
    that shortens the last round (costs in units of one 256x256 tile per compute unit)."""
    import itertools
    import random
    rng = random.Random(0)
    cases = [(4096, 11008, 256), (8192, 8192, 256), (4096, 4096, 256), (11008, 4096, 256), (1, 1, 256)]
    cases += [(rng.randint(1, 6000), rng.randint(1, 14000), rng.choice([1, 3, 8, 64, 256, 304]))
              for _ in range(300)]
    split = 0
    for rows, cols, cus in cases:
        n_main, main_tj, tail_tj = fq.fq_gemm_tile_plan(rows, cols, cus)
        nib, njb = -(-rows // 128), -(-cols // 128)
        tiles_i, tiles_j = -(-nib // 2), -(-njb // 2)
        assert n_main == tiles_i * main_tj and 0 <= main_tj <= tiles_j and tail_tj >= 0
        if tail_tj == 0:
            assert main_tj == tiles_j
            continue
        split += 1
        tail_cols = njb - 2 * main_tj
        assert tail_cols > 0 and 3 * (tail_tj - 1) < tail_cols <= 3 * tail_tj
        rounds = lambda n: -(-n // cus)
        assert rounds(n_main) + 0.75 * rounds(nib * tail_tj) < rounds(tiles_i * tiles_j)
    assert split > 10
    assert fq.fq_gemm_tile_plan(4096, 11008, 256) == (512, 32, 8)
    assert fq.fq_gemm_tile_plan(8192, 8192, 256) == (1024, 32, 0)
    p = (C.c_int32 * 3)()
    assert fq.lib().fq_gemm_tile_plan(-1, 5, 4, p) == fq.FQ_ERR_SHAPE
    assert fq.lib().fq_gemm_tile_plan(5, 5, 4, None) == fq.FQ_ERR_NULL
