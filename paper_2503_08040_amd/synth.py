"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module draws random matrices and rounds them to bf16.  It holds none of
the method's arithmetic (no quantization, no thresholds decided from codes):
both the HIP library and the CPU oracle receive the same arrays from here.

The recipes stand in for the paper's workloads (GLU-transformer activations,
Sec. 4.1): outlier magnitudes follow Table 1 (channel-wise 124-623 for GLU
models), outliers are sparse even inside an outlier channel (pattern P3), occur
in isolated blocks (P2) or along whole channels (Sec. 6.3, channel-wise
fallback pattern), and are orders of magnitude above the N(0,1) bulk (P1).

All matrices are returned as uint16 arrays of bf16 bit patterns.
"""
from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

BLOCK = 128


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    w = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (w >> np.uint32(16)) & np.uint32(1)
    return ((w + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng, shape, std=1.0) -> np.ndarray:
    x = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return to_bf16_bits(x)


@dataclass
class Workload:
    """One benchmark / parity configuration."""
    name: str
    M: int
    K: int
    N: int
    X: Optional[np.ndarray] = None      # [M, K] activations (bf16 bits)
    W: Optional[np.ndarray] = None      # [N, K] weights
    dY: Optional[np.ndarray] = None     # [M, N] output gradient (backward configs)
    theta: float = 10.0                 # fallback threshold for the A operand
    flagged_blocks: Optional[np.ndarray] = None   # block ids built to exceed theta
    notes: Dict[str, object] = field(default_factory=dict)


def _spike_block_columns(rng, x_f32, bi, bk, n_cols, lo, hi, density=0.25):
    """Replace a sparse subset of `n_cols` columns of block (bi, bk) by +-U(lo, hi)."""
    r0, c0 = bi * BLOCK, bk * BLOCK
    rows = min(BLOCK, x_f32.shape[0] - r0)
    cols = rng.choice(min(BLOCK, x_f32.shape[1] - c0), size=n_cols, replace=False)
    for c in cols:
        hit = rng.random(rows) < density
        hit[rng.integers(rows)] = True
        mag = rng.uniform(lo, hi, size=rows).astype(np.float32)
        sign = np.where(rng.random(rows) < 0.5, -1.0, 1.0).astype(np.float32)
        seg = x_f32[r0:r0 + rows, c0 + c]
        seg[hit] = (mag * sign)[hit]


def config1(seed: int = 0) -> Workload:
    """Forward, M=256 K=512 N=512; one of the 8 X blocks holds 4 channels x100."""
    rng = np.random.default_rng(seed)
    M, K, N = 256, 512, 512
    x = rng.standard_normal((M, K), dtype=np.float32)
    bi, bk = 1, 2
    cols = bk * BLOCK + rng.choice(BLOCK, size=4, replace=False)
    x[bi * BLOCK:(bi + 1) * BLOCK, cols] *= np.float32(100.0)
    w = normal_bf16(rng, (N, K), 0.02)
    return Workload("cfg1_fwd_256x512x512", M, K, N, X=to_bf16_bits(x), W=w, theta=10.0,
                    flagged_blocks=np.array([bi * (K // BLOCK) + bk]))


def config2(seed: int = 0, M: int = 4096, K: int = 4096, N: int = 11008,
            frac: float = 0.05) -> Workload:
    """GLU up/gate projection; ~5 % of X blocks hold sparse outlier channels 50-200."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K), dtype=np.float32)
    nbr, nbc = -(-M // BLOCK), -(-K // BLOCK)
    n_fb = int(round(frac * nbr * nbc))
    ids = np.sort(rng.choice(nbr * nbc, size=n_fb, replace=False))
    for b in ids:
        _spike_block_columns(rng, x, int(b) // nbc, int(b) % nbc, int(rng.integers(1, 5)),
                             50.0, 200.0)
    w = normal_bf16(rng, (N, K), 0.02)
    return Workload(f"cfg2_glu_upgate_{M}x{K}x{N}", M, K, N, X=to_bf16_bits(x), W=w, theta=10.0,
                    flagged_blocks=ids)


def config3(seed: int = 0, M: int = 4096, K: int = 11008, N: int = 4096,
            n_channels: int = 4) -> Workload:
    """GLU down projection; X = silu(A) * B with a few whole channels x100."""
    rng = np.random.default_rng(seed)
    a = bf16_bits_to_f32(normal_bf16(rng, (M, K)))
    b = bf16_bits_to_f32(normal_bf16(rng, (M, K)))
    x = (a / (1.0 + np.exp(-a))) * b
    del a, b
    nbr, nbc = -(-M // BLOCK), -(-K // BLOCK)
    bcols = np.sort(rng.choice(nbc, size=min(n_channels, nbc), replace=False))
    for bc in bcols:
        c = int(bc) * BLOCK + int(rng.integers(min(BLOCK, K - int(bc) * BLOCK)))
        x[:, c] *= np.float32(100.0)
    ids = np.sort(np.array([r * nbc + int(c) for r in range(nbr) for c in bcols]))
    w = normal_bf16(rng, (N, K), 0.02)
    return Workload(f"cfg3_glu_down_{M}x{K}x{N}", M, K, N, X=to_bf16_bits(x.astype(np.float32)),
                    W=w, theta=30.0, flagged_blocks=ids)


def config4(seed: int = 0) -> Workload:
    """Backward of config 1: dY = 1e-3 * Student-t(3); theta set so 2 of 8 dY blocks fall back."""
    base = config1(seed)
    rng = np.random.default_rng(seed + 1000)
    M, K, N = base.M, base.K, base.N
    dy = (1e-3 * rng.standard_t(3.0, size=(M, N))).astype(np.float32)
    dyb = to_bf16_bits(dy)
    # harness-side TopK (Sec. 4.4): threshold between the 2nd and 3rd largest block abs-max
    v = np.abs(bf16_bits_to_f32(dyb)).reshape(M // BLOCK, BLOCK, N // BLOCK, BLOCK).max(axis=(1, 3))
    s = np.sort(v.ravel())[::-1]
    theta = float(np.float32(0.5) * (s[1] + s[2]))
    ids = np.sort(np.nonzero(v.ravel() > theta)[0])
    return Workload("cfg4_bwd_256x512x512", M, K, N, X=base.X, W=base.W, dY=dyb, theta=theta,
                    flagged_blocks=ids)


def config5(seed: int = 0, frac: float = 0.05, placement: str = "random",
            M: int = 8192, K: int = 8192, N: int = 8192) -> Workload:
    """Square GEMM; exactly round(frac * blocks) X blocks get one column x100.

    placement "random": flagged blocks drawn uniformly; "sequential": packed
    into the fewest block-rows (the worst case of Sec. 6.3)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K), dtype=np.float32)
    nbr, nbc = -(-M // BLOCK), -(-K // BLOCK)
    n_fb = int(round(frac * nbr * nbc))
    if placement == "random":
        ids = np.sort(rng.choice(nbr * nbc, size=n_fb, replace=False))
    elif placement == "sequential":
        ids = np.arange(n_fb)
    else:
        raise ValueError(placement)
    for b in ids:
        bi, bk = int(b) // nbc, int(b) % nbc
        c = bk * BLOCK + int(rng.integers(min(BLOCK, K - bk * BLOCK)))
        x[bi * BLOCK:(bi + 1) * BLOCK, c] *= np.float32(100.0)
    w = normal_bf16(rng, (N, K), 1.0)
    return Workload(f"cfg5_square_{M}_f{frac:g}_{placement}", M, K, N, X=to_bf16_bits(x), W=w,
                    theta=10.0, flagged_blocks=ids)
