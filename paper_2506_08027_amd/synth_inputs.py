"""Seeded synthetic tensors with the shapes and value structure of 8B-class LLM linear layers.

These stand in for the paper's (unavailable) training tensors: hidden size 4096, 32 heads, 8 KV
heads of 128 channels (Section 3.1), FFN width 14336. They serve the GPU tests, the benchmark and
the CPU oracle alike and contain none of the method's arithmetic: only random draws, the usual
round-to-nearest cast to BF16 and the placement of special blocks.

Everything is generated on the host with ``numpy.random.default_rng(seed)`` in FP32. BF16 tensors
are returned as ``uint16`` bit patterns (what both the oracle and the device buffers consume).
"N(0, x)" means standard deviation x.
"""
from __future__ import annotations

import numpy as np

K_BLOCK = 32
E4M3_MAX = 448.0


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round FP32 to BF16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    r = np.where(nan, (u >> 16) | 0x40, r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def activations(rows: int, cols: int, seed: int = 2, bf16: bool = True) -> np.ndarray:
    """N(0,1) times a per-channel lognormal(0,1) gain; 0.1 % of channels (at least one) x50."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols), dtype=np.float32)
    gain = np.exp(rng.standard_normal(cols)).astype(np.float32)
    n_out = max(1, round(cols * 0.001))
    out_cols = rng.choice(cols, size=n_out, replace=False)
    gain[out_cols] *= 50.0
    x *= gain[None, :]
    return to_bf16_bits(x) if bf16 else x


def weights(rows: int, cols: int, seed: int = 4, bf16: bool = True) -> np.ndarray:
    """N(0, 0.02)."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(0.02)
    return to_bf16_bits(w) if bf16 else w


def gradients(rows: int, cols: int, seed: int = 3, spikes: bool = False, bf16: bool = False) -> np.ndarray:
    """N(0, 1e-3); with ``spikes`` 0.5 % of the entries are multiplied by 100."""
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(1e-3)
    if spikes:
        mask = rng.random((rows, cols), dtype=np.float32) < np.float32(0.005)
        g[mask] *= np.float32(100.0)
    return to_bf16_bits(g) if bf16 else g


def _block_with_amax(rng, amax: np.float32) -> np.ndarray:
    """32 FP32 values with magnitudes below ``amax`` except one element equal to +-amax."""
    v = (rng.uniform(-0.9, 0.9, K_BLOCK).astype(np.float32) * amax).astype(np.float32)
    v[rng.integers(K_BLOCK)] = amax if rng.random() < 0.5 else -amax
    return v


def special_blocks(seed: int = 0):
    """The degenerate 32-element blocks of the tiny configuration, as (name, values) pairs."""
    rng = np.random.default_rng(seed + 1000)
    out = []
    z = np.zeros(K_BLOCK, np.float32)
    z[1::2] = -0.0
    out.append(("zero", z))
    sub = (rng.integers(1, 1 << 23, K_BLOCK).astype(np.uint32)
           | (rng.integers(0, 2, K_BLOCK).astype(np.uint32) << 31)).view(np.float32)
    out.append(("subnormal", sub.copy()))
    tiny = sub.copy()
    tiny[3] = np.float32(2.0 ** -137)       # exact tie between 0 and the smallest subnormal code
    tiny[4] = np.float32(-(2.0 ** -137))
    tiny[5] = np.float32(2.0 ** -137 * 1.5)
    tiny[6] = np.float32(2.0 ** -149)
    out.append(("subnormal_ties", tiny))
    for k in (-130, -129, -128, -127, -126, -8, 0, 7, 119):
        a = np.float32(E4M3_MAX * 2.0 ** k)
        for tag, val in (("", a), ("_up", np.nextafter(a, np.float32(np.inf))),
                         ("_down", np.nextafter(a, np.float32(0)))):
            out.append((f"amax448p{k}{tag}", _block_with_amax(rng, np.float32(val))))
    base = rng.standard_normal(K_BLOCK).astype(np.float32)
    for name, pos_val in (("pinf", [(7, np.inf)]), ("ninf", [(9, -np.inf)]), ("nan", [(11, np.nan)]),
                          ("nan_inf", [(2, np.nan), (30, np.inf)]),
                          ("inf_big", [(0, np.inf), (1, np.float32(3.0e38)), (2, np.float32(-2.0 ** 127))])):
        v = base.copy()
        for p, x in pos_val:
            v[p] = x
        out.append((name, v))
    return out


def tiny_with_specials(n: int = 256, seed: int = 0) -> np.ndarray:
    """[n x n] FP32: N(0,1), 1 % of entries x100, then every special block written once along a
    row (32 consecutive columns) and once down a column (32 consecutive rows)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, n), dtype=np.float32)
    mask = rng.random((n, n), dtype=np.float32) < np.float32(0.01)
    x[mask] *= np.float32(100.0)
    blocks = special_blocks(seed)
    nb = n // K_BLOCK
    # Row-direction copies live in rows [0, n/2), column-direction copies in rows [n/2, n) so that
    # the two families never overwrite each other.
    slots_row = [(r, b) for r in range(0, n // 2, 2) for b in range(nb)]
    slots_col = [(b, c) for c in range(1, n, 3) for b in range(nb // 2, nb)]
    prm = np.random.default_rng(seed + 2000)
    prm.shuffle(slots_row)
    prm.shuffle(slots_col)
    if len(blocks) > len(slots_row) or len(blocks) > len(slots_col):
        raise ValueError("matrix too small for the special blocks")
    for (name, v), (r, b) in zip(blocks, slots_row):
        x[r, b * K_BLOCK:(b + 1) * K_BLOCK] = v
    for (name, v), (b, c) in zip(blocks, slots_col):
        x[b * K_BLOCK:(b + 1) * K_BLOCK, c] = v
    return x


def fp4_hard_cases(rows: int, cols: int, seed: int) -> np.ndarray:
    """N(0,1) with outliers, plus blocks whose elements sit on every rounding tie and whose amax sits on, just
    above and just below the scale boundary 6 * 2^k, for k over the whole exponent range; NaN / Inf blocks."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols), dtype=np.float32)
    x[rng.random((rows, cols)) < 0.01] *= np.float32(100.0)
    ties = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0, 0.0, 0.24999999, 0.25000003,
                     2.4999998, 2.5000002, 4.9999995, 5.0000005, 5.9999995], np.float64)
    ks = [-149, -140, -129, -128, -127, -126, -125, -60, -1, 0, 1, 50, 124, 125]
    slot = 0
    for k in ks:
        for top in (6.0, np.nextafter(np.float32(6.0), np.float32(7.0)), np.nextafter(np.float32(6.0), np.float32(0.0)), 4.0, 3.0):
            blk = rng.choice(ties, 32) * rng.choice([-1.0, 1.0], 32)
            blk[rng.integers(32)] = float(top)
            with np.errstate(over="ignore", under="ignore"):
                v = np.ldexp(blk, k).astype(np.float32)
            r, b = (slot * 7) % rows, (slot * 3) % (cols // 32)
            x[r, 32 * b:32 * b + 32] = v                                   # along a row
            c, rb = (slot * 5 + 1) % cols, (slot * 2 + 1) % (rows // 32)
            x[32 * rb:32 * rb + 32, c] = v                                 # down a column
            slot += 1
    x[1, 0] = np.nan
    x[3, 40] = np.inf
    x[rows - 1, cols - 1] = -np.inf
    x[rows - 2, cols - 2] = np.nan
    x[5, 64:96] = 0.0
    x[5, 65] = -0.0
    return x


def fp6_hard_cases(rows: int, cols: int, seed: int, top: float) -> np.ndarray:
    """N(0,1) with outliers, plus blocks drawn from the grid k * 2^-6 (it holds every magnitude of both 6-bit formats
    and every midpoint between two of them) and from its neighbours one FP32 step away, with the block maximum on,
    just above and just below `top` * 2^k (the scale boundary of the format whose largest magnitude is `top`), for k
    over the whole exponent range; NaN / Inf blocks; signed zeros."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols), dtype=np.float32)
    x[rng.random((rows, cols)) < 0.01] *= np.float32(100.0)
    ks = [-149, -140, -131, -130, -129, -128, -127, -126, -60, -1, 0, 1, 50, 120, 122]
    slot = 0
    t32 = np.float32(top)
    for k in ks:
        for peak in (t32, np.nextafter(t32, np.float32(2 * top)), np.nextafter(t32, np.float32(0.0)), np.float32(top / 2),
                     np.nextafter(np.float32(top / 2), np.float32(top))):
            grid = (rng.integers(0, int(top * 64) + 1, 32).astype(np.float32) / np.float32(64.0)).astype(np.float32)
            nudge = rng.integers(-1, 2, 32)
            blk = np.where(nudge > 0, np.nextafter(grid, np.float32(1e9)), np.where(nudge < 0, np.nextafter(grid, np.float32(-1.0)), grid))
            blk = np.minimum(np.abs(blk), float(peak)) * rng.choice([-1.0, 1.0], 32)
            blk[rng.integers(32)] = float(peak)
            with np.errstate(over="ignore", under="ignore"):
                v = np.ldexp(blk.astype(np.float64), k).astype(np.float32)
            r, b = (slot * 7) % rows, (slot * 3) % (cols // 32)
            x[r, 32 * b:32 * b + 32] = v
            c, rb = (slot * 5 + 1) % cols, (slot * 2 + 1) % (rows // 32)
            x[32 * rb:32 * rb + 32, c] = v
            slot += 1
    x[1, 0] = np.nan
    x[3, 40] = np.inf
    x[rows - 1, cols - 1] = -np.inf
    x[rows - 2, cols - 2] = np.nan
    x[5, 64:96] = 0.0
    x[5, 65] = -0.0
    return x
