"""Seeded synthetic pruned weight matrices.

This module only draws random dense matrices with exact zeros; it holds none of
the format's arithmetic (no bitmaps, no packing, no counting).  Both the CPU
oracle's tests and the GPU library's tests / benchmark take their inputs from
here, so the two sides always see the same host buffer.

The matrices stand in for the pruned OPT-66B / Llama2-70B weights the paper
measures on (Section 3.1 and Appendix C.1 give the shapes; Section 4.1 the 50 %
pruning ratio), which need the trained models:

  values  x ~ N(0, 0.02^2) drawn in fp32, rounded to fp16 (round to nearest
          even); a draw whose fp16 pattern is +-0 is drawn again, so a kept
          element is never a zero pattern
  mask    every element kept independently with probability `keep`
          (`row_skew=True`: row i keeps with its own p_i ~ Beta(2,2), mean 0.5,
          the stand-in for the per-row imbalance of real pruning)
  dropped elements are the all-zero pattern 0x0000

Generation is counter-based per block of rows (numpy Philox keyed by
(seed, block)), so the result does not depend on the number of worker threads.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

SIGMA = 0.02
_BLOCK_ELEMS = 1 << 22

# (rows, cols) lists, PyTorch [out_features, in_features] orientation.
OPT66B_ATTN = [("q", 9216, 9216), ("k", 9216, 9216), ("v", 9216, 9216), ("out", 9216, 9216)]
OPT66B_FFN = [("fc1", 36864, 9216), ("fc2", 9216, 36864)]
LLAMA2_70B_LAYER = [
    ("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192), ("o", 8192, 8192),
    ("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672),
]
CONFIGS = {
    0: [("w", 1024, 1024)],
    1: OPT66B_ATTN,
    2: OPT66B_FFN,
    3: LLAMA2_70B_LAYER,
    4: [("down", 8192, 28672)],
}


def seed_for(config: int, matrix_index: int, variant: int = 0) -> int:
    return 20240611 + 1000 * config + matrix_index + 100 * variant


def _rng(seed: int, stream: int, block: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 8) ^ stream, block]))


def row_keep_probabilities(rows: int, keep: float, seed: int, row_skew: bool) -> np.ndarray:
    """Per-row keep probability.  Beta(2,2) is the median of three U(0,1)."""
    if not row_skew:
        return np.full(rows, keep, dtype=np.float32)
    u = _rng(seed, 3, 0).random((rows, 3), dtype=np.float32)
    return np.median(u, axis=1).astype(np.float32)


def _fill_block(out: np.ndarray, r0: int, r1: int, cols: int, p_rows: np.ndarray, seed: int, block: int):
    n = (r1 - r0) * cols
    g_val = _rng(seed, 1, block)
    g_mask = _rng(seed, 2, block)
    x = (g_val.standard_normal(n, dtype=np.float32) * np.float32(SIGMA)).astype(np.float16)
    bits = x.view(np.uint16)
    while True:
        bad = np.flatnonzero((bits & 0x7FFF) == 0)
        if bad.size == 0:
            break
        redo = (g_val.standard_normal(bad.size, dtype=np.float32) * np.float32(SIGMA)).astype(np.float16)
        bits[bad] = redo.view(np.uint16)
    u = g_mask.random(n, dtype=np.float32).reshape(r1 - r0, cols)
    drop = u >= p_rows[r0:r1, None]
    blk = bits.reshape(r1 - r0, cols)
    blk[drop] = 0
    out[r0:r1] = blk


def pruned_fp16(rows: int, cols: int, keep: float = 0.5, seed: int = 0,
                row_skew: bool = False, threads: int | None = None) -> np.ndarray:
    """rows x cols matrix of fp16 BIT PATTERNS (uint16); view as float16 if wanted."""
    out = np.empty((rows, cols), dtype=np.uint16)
    if rows == 0 or cols == 0:
        return out
    p_rows = row_keep_probabilities(rows, keep, seed, row_skew)
    rows_per_block = max(1, _BLOCK_ELEMS // cols)
    blocks = [(b, r0, min(rows, r0 + rows_per_block))
              for b, r0 in enumerate(range(0, rows, rows_per_block))]
    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    if threads <= 1 or len(blocks) == 1:
        for b, r0, r1 in blocks:
            _fill_block(out, r0, r1, cols, p_rows, seed, b)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(lambda a: _fill_block(out, a[1], a[2], cols, p_rows, seed, a[0]), blocks))
    return out


def pruned_int8(rows: int, cols: int, keep: float = 0.5, seed: int = 0) -> np.ndarray:
    """rows x cols matrix of 8-bit patterns (uint8 view of int8 codes in
    [-127,127] without 0), for the 8-bit variant of Section 4.2."""
    g = _rng(seed, 4, 0)
    mag = g.integers(1, 128, size=(rows, cols), dtype=np.int16)
    sign = g.integers(0, 2, size=(rows, cols), dtype=np.int16) * 2 - 1
    q = (mag * sign).astype(np.int8).view(np.uint8)
    drop = g.random((rows, cols), dtype=np.float32) >= np.float32(keep)
    q[drop] = 0
    return q
