"""Oracle for one-shot magnitude pruning at a uniform per-layer sparsity (TEST INFRASTRUCTURE ONLY).

Sec. 2.3: every decoder linear is pruned one-shot to the same sparsity; the paper uses a second-order criterion on
calibration data, which needs a model and data.  The criterion implemented here is weight magnitude (the stand-in this
build uses for its synthetic weights), in the two patterns the paper evaluates:

  rows : per output row keep the n_keep = K - (p K) div 100 entries of largest |w|;
  2:4  : in every aligned group of four columns keep the two entries of largest |w|.

Ties go to the lower column.  Pruned entries become +0; kept entries keep their bits.  Written as a literal sort per
row / per group, with nothing shared with the input generator's mask code.
"""

import numpy as np


def _magnitude(w_bits: np.ndarray) -> np.ndarray:
    return (np.asarray(w_bits, dtype=np.uint16) & np.uint16(0x7FFF)).astype(np.int64)  # bf16 magnitudes order like their bits


def prune_rows(w_bits: np.ndarray, sparsity_pct: int) -> np.ndarray:
    w = np.asarray(w_bits, dtype=np.uint16)
    n, k = w.shape
    n_keep = k - (sparsity_pct * k) // 100
    out = np.zeros_like(w)
    mag = _magnitude(w)
    for r in range(n):
        order = sorted(range(k), key=lambda c: (-int(mag[r, c]), c))  # largest first, lower column first among equals
        for c in order[:n_keep]:
            out[r, c] = w[r, c]
    return out


def prune_2of4(w_bits: np.ndarray) -> np.ndarray:
    w = np.asarray(w_bits, dtype=np.uint16)
    n, k = w.shape
    if k % 4:
        raise ValueError("k_in must be a multiple of 4")
    out = np.zeros_like(w)
    mag = _magnitude(w)
    for r in range(n):
        for g0 in range(0, k, 4):
            order = sorted(range(g0, g0 + 4), key=lambda c: (-int(mag[r, c]), c))
            for c in order[:2]:
                out[r, c] = w[r, c]
    return out
