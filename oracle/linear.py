"""Oracle for one pruned linear layer at decode shape.

The draft model's linears keep a fixed binary mask; pruned parameters are
exactly zero (Sec. 2.4).  The sparse product is therefore, by definition, the
dense product of the masked matrix:

    Y[t, n] = sum_c (W[n, c] * M[n, c]) * X[t, c]

computed here in float64 from the exact values of the bf16 inputs.
"""

import numpy as np

from .bf16 import bits_to_f64


def nonzero_mask(w_bits: np.ndarray) -> np.ndarray:
    """M: True where the bf16 weight is not +-0 (the pattern IS the nonzero pattern)."""
    return (np.asarray(w_bits, dtype=np.uint16) & np.uint16(0x7FFF)) != 0


def masked_dense_f64(w_bits: np.ndarray, mask: np.ndarray = None) -> np.ndarray:
    """W * M as float64.  ``mask`` defaults to the nonzero pattern of W."""
    w = bits_to_f64(w_bits)
    m = nonzero_mask(w_bits) if mask is None else np.asarray(mask, dtype=bool)
    return w * m


def sparse_linear(w_bits: np.ndarray, x_bits: np.ndarray, mask: np.ndarray = None) -> np.ndarray:
    """Y [k_tok][n_out] float64 for bf16 W [n_out][k_in] and bf16 X [k_tok][k_in]."""
    wm = masked_dense_f64(w_bits, mask)
    x = bits_to_f64(x_bits)
    return x @ wm.T


def sparse_linear_f64x(w_bits: np.ndarray, x: np.ndarray, mask: np.ndarray = None) -> np.ndarray:
    """Same product with activations already given as float64 [k_tok][k_in]."""
    return np.asarray(x, dtype=np.float64) @ masked_dense_f64(w_bits, mask).T


def sparse_linear_rowloop(w_bits: np.ndarray, x_bits: np.ndarray, mask: np.ndarray = None) -> np.ndarray:
    """Second code path: explicit loop over rows, summing kept columns only."""
    w = bits_to_f64(w_bits)
    x = bits_to_f64(x_bits)
    m = nonzero_mask(w_bits) if mask is None else np.asarray(mask, dtype=bool)
    n_out = w.shape[0]
    y = np.zeros((x.shape[0], n_out), dtype=np.float64)
    for n in range(n_out):
        cols = np.flatnonzero(m[n])
        if cols.size:
            y[:, n] = x[:, cols] @ w[n, cols]
    return y


def rel_l2(y, y_ref) -> float:
    """|| y - y_ref ||_2 / || y_ref ||_2 over the whole tensor (0/0 -> 0)."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    den = float(np.linalg.norm(y_ref.ravel()))
    num = float(np.linalg.norm((y - y_ref).ravel()))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den
