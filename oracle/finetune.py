"""Oracle for the masked-gradient step of sparse fine-tuning (TEST INFRASTRUCTURE ONLY).

Sec. 2.4 (and the sparse fine-tuning algorithm it refers to): the binary mask is fixed, pruned parameters start at
zero and their gradients are set to zero during back-propagation, so that they neither move nor enter the optimizer
state.  With M the non-zero pattern of the pruned bf16 weight matrix:

    g <- g where M, +0 elsewhere            (a selection, not a product: a NaN or Inf at a pruned position vanishes)
"""

import numpy as np

from .linear import nonzero_mask


def mask_gradient(w_bits: np.ndarray, grad: np.ndarray) -> np.ndarray:
    m = nonzero_mask(w_bits)
    if grad.shape != m.shape:
        raise ValueError("gradient and weight shapes differ")
    return np.where(m, grad, np.zeros((), dtype=grad.dtype))


def sgd_step(w: np.ndarray, w_bits: np.ndarray, grad: np.ndarray, lr: float) -> np.ndarray:
    """One plain SGD step on fp64 weights with the masked gradient (used by the pins only)."""
    return w - lr * mask_gradient(w_bits, grad.astype(np.float64))
