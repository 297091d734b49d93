"""Oracle for the drafter's dense LM head with a greedy choice (TEST INFRASTRUCTURE ONLY).

Eq. 1 (Sec. 2.1): a draft token is drawn from the drafter's distribution given the prefix; greedy drafting takes
the most likely token, i.e. the largest logit.  The LM head is the one linear of the drafter that is never pruned
(Sec. 2.3 prunes the decoder blocks only; Sec. 3.2 counts the head's MACs as dense).  With the stack's glue:

    a        = bf16(rmsnorm(h))              h: final residual [k][hidden]; eps 1e-5, no learned scale
    logits   = a W^T                         W: [vocab][hidden] bf16, dense; float64 here
    token[t] = the lowest index among the largest logits of row t

Everything is float64 except the one rounding to bf16 where the HIP path hands activations to the linear.
"""

import numpy as np

from .bf16 import bits_to_f64, round_to_bf16
from .stack import rmsnorm


def lm_head_logits(w_bits: np.ndarray, h: np.ndarray, chunk: int = 8192) -> np.ndarray:
    """[k][vocab] float64 logits; the weight matrix is converted chunk by chunk (it can be 128k x 3k)."""
    a = round_to_bf16(rmsnorm(np.asarray(h, dtype=np.float64)))
    vocab = w_bits.shape[0]
    out = np.empty((a.shape[0], vocab), dtype=np.float64)
    for r0 in range(0, vocab, chunk):
        r1 = min(vocab, r0 + chunk)
        out[:, r0:r1] = a @ bits_to_f64(w_bits[r0:r1]).T
    return out


def first_argmax(logits: np.ndarray) -> np.ndarray:
    """Lowest index of the maximum of each row (numpy.argmax has exactly this tie rule)."""
    return np.argmax(logits, axis=-1).astype(np.int32)


def lm_head_argmax(w_bits: np.ndarray, h: np.ndarray):
    """-> (token ids int32 [k], logits float64 [k][vocab])"""
    logits = lm_head_logits(w_bits, h)
    return first_argmax(logits), logits
