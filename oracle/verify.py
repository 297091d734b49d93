"""Oracle for greedy (strict top-1) verification, Eq. 2 of Sec. 2.1.

A draft token is kept iff it equals the target model's arg-max at that
position; the first disagreement ends the round and the target's own token is
emitted there.  Each round therefore emits the accepted drafts plus exactly one
target token (footnote to Eq. 3), so 1 <= emitted <= k + 1.

Readings taken where the text is loose: Eq. 2 is printed position by position,
but tokens after a mismatch were conditioned on a rejected prefix, so the
accepted run is the longest matching *prefix*; the target supplies k + 1
arg-maxes, entry i being its choice after the prompt plus draft[0:i].
"""

import numpy as np


def greedy_verify(draft, target, vocab=None):
    """draft [B][k], target [B][k+1] -> (accepted_len [B], out_tokens [B][k+1], tail -1)."""
    draft = np.asarray(draft)
    target = np.asarray(target)
    if draft.ndim != 2 or target.ndim != 2 or target.shape != (draft.shape[0], draft.shape[1] + 1):
        raise ValueError("need draft [B][k] and target [B][k+1]")
    if vocab is not None:
        for a in (draft, target):
            if a.size and (a.min() < 0 or a.max() >= vocab):
                raise ValueError("token id outside [0, vocab)")
    b_sz, k = draft.shape
    acc = np.zeros(b_sz, dtype=np.int32)
    out = np.full((b_sz, k + 1), -1, dtype=np.int32)
    for b in range(b_sz):
        n = 0
        while n < k and int(draft[b, n]) == int(target[b, n]):
            out[b, n] = draft[b, n]
            n += 1
        out[b, n] = target[b, n]
        acc[b] = n
    return acc, out


def expected_emitted(alpha: float, k: int) -> float:
    """Mean tokens per round when each position matches independently with prob. alpha."""
    if alpha == 1.0:
        return float(k + 1)
    return (1.0 - alpha ** (k + 1)) / (1.0 - alpha)
