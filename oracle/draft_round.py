"""Oracle for one drafting round of the sparse drafter (TEST INFRASTRUCTURE ONLY).

Sec. 2.1: per round the draft model proposes k tokens autoregressively (Eq. 1), each from the prefix extended by the
tokens it has proposed so far; greedy decoding takes the largest logit (lowest id on ties).  With this build's glue
(attention among the tokens of the call only, i.e. the round's window with an empty history) step i is:

    window  = [t_start, d_0, ..., d_{i-1}]            i + 1 tokens
    h_in    = E[window]                                rows of the embedding matrix (bf16); the head is tied to it
    h_out   = drafter_forward(h_in)                    the decoder-linear stack
    d_i     = first_argmax( lm_head( h_out[last] ) )   final norm + dense head on the last position

Recomputing the window each step equals keeping its keys and values in a cache: the stack is causal.
"""

import numpy as np

from . import lm_head as olm
from . import stack as ostack


def draft_round(shape, weight_bits, emb_bits: np.ndarray, t_start: int, k: int, forced=None):
    """-> (draft ids [k] int32, last-position logits per step [k][vocab] float64).

    ``emb_bits``: [vocab][hidden] bf16 bits, embedding and (tied) LM head.  ``forced``: optional ids to feed instead
    of the oracle's own choices (teacher forcing: step i then sees forced[0..i))."""
    window = [int(t_start)]
    ids, logits_all = [], []
    for i in range(k):
        h_in = emb_bits[np.asarray(window, dtype=np.int64)]
        h_out = ostack.drafter_forward(shape, weight_bits, h_in)
        tok, logits = olm.lm_head_argmax(emb_bits, h_out[-1:])
        ids.append(int(tok[0]))
        logits_all.append(logits[0])
        window.append(int(forced[i]) if forced is not None else int(tok[0]))
    return np.asarray(ids, dtype=np.int32), np.stack(logits_all)


def draft_round_cached(shape, weight_bits, emb_bits: np.ndarray, t_start: int, k: int, k_cache_bits, v_cache_bits,
                       pos0: int, theta: float, forced=None):
    """The round against a key/value cache (rotary embedding, history of pos0 positions): k single-token decode steps.

    The start token sits at position pos0; step i embeds one token (t_start, then the token chosen -- or forced --
    at step i - 1), runs oracle/decode.py on it at position pos0 + i (which appends its key and value to the caches,
    updated in place) and gives the result to the final norm and the tied head.  -> (ids [k], logits [k][vocab])."""
    from . import decode as odec
    cur = int(t_start)
    ids, logits_all = [], []
    for i in range(k):
        h_out = odec.drafter_decode(shape, weight_bits, emb_bits[cur:cur + 1], k_cache_bits, v_cache_bits, pos0 + i, theta)
        tok, logits = olm.lm_head_argmax(emb_bits, h_out)
        ids.append(int(tok[0]))
        logits_all.append(logits[0])
        cur = int(forced[i]) if forced is not None else int(tok[0])
    return np.asarray(ids, dtype=np.int32), np.stack(logits_all)
