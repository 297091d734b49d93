"""MAC accounting and the improvement factor (Sec. 3.2 and Eq. 3).

Counting rule read from the paper: every linear of every decoder block is
pruned at one uniform sparsity, the embedding and the LM head stay dense
(Sec. 3), and the LM head's MACs are counted with the drafter's (Sec. 3.2).
Attention-score MACs and the embedding lookup are not counted.
"""

from fractions import Fraction


def decoder_linear_macs(layers, hidden, q_out, kv_out, inter) -> int:
    """Dense MACs per token in the decoder linears (q, k, v, o, gate, up, down)."""
    per_layer = hidden * q_out + 2 * hidden * kv_out + q_out * hidden + 3 * hidden * inter
    return layers * per_layer


def lm_head_macs(hidden, vocab) -> int:
    return hidden * vocab


def drafter_macs(layers, hidden, q_out, kv_out, inter, vocab, sparsity_pct=0) -> Fraction:
    """MACs per token of a drafter pruned to ``sparsity_pct`` in its decoder linears."""
    dense = decoder_linear_macs(layers, hidden, q_out, kv_out, inter)
    kept = Fraction(dense * (100 - sparsity_pct), 100)
    return kept + lm_head_macs(hidden, vocab)


def mac_reduction(layers, hidden, q_out, kv_out, inter, vocab, sparsity_pct) -> Fraction:
    """1 - MACs(sparse) / MACs(dense), as an exact fraction."""
    d = drafter_macs(layers, hidden, q_out, kv_out, inter, vocab, 0)
    s = drafter_macs(layers, hidden, q_out, kv_out, inter, vocab, sparsity_pct)
    return 1 - s / d


def improvement_factor(mal: float, k: int, c: float) -> float:
    """Eq. 3: expected speed-up of draft-then-verify over plain target decoding."""
    return mal / (k * c + 1.0)
