"""Pins for the LM-head oracle: closed forms, brute force, tie rule (no GPU)."""
import numpy as np

import sd2_workload as wl
from oracle import lm_head as olm
from oracle.bf16 import bits_to_f64, f64_to_bits
from oracle.stack import rmsnorm


def _bits(x):
    return f64_to_bits(np.asarray(x, dtype=np.float64))


def test_one_hot_rows_pick_the_matching_coordinate():
    # W = identity (bf16-exact): logits are the normalised activations themselves, argmax = largest coordinate
    hidden = 16
    w = _bits(np.eye(hidden))
    h = np.zeros((3, hidden))
    h[0, 5] = 2.0; h[0, 9] = -7.0
    h[1, :] = -1.0; h[1, 11] = -0.5
    h[2, 0] = 1.0; h[2, 1] = 3.0
    ids, logits = olm.lm_head_argmax(w, h)
    assert ids.tolist() == [5, 11, 1]
    # the logits are the bf16-rounded RMS-normalised inputs
    from oracle.bf16 import round_to_bf16
    assert np.array_equal(logits, round_to_bf16(rmsnorm(h)))


def test_ties_go_to_the_lowest_index():
    hidden = 8
    row = np.array([0.5, -1, 2, 0, 0, 1, 0, 0.25])
    w = _bits(np.stack([row * 0.5, row, row, row * 0.25, row]))      # rows 1, 2 and 4 are identical and largest
    h = np.tile(row, (2, 1))
    ids, logits = olm.lm_head_argmax(w, h)
    assert logits[0, 1] == logits[0, 2] == logits[0, 4] and logits[0, 1] > logits[0, 0]
    assert ids.tolist() == [1, 1]
    assert olm.first_argmax(np.array([[1.0, 3.0, 3.0], [2.0, 2.0, 2.0], [0.0, -1.0, 0.0]])).tolist() == [1, 0, 0]


def test_triple_loop_brute_force_on_a_tiny_case():
    rng = np.random.default_rng(7)
    vocab, hidden, k = 11, 6, 3
    w_bits = wl.f32_to_bf16_bits(rng.standard_normal((vocab, hidden)).astype(np.float32))
    h = rng.standard_normal((k, hidden))
    a = bits_to_f64(_bits(rmsnorm(h)))            # round to bf16 by the bit-level converter, back to float64
    want = np.zeros((k, vocab))
    for t in range(k):
        for v in range(vocab):
            for c in range(hidden):
                want[t, v] += a[t, c] * float(bits_to_f64(w_bits[v:v + 1, c:c + 1])[0, 0])
    ids, logits = olm.lm_head_argmax(w_bits, h)
    assert np.allclose(logits, want, rtol=1e-14, atol=1e-14)
    assert ids.tolist() == [int(np.argmax(want[t])) for t in range(k)]


def test_scale_of_the_residual_does_not_matter_and_chunking_is_invisible():
    rng = np.random.default_rng(11)
    w_bits = wl.f32_to_bf16_bits((0.02 * rng.standard_normal((300, 64))).astype(np.float32))
    h = rng.standard_normal((4, 64))
    ids, logits = olm.lm_head_argmax(w_bits, h)
    ids4, _ = olm.lm_head_argmax(w_bits, 4.0 * h)   # a power of two: rmsnorm(4h) differs from rmsnorm(h) only through eps
    assert ids.tolist() == ids4.tolist()
    small = olm.lm_head_logits(w_bits, h, chunk=7)
    assert np.array_equal(small, logits)
    # negating the activations negates the logits: the greedy token becomes the smallest logit's index
    _, neg = olm.lm_head_argmax(w_bits, -h)
    assert np.array_equal(neg, -logits)
