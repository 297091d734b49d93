"""Pins for the drafting-round oracle (Eq. 1, greedy)."""
from types import SimpleNamespace

import numpy as np

import sd2_workload as wl
from oracle import draft_round as odr
from oracle import lm_head as olm
from oracle import stack as ostack


def _setup(layers=1):
    shape = SimpleNamespace(layers=layers, hidden=256, q_out=256, kv_out=128, inter=512, n_heads=2, n_kv=1, head_dim=128)
    table = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(shape)}
    cache = {}

    def get(layer, proj):
        if (layer, proj) not in cache:
            cache[(layer, proj)] = wl.gen_weight(77, layer, proj, table[proj][0], table[proj][1], 50)
        return cache[(layer, proj)]

    emb = wl.gen_lm_head(77, 300, shape.hidden)
    return shape, get, emb


def test_zero_layers_is_a_lookup_and_an_argmax():
    """Without decoder layers step i is: embed the last token, normalise, multiply with the (tied) head."""
    shape, get, emb = _setup(layers=0)
    ids, logits = odr.draft_round(shape, get, emb, t_start=7, k=3)
    cur = 7
    for i in range(3):
        ref_id, ref_logits = olm.lm_head_argmax(emb, wl.bf16_bits_to_f32(emb[cur:cur + 1]).astype(np.float64))
        assert ids[i] == ref_id[0] and np.array_equal(logits[i], ref_logits[0])
        cur = int(ids[i])


def test_each_step_sees_the_window_so_far():
    """Step i equals a fresh forward over [t_start, d_0..d_{i-1}] -- and, the stack being causal, the rows of the
    earlier positions in that forward equal what the earlier steps computed (recompute = cache)."""
    shape, get, emb = _setup(layers=2)
    ids, logits = odr.draft_round(shape, get, emb, t_start=11, k=4)
    window = [11] + ids[:3].tolist()
    h_full = ostack.drafter_forward(shape, get, emb[np.asarray(window)])
    for i in range(4):
        h_i = ostack.drafter_forward(shape, get, emb[np.asarray(window[:i + 1])])
        assert np.array_equal(h_i, h_full[:i + 1])          # causality: a longer window does not change earlier rows
        tok, lg = olm.lm_head_argmax(emb, h_i[-1:])
        assert tok[0] == ids[i] and np.array_equal(lg[0], logits[i])


def test_teacher_forcing_feeds_the_given_ids():
    shape, get, emb = _setup(layers=1)
    free_ids, _ = odr.draft_round(shape, get, emb, t_start=3, k=3)
    forced = np.array([5, 9, 2], dtype=np.int32)
    ids, _ = odr.draft_round(shape, get, emb, t_start=3, k=3, forced=forced)
    assert ids[0] == free_ids[0]                             # the first step sees only t_start either way
    h = ostack.drafter_forward(shape, get, emb[np.array([3, 5, 9])])
    assert ids[2] == olm.lm_head_argmax(emb, h[-1:])[0][0]   # the third step saw the forced ids


def test_cached_round_equals_one_decode_call_over_the_window():
    """k single-token steps against the cache give, position by position, what one decode call over the whole window
    [t_start, d_0 .. d_{k-2}] gives (the cache makes the sequential forwards of a round equal one causal pass), and
    leave the same cache."""
    from oracle import decode as odec
    shape, get, emb = _setup(layers=2)
    theta, pos0, k = 500000.0, 6, 4
    kc, vc = wl.gen_kv_history(77, shape.layers, shape.n_kv, 32, shape.head_dim, pos0)
    ids, logits = odr.draft_round_cached(shape, get, emb, 11, k, kc, vc, pos0, theta)
    window = [11] + ids[:k - 1].tolist()
    kc2, vc2 = wl.gen_kv_history(77, shape.layers, shape.n_kv, 32, shape.head_dim, pos0)
    h = odec.drafter_decode(shape, get, emb[np.asarray(window)], kc2, vc2, pos0, theta)
    tok, lg = olm.lm_head_argmax(emb, h)
    assert np.array_equal(tok, ids) and np.allclose(lg, logits, rtol=1e-10, atol=1e-10)
    assert np.array_equal(kc, kc2) and np.array_equal(vc, vc2)


def test_cached_round_depends_on_the_history_and_forcing_feeds_the_given_ids():
    from oracle import decode as odec
    shape, get, emb = _setup(layers=1)
    theta, pos0 = 500000.0, 5
    kc, vc = wl.gen_kv_history(77, shape.layers, shape.n_kv, 16, shape.head_dim, pos0)
    _, lg_a = odr.draft_round_cached(shape, get, emb, 3, 2, kc, vc, pos0, theta)
    kc, vc = wl.gen_kv_history(78, shape.layers, shape.n_kv, 16, shape.head_dim, pos0)  # another history
    _, lg_b = odr.draft_round_cached(shape, get, emb, 3, 2, kc, vc, pos0, theta)
    assert not np.allclose(lg_a, lg_b, rtol=1e-6)
    kc, vc = wl.gen_kv_history(77, shape.layers, shape.n_kv, 16, shape.head_dim, pos0)
    forced = np.array([5, 9], dtype=np.int32)
    ids, _ = odr.draft_round_cached(shape, get, emb, 3, 3, kc, vc, pos0, theta, forced=np.array([5, 9, 0]))
    kc2, vc2 = wl.gen_kv_history(77, shape.layers, shape.n_kv, 16, shape.head_dim, pos0)
    h = odec.drafter_decode(shape, get, emb[np.array([3, 5, 9])], kc2, vc2, pos0, theta)
    assert ids[2] == olm.lm_head_argmax(emb, h[-1:])[0][0]
