"""Pins for the decode-step oracle (rotary embedding, key/value cache): closed forms, invariants, brute force."""
import math
from types import SimpleNamespace

import numpy as np

import sd2_workload as wl
from oracle import decode as od
from oracle import stack as os_
from oracle.bf16 import bits_to_f64, f64_to_bits, round_to_bf16

SHAPE = SimpleNamespace(layers=2, hidden=256, q_out=256, kv_out=128, inter=512, n_heads=2, n_kv=1, head_dim=128)
THETA = 500000.0


def _weights(shape, cfg=13, pct=50):
    table = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(shape)}
    cache = {}

    def get(layer, proj):
        if (layer, proj) not in cache:
            n, k = table[proj]
            cache[(layer, proj)] = wl.gen_weight(cfg, layer, proj, n, k, pct)
        return cache[(layer, proj)]
    return get


def test_rope_is_a_complex_rotation_of_each_pair():
    # dimension i and i + D/2 form the complex number x_i + j x_{i+D/2}; position p multiplies it by exp(j p theta^(-2i/D))
    rng = np.random.default_rng(1)
    D, heads = 16, 3
    x = rng.standard_normal((4, heads * D))
    pos = [0, 1, 7, 1000]
    y = od.rope(x, pos, D, 10000.0)
    for t, p in enumerate(pos):
        for h in range(heads):
            z = x[t, h * D:h * D + D // 2] + 1j * x[t, h * D + D // 2:(h + 1) * D]
            w = z * np.exp(1j * p * 10000.0 ** (-2.0 * np.arange(D // 2) / D))
            assert np.allclose(y[t, h * D:h * D + D // 2], w.real, rtol=1e-12, atol=1e-12)
            assert np.allclose(y[t, h * D + D // 2:(h + 1) * D], w.imag, rtol=1e-12, atol=1e-12)
    assert np.array_equal(y[0], x[0])  # position 0: no rotation


def test_rope_known_angles():
    # D = 2: one pair, frequency 1; a quarter turn maps (1, 0) to (0, 1)
    y = od.rope(np.array([[1.0, 0.0]]), [math.pi / 2], 2, 10000.0)
    assert np.allclose(y, [[0.0, 1.0]], atol=1e-15)
    # D = 4, theta = 100: pair 1 turns at 100^(-1/2) = 0.1 rad per position
    y = od.rope(np.array([[0.0, 1.0, 0.0, 0.0]]), [5], 4, 100.0)
    assert np.allclose(y, [[0.0, math.cos(0.5), 0.0, math.sin(0.5)]], atol=1e-15)


def test_rope_keeps_norms_and_scores_depend_on_distance_only():
    rng = np.random.default_rng(2)
    D = 128
    q, k = rng.standard_normal((1, D)), rng.standard_normal((1, D))
    assert np.isclose(np.linalg.norm(od.rope(q, [77], D, THETA)), np.linalg.norm(q), rtol=1e-13)
    ref = od.rope(q, [9], D, THETA) @ od.rope(k, [4], D, THETA).T
    for shift in (1, 50, 3000):
        s = od.rope(q, [9 + shift], D, THETA) @ od.rope(k, [4 + shift], D, THETA).T
        assert np.allclose(s, ref, rtol=1e-9, atol=1e-9)
    # and it does depend on the distance
    assert not np.allclose(od.rope(q, [10], D, THETA) @ od.rope(k, [4], D, THETA).T, ref, rtol=1e-3)


def test_cached_attention_special_cases():
    rng = np.random.default_rng(3)
    n_heads, n_kv, D, P = 4, 2, 8, 12
    kc, vc = rng.standard_normal((n_kv, P, D)), rng.standard_normal((n_kv, P, D))
    # zero queries: plain average of the values of positions 0 .. pos0 + t
    ctx = od.cached_attention(np.zeros((3, n_heads * D)), kc, vc, 5, n_heads, n_kv, D)
    for t in range(3):
        for h in range(n_heads):
            assert np.allclose(ctx[t, h * D:(h + 1) * D], vc[h // 2, :5 + t + 1].mean(axis=0), rtol=1e-13)
    # a query that is a huge multiple of one key picks that position's value; a later position must not be seen
    q = np.zeros((1, n_heads * D))
    kc2 = np.zeros_like(kc)
    kc2[:, 3, 0] = 1.0
    kc2[:, 9, 0] = 2.0  # beyond pos0: invisible
    q[0, 0::D] = 500.0
    ctx = od.cached_attention(q, kc2, vc, 6, n_heads, n_kv, D)
    for h in range(n_heads):
        assert np.allclose(ctx[0, h * D:(h + 1) * D], vc[h // 2, 3], atol=1e-9)


def test_cached_attention_against_scalar_loops():
    rng = np.random.default_rng(4)
    n_heads, n_kv, D, pos0, T = 2, 1, 4, 3, 2
    kc, vc = rng.standard_normal((n_kv, 8, D)), rng.standard_normal((n_kv, 8, D))
    q = rng.standard_normal((T, n_heads * D))
    ctx = od.cached_attention(q, kc, vc, pos0, n_heads, n_kv, D)
    for t in range(T):
        for h in range(n_heads):
            scores = []
            for j in range(pos0 + t + 1):
                scores.append(sum(q[t, h * D + d] * kc[0, j, d] for d in range(D)) / math.sqrt(D))
            mx = max(scores)
            e = [math.exp(s - mx) for s in scores]
            for d in range(D):
                want = sum(e[j] * vc[0, j, d] for j in range(len(e))) / sum(e)
                assert math.isclose(ctx[t, h * D + d], want, rel_tol=1e-12, abs_tol=1e-14)


def _run(shape, h_bits, n_hist, pos0, chunks, max_pos=64, cfg=13):
    get = _weights(shape, cfg)
    kc, vc = wl.gen_kv_history(cfg, shape.layers, shape.n_kv, max_pos, shape.head_dim, n_hist)
    outs, p = [], pos0
    for c in chunks:
        outs.append(od.drafter_decode(shape, get, h_bits[p - pos0:p - pos0 + c], kc, vc, p, THETA))
        p += c
    return np.concatenate(outs), kc, vc


def test_decode_is_the_same_one_token_at_a_time():
    # the cache is what makes the k sequential single-token forwards of a drafting round equal to one pass over
    # the window: five tokens in one call, as 1+1+1+1+1 and as 2+3 give the same residuals and the same caches
    h_bits = wl.gen_x(13, 0, "q", 5, SHAPE.hidden)
    a, ka, va = _run(SHAPE, h_bits, 9, 9, [5])
    b, kb, vb = _run(SHAPE, h_bits, 9, 9, [1, 1, 1, 1, 1])
    c, kc, vc = _run(SHAPE, h_bits, 9, 9, [2, 3])
    assert np.allclose(a, b, rtol=1e-11, atol=1e-11) and np.allclose(a, c, rtol=1e-11, atol=1e-11)
    assert np.array_equal(ka, kb) and np.array_equal(va, vb) and np.array_equal(ka, kc) and np.array_equal(va, vc)
    # history beyond the written positions is untouched, positions 9..13 are written
    k0, v0 = wl.gen_kv_history(13, SHAPE.layers, SHAPE.n_kv, 64, SHAPE.head_dim, 9)
    assert np.array_equal(ka[:, :, :9], k0[:, :, :9]) and np.array_equal(ka[:, :, 14:], k0[:, :, 14:])
    assert np.all(ka[:, :, 9:14].astype(np.int64).sum(axis=-1) != 0)


def test_decode_without_history_at_position_zero_first_token_matches_the_window_forward():
    # one token at position 0: no rotation, attention over itself only -> ctx = bf16(bf16(v)); the window forward
    # (no rotary embedding, no cache) computes ctx = bf16(v): the same number
    h_bits = wl.gen_x(13, 0, "q", 1, SHAPE.hidden)
    a, _, _ = _run(SHAPE, h_bits, 0, 0, [1])
    b = os_.drafter_forward(SHAPE, _weights(SHAPE), h_bits)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-12)


def test_decode_sees_the_history():
    h_bits = wl.gen_x(13, 0, "q", 2, SHAPE.hidden)
    a, _, _ = _run(SHAPE, h_bits, 20, 20, [2])
    b, _, _ = _run(SHAPE, h_bits, 20, 20, [2], cfg=13)
    assert np.array_equal(a, b)  # deterministic
    get = _weights(SHAPE)
    kc, vc = wl.gen_kv_history(13, SHAPE.layers, SHAPE.n_kv, 64, SHAPE.head_dim, 20)
    vc[:, :, 5] = f64_to_bits(bits_to_f64(vc[:, :, 5]) + 4.0)  # change one old value row
    c = od.drafter_decode(SHAPE, get, h_bits, kc, vc, 20, THETA)
    assert not np.allclose(a, c, rtol=1e-6)
    kc, vc = wl.gen_kv_history(13, SHAPE.layers, SHAPE.n_kv, 64, SHAPE.head_dim, 20)
    vc[:, :, 40] = 0x4000  # a position no token of this call may see
    d = od.drafter_decode(SHAPE, get, h_bits, kc, vc, 20, THETA)
    assert np.array_equal(a, d)


def test_cache_holds_rounded_rotated_keys_and_plain_values():
    get = _weights(SHAPE)
    h_bits = wl.gen_x(13, 0, "q", 3, SHAPE.hidden)
    kc, vc = wl.gen_kv_history(13, SHAPE.layers, SHAPE.n_kv, 64, SHAPE.head_dim, 4)
    od.drafter_decode(SHAPE, get, h_bits, kc, vc, 4, THETA, n_layers=1)
    from oracle.linear import sparse_linear_f64x
    a = round_to_bf16(os_.rmsnorm(bits_to_f64(h_bits)))
    kk = sparse_linear_f64x(get(0, "k"), a)
    v = sparse_linear_f64x(get(0, "v"), a)
    assert np.array_equal(vc[0, 0, 4:7], f64_to_bits(v))
    assert np.array_equal(kc[0, 0, 4:7], f64_to_bits(od.rope(kk, [4, 5, 6], SHAPE.head_dim, THETA)))
