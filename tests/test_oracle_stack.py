import math
from types import SimpleNamespace

import numpy as np
import pytest

import sd2_workload as wl
from oracle import stack as os_
from oracle.bf16 import bits_to_f64, round_to_bf16, f64_to_bits

SHAPE = SimpleNamespace(layers=2, hidden=256, q_out=256, kv_out=128, inter=512, n_heads=2, n_kv=1, head_dim=128)


def _weights(shape, cfg=11, pct=50):
    table = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(shape)}
    cache = {}

    def get(layer, proj):
        if (layer, proj) not in cache:
            n, k = table[proj]
            cache[(layer, proj)] = wl.gen_weight(cfg, layer, proj, n, k, pct)
        return cache[(layer, proj)]
    return get


def test_round_to_bf16_matches_bit_trick_on_float32_inputs():
    rng = np.random.default_rng(3)
    x = rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-20, 20, 20000).astype(np.float32)
    a = f64_to_bits(x.astype(np.float64))
    b = wl.f32_to_bf16_bits(x)
    assert np.array_equal(a, b)


def test_round_to_bf16_ties_and_subnormals():
    one = 1.0
    assert round_to_bf16(np.array([one + 2.0 ** -8]))[0] == 1.0            # tie -> even
    assert round_to_bf16(np.array([one + 3 * 2.0 ** -8]))[0] == one + 2.0 ** -6  # tie -> even (up)
    assert round_to_bf16(np.array([one + 2.0 ** -8 + 2.0 ** -30]))[0] == one + 2.0 ** -7
    tiny = 2.0 ** -133
    assert round_to_bf16(np.array([0.5 * tiny]))[0] == 0.0                # tie -> even (zero)
    assert round_to_bf16(np.array([1.5 * tiny]))[0] == 2 * tiny
    assert round_to_bf16(np.array([2.4 * tiny]))[0] == 2 * tiny


def test_rmsnorm_and_silu_closed_forms():
    h = np.full((2, 64), 3.0)
    assert np.allclose(os_.rmsnorm(h), 3.0 / math.sqrt(9.0 + 1e-5), rtol=1e-15)
    x = np.linspace(-6, 6, 25)
    assert np.allclose(os_.silu(x), x * (1 + np.tanh(x / 2)) / 2, rtol=1e-13, atol=1e-15)
    assert os_.silu(np.array([0.0]))[0] == 0.0


def test_attention_zero_queries_average_values():
    rng = np.random.default_rng(4)
    k_tok, nh, nkv, hd = 4, 4, 2, 128
    v = rng.standard_normal((k_tok, nkv * hd))
    kk = rng.standard_normal((k_tok, nkv * hd))
    ctx = os_.inflight_attention(np.zeros((k_tok, nh * hd)), kk, v, nh, nkv, hd)
    for i in range(k_tok):
        for h in range(nh):
            g = h // 2
            assert np.allclose(ctx[i, h * hd:(h + 1) * hd], v[: i + 1, g * hd:(g + 1) * hd].mean(0), rtol=1e-13)


def test_attention_is_causal_and_sharp():
    """A huge score on an allowed key selects it; a huge score on a future key is ignored."""
    k_tok, hd = 3, 128
    q = np.zeros((k_tok, hd)); kk = np.zeros((k_tok, hd)); v = np.arange(k_tok * hd, dtype=float).reshape(k_tok, hd)
    q[:, 0] = 1000.0
    kk[2, 0] = 1000.0   # only token 2 may see key 2
    ctx = os_.inflight_attention(q, kk, v, 1, 1, hd)
    assert np.allclose(ctx[0], v[0])
    assert np.allclose(ctx[1], v[:2].mean(0))
    assert np.allclose(ctx[2], v[2])


def test_single_token_attention_copies_v():
    get = _weights(SHAPE)
    h_in = wl.gen_x(11, 0, "q", 1, SHAPE.hidden)
    trace = []
    os_.drafter_forward(SHAPE, get, h_in, n_layers=1, trace=trace)
    (_, _, a, qkv), (_, _, ctx, _o) = trace[0], trace[1]
    v = qkv[:, SHAPE.q_out + SHAPE.kv_out:]
    expect = round_to_bf16(np.concatenate([v, v], axis=1))  # two heads share the one KV head
    assert np.array_equal(ctx, expect)


def test_zero_layers_is_identity_and_zero_weights_keep_residual():
    h_in = wl.gen_x(11, 0, "q", 3, SHAPE.hidden)
    assert np.array_equal(os_.drafter_forward(SHAPE, None, h_in, n_layers=0), bits_to_f64(h_in))
    table = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(SHAPE)}
    zero = lambda l, p: np.zeros(table[p], dtype=np.uint16)
    assert np.array_equal(os_.drafter_forward(SHAPE, zero, h_in, n_layers=2), bits_to_f64(h_in))


def test_stack_step_by_step_recomputation():
    """One layer recomputed with explicit loops for the glue (independent of the vectorised code)."""
    get = _weights(SHAPE)
    h_in = wl.gen_x(11, 0, "q", 2, SHAPE.hidden)
    trace = []
    out = os_.drafter_forward(SHAPE, get, h_in, n_layers=1, trace=trace)
    h = bits_to_f64(h_in)
    # rmsnorm by loops
    a = np.zeros_like(h)
    for t in range(2):
        ms = sum(float(v) ** 2 for v in h[t]) / SHAPE.hidden
        a[t] = [float(v) / math.sqrt(ms + 1e-5) for v in h[t]]
    assert np.allclose(trace[0][2], round_to_bf16(a), rtol=0, atol=0) or np.mean(trace[0][2] != round_to_bf16(a)) < 1e-2
    # residual wiring: out = h + o + down
    assert np.allclose(out, h + trace[1][3] + trace[3][3], rtol=1e-15)
    # gated product wiring
    gu = trace[2][3]
    g, u = gu[:, :SHAPE.inter], gu[:, SHAPE.inter:]
    m = round_to_bf16(np.array([[float(gv) / (1 + math.exp(-float(gv))) * float(uv) for gv, uv in zip(gr, ur)] for gr, ur in zip(g, u)]))
    assert np.mean(trace[3][2] != m) < 1e-3  # identical up to rare last-bit differences of exp


def test_mlp_block_against_scalar_loops_and_a_swapped_gate():
    """The stand-alone MLP block down(bf16(silu(gate x) * (up x))), recomputed entry by entry with math.exp and
    Python sums on small integer-valued weights; swapping gate and up (a plausible slip: silu then lands on the
    wrong branch) must change the result."""
    rng = np.random.default_rng(17)
    k_in, inter, k_tok = 6, 5, 3
    def ints(shape, lo, hi, p_zero):
        a = rng.integers(lo, hi + 1, size=shape)
        a[rng.random(shape) < p_zero] = 0
        return a
    wg_i, wu_i, wd_i = ints((inter, k_in), -3, 3, 0.4), ints((inter, k_in), -3, 3, 0.4), ints((k_in, inter), -3, 3, 0.4)
    x_i = rng.integers(-2, 3, size=(k_tok, k_in))
    bits = lambda a: wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))
    y, m = os_.mlp_block(bits(wg_i), bits(wu_i), bits(wd_i), bits(x_i))
    assert y.shape == (k_tok, k_in) and m.shape == (k_tok, inter)
    for t in range(k_tok):
        m_row = []
        for j in range(inter):
            g = sum(int(wg_i[j, c]) * int(x_i[t, c]) for c in range(k_in))
            u = sum(int(wu_i[j, c]) * int(x_i[t, c]) for c in range(k_in))
            val = g / (1.0 + math.exp(-g)) * u
            m_row.append(float(bits_to_f64(wl.f32_to_bf16_bits(np.array([val], dtype=np.float32)))[0]))   # the workload's own rounding routine
            assert m[t, j] == pytest.approx(m_row[-1], rel=0, abs=abs(m_row[-1]) * 2.0 ** -8)  # same value or its bf16 neighbour
        for n in range(k_in):
            want = sum(int(wd_i[n, j]) * m[t, j] for j in range(inter))
            assert y[t, n] == pytest.approx(want, rel=1e-12, abs=1e-12)
    y_swapped, _ = os_.mlp_block(bits(wu_i), bits(wg_i), bits(wd_i), bits(x_i))
    assert np.abs(y_swapped - y).max() > 1e-3
    # a down projection applied to the unrounded product differs as well (the rounding point is part of the definition)
    x = bits_to_f64(bits(x_i))
    g = x @ wg_i.T.astype(np.float64)
    u = x @ wu_i.T.astype(np.float64)
    unrounded = (g / (1.0 + np.exp(-g)) * u) @ wd_i.T.astype(np.float64)
    assert np.abs(unrounded - y).max() > 0
    assert np.abs(unrounded - y).max() <= np.abs(wd_i).sum(axis=1).max() * np.abs(m).max() * 2.0 ** -8
