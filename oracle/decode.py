"""Oracle for a decode step of the drafter with rotary position embedding and a key/value cache.

TEST INFRASTRUCTURE: only tests, the smoke check and the bench's CPU baseline may import this.

The drafter produces its k candidates one token at a time, each conditioned on the prompt and on
the candidates before it (Sec. 2, the sentence that defines p_{n+j+1}); for a Llama / Qwen decoder
(Sec. 3) that means rotary position embedding on queries and keys and attention over the keys and
values of every earlier position, which a serving stack keeps in a cache.  The paper gives no
formula for either, so the public definition of those models is followed (a reading, listed with
the others in the design notes):

  * rotary embedding, half-split pairing: within a head of D dimensions, dimension i < D/2 is paired
    with i + D/2; at position p the pair is rotated by the angle p * theta^(-2 i / D);
  * queries and keys are rotated, values are not; the rotated key and the value of a position are
    rounded to bf16 and stored in the cache; attention reads every position, old or new, from the
    cache, so a token sees exactly what later calls will see;
  * token t of a call sits at position pos0 + t and attends to positions 0 .. pos0 + t.

Everything else (norms, linears, roundings to bf16 before each linear, residuals) is the block of
oracle/stack.py.  All arithmetic is float64.
"""

import numpy as np

from .bf16 import bits_to_f64, f64_to_bits, round_to_bf16
from .linear import sparse_linear_f64x
from .stack import rmsnorm, silu


def rope(x: np.ndarray, positions, head_dim: int, theta: float) -> np.ndarray:
    """Rotate every head of x [tokens][heads * head_dim]; token t sits at positions[t]."""
    tokens, width = x.shape
    half = head_dim // 2
    out = np.empty_like(x, dtype=np.float64)
    freq = np.array([theta ** (-2.0 * i / head_dim) for i in range(half)], dtype=np.float64)
    for t in range(tokens):
        ang = float(positions[t]) * freq
        c, s = np.cos(ang), np.sin(ang)
        for h0 in range(0, width, head_dim):
            lo = x[t, h0:h0 + half]
            hi = x[t, h0 + half:h0 + head_dim]
            out[t, h0:h0 + half] = lo * c - hi * s
            out[t, h0 + half:h0 + head_dim] = hi * c + lo * s
    return out


def cached_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, pos0: int, n_heads: int, n_kv: int,
                     head_dim: int) -> np.ndarray:
    """Softmax attention of q [tokens][n_heads * head_dim] over cache positions 0 .. pos0 + t.

    k_cache, v_cache: float64 [n_kv][positions][head_dim] (the values the cache holds).
    """
    tokens = q.shape[0]
    rep = n_heads // n_kv
    scale = 1.0 / np.sqrt(float(head_dim))
    ctx = np.zeros((tokens, n_heads * head_dim), dtype=np.float64)
    for h in range(n_heads):
        g = h // rep
        for t in range(tokens):
            n = pos0 + t + 1
            s = (k_cache[g, :n] @ q[t, h * head_dim:(h + 1) * head_dim]) * scale
            p = np.exp(s - s.max())
            p /= p.sum()
            ctx[t, h * head_dim:(h + 1) * head_dim] = p @ v_cache[g, :n]
    return ctx


def drafter_decode(shape, weight_bits, h_in_bits, k_cache_bits, v_cache_bits, pos0: int, theta: float, n_layers=None):
    """One call of the decode path: h_out [tokens][hidden] float64; the caches are updated in place.

    ``k_cache_bits``, ``v_cache_bits`` -- uint16 [layers][n_kv][max_pos][head_dim]; positions below pos0 hold
    the history, positions pos0 .. pos0 + tokens - 1 are written.
    """
    h = bits_to_f64(h_in_bits)
    tokens = h.shape[0]
    layers = shape.layers if n_layers is None else n_layers
    D = shape.head_dim
    positions = [pos0 + t for t in range(tokens)]
    assert pos0 >= 0 and pos0 + tokens <= k_cache_bits.shape[2]
    for l in range(layers):
        a = round_to_bf16(rmsnorm(h))
        q = rope(sparse_linear_f64x(weight_bits(l, "q"), a), positions, D, theta)
        kk = rope(sparse_linear_f64x(weight_bits(l, "k"), a), positions, D, theta)
        v = sparse_linear_f64x(weight_bits(l, "v"), a)
        for g in range(shape.n_kv):
            k_cache_bits[l, g, pos0:pos0 + tokens] = f64_to_bits(round_to_bf16(kk[:, g * D:(g + 1) * D]))
            v_cache_bits[l, g, pos0:pos0 + tokens] = f64_to_bits(round_to_bf16(v[:, g * D:(g + 1) * D]))
        n = pos0 + tokens
        ctx = round_to_bf16(cached_attention(q, bits_to_f64(k_cache_bits[l, :, :n]), bits_to_f64(v_cache_bits[l, :, :n]),
                                             pos0, shape.n_heads, shape.n_kv, D))
        h = h + sparse_linear_f64x(weight_bits(l, "o"), ctx)
        a2 = round_to_bf16(rmsnorm(h))
        g_ = sparse_linear_f64x(weight_bits(l, "gate"), a2)
        u = sparse_linear_f64x(weight_bits(l, "up"), a2)
        m = round_to_bf16(silu(g_) * u)
        h = h + sparse_linear_f64x(weight_bits(l, "down"), m)
    return h
