"""Oracle for the drafter's linear stack with its minimal glue.

The paper's drafter is an ordinary Llama/Qwen decoder whose seven linears per
block are pruned (Sec. 3); this build covers the linears, so the operations
between them are a fixed synthetic stand-in that keeps the true data
dependencies of a block (q, k, v share one input; o follows attention; gate and
up share one input; down follows the gated product) and keeps activations O(1):

    h <- h_in                                        [k][hidden]
    per layer:
      a      = bf16(rmsnorm(h))                      eps 1e-5, no learned scale
      q,kk,v = a Wq^T, a Wk^T, a Wv^T
      ctx    = causal softmax attention among the k in-flight tokens only
               (head_dim 128, scale 1/sqrt(128), grouped KV heads, no rotary
               embedding, no cache)
      h      = h + bf16(ctx) Wo^T
      a2     = bf16(rmsnorm(h))
      m      = bf16(silu(a2 Wg^T) * (a2 Wu^T))
      h      = h + m Wd^T
    h_out = h

Everything is float64 except the four explicit roundings to bf16, which sit
exactly where the HIP path hands a bf16 activation to a linear.
"""

import numpy as np

from .bf16 import bits_to_f64, round_to_bf16
from .linear import sparse_linear_f64x

EPS = 1e-5


def rmsnorm(h: np.ndarray) -> np.ndarray:
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h / np.sqrt(ms + EPS)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def inflight_attention(q, kk, v, n_heads, n_kv, head_dim):
    """Causal softmax attention over the k tokens of this call only."""
    k_tok = q.shape[0]
    rep = n_heads // n_kv
    ctx = np.zeros((k_tok, n_heads * head_dim), dtype=np.float64)
    scale = 1.0 / np.sqrt(float(head_dim))
    for h in range(n_heads):
        g = h // rep
        qh = q[:, h * head_dim:(h + 1) * head_dim]
        kg = kk[:, g * head_dim:(g + 1) * head_dim]
        vg = v[:, g * head_dim:(g + 1) * head_dim]
        s = (qh @ kg.T) * scale
        for i in range(k_tok):
            row = s[i, : i + 1]
            p = np.exp(row - row.max())
            p /= p.sum()
            ctx[i, h * head_dim:(h + 1) * head_dim] = p @ vg[: i + 1]
    return ctx


def drafter_forward(shape, weight_bits, h_in_bits, n_layers=None, trace=None):
    """h_out [k][hidden] float64.

    ``shape``       -- object with hidden, q_out, kv_out, inter, n_heads, n_kv, head_dim, layers
    ``weight_bits`` -- callable (layer, projection) -> bf16 bit matrix [n_out][k_in]
    ``trace``       -- optional list; receives (layer, name, input_f64, output_f64) per linear group
    """
    h = bits_to_f64(h_in_bits)
    layers = shape.layers if n_layers is None else n_layers
    for l in range(layers):
        a = round_to_bf16(rmsnorm(h))
        q = sparse_linear_f64x(weight_bits(l, "q"), a)
        kk = sparse_linear_f64x(weight_bits(l, "k"), a)
        v = sparse_linear_f64x(weight_bits(l, "v"), a)
        ctx = round_to_bf16(inflight_attention(q, kk, v, shape.n_heads, shape.n_kv, shape.head_dim))
        o = sparse_linear_f64x(weight_bits(l, "o"), ctx)
        h = h + o
        a2 = round_to_bf16(rmsnorm(h))
        g = sparse_linear_f64x(weight_bits(l, "gate"), a2)
        u = sparse_linear_f64x(weight_bits(l, "up"), a2)
        m = round_to_bf16(silu(g) * u)
        d = sparse_linear_f64x(weight_bits(l, "down"), m)
        h = h + d
        if trace is not None:
            trace.append((l, "qkv", a, np.concatenate([q, kk, v], axis=1)))
            trace.append((l, "o", ctx, o))
            trace.append((l, "gateup", a2, np.concatenate([g, u], axis=1)))
            trace.append((l, "down", m, d))
    return h


def mlp_block(w_gate_bits, w_up_bits, w_down_bits, x_bits):
    """down(bf16(silu(gate x) * up x)) for the stand-alone MLP-block configuration."""
    x = bits_to_f64(x_bits)
    g = sparse_linear_f64x(w_gate_bits, x)
    u = sparse_linear_f64x(w_up_bits, x)
    m = round_to_bf16(silu(g) * u)
    return sparse_linear_f64x(w_down_bits, m), m
