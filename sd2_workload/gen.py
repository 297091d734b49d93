"""Seed-defined tensors for every benchmark configuration.

Recipe (all of it is a stand-in for pruned Llama-3.2 / Qwen-2.5 drafters, whose
weights are not available here):

* one ``numpy.random.default_rng([SEED, cfg_id, layer, proj_id])`` per tensor;
* weights  W = 0.02 * z,  activations X = z,  z ~ N(0, 1) drawn as float32,
  rounded to bf16 (round to nearest, ties to even) *before* pruning;
* pruning pattern: per output row keep the ``n_keep(K, p)`` largest |w|
  (ties: lowest column first); pruned entries become +0.  The paper prunes
  with a one-shot second-order method at uniform per-layer sparsity (Sec. 2.3);
  magnitude pruning per row has the same density and the same "fixed binary
  mask" structure (Sec. 2.4) and needs no calibration data;
* a second pattern, ``global`` (one magnitude threshold per matrix), gives rows
  of unequal population for load-balance tests;
* verification ids: target ids uniform over the vocabulary, each draft id equal
  to the target id with probability ``alpha`` and otherwise guaranteed different.

Arrays of bf16 are carried as ``numpy.uint16`` bit patterns.
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Iterator, List, Tuple

import numpy as np

SEED = 250408838

# projection ids used in the RNG key
PROJ: Dict[str, int] = {"q": 0, "k": 1, "v": 2, "o": 3, "gate": 4, "up": 5, "down": 6}
_X_BASE = 100
_VERIFY_BASE = 200


@dataclass(frozen=True)
class StackShape:
    """Shape of one drafter's decoder-linear stack."""

    name: str
    layers: int
    hidden: int
    q_out: int
    kv_out: int
    inter: int
    n_heads: int
    n_kv: int
    head_dim: int
    vocab: int


CONFIGS: Dict[int, dict] = {
    1: {"name": "single-512", "n_out": 512, "k_in": 512, "sparsity": 50, "k_tok": 1},
    2: {
        "name": "llama1b-mlp",
        "hidden": 2048,
        "inter": 8192,
        "sparsity": 50,
        "k_tok": 5,
    },
    3: {
        "name": "llama3b-stack",
        "shape": StackShape("llama-3b-shape", 28, 3072, 3072, 1024, 8192, 24, 8, 128, 128256),
        "sparsity": 50,
        "k_tok": 5,
    },
    4: {
        "name": "qwen1.5b-stack",
        "shape": StackShape("qwen-1.5b-shape", 28, 1536, 1536, 256, 8960, 12, 2, 128, 151936),
        "sparsity": (50, 60, 70),
        "k_tok": (1, 3, 5, 8),
    },
    5: {
        "name": "llama3b-wide",
        "shape": StackShape("llama-3b-shape", 28, 3072, 3072, 1024, 8192, 24, 8, 128, 128256),
        "sparsity": 50,
        "k_tok": (16, 32, 64),
        "verify": {"batch": 64, "k": 5, "vocab": 128256, "alpha": 0.85},
    },
}


# --------------------------------------------------------------------------- bf16


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern, round to nearest even (finite inputs)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- masks


def n_keep(k_in: int, sparsity_pct: int) -> int:
    """Kept weights per row: integer rule, no float multiply."""
    if not 0 <= sparsity_pct <= 100:
        raise ValueError("sparsity_pct must be in [0, 100]")
    return k_in - (sparsity_pct * k_in) // 100


def magnitude_mask_per_row(w_bits: np.ndarray, sparsity_pct: int) -> np.ndarray:
    """Boolean keep-mask: per row the n_keep largest |w|, ties to lowest column."""
    n, k = w_bits.shape
    keep = n_keep(k, sparsity_pct)
    if keep == k:
        return np.ones((n, k), dtype=bool)
    if keep == 0:
        return np.zeros((n, k), dtype=bool)
    mag = (w_bits & np.uint16(0x7FFF)).astype(np.uint16)
    kth = k - keep  # ascending index of the smallest kept magnitude
    thr = np.partition(mag, kth, axis=1)[:, kth][:, None]
    gt = mag > thr
    eq = mag == thr
    need = (keep - gt.sum(axis=1, dtype=np.int32))[:, None]
    rank = np.cumsum(eq, axis=1, dtype=np.int32)  # 1-based rank among ties, by column
    return gt | (eq & (rank <= need))


def magnitude_mask_global(w_bits: np.ndarray, sparsity_pct: int) -> np.ndarray:
    """One threshold for the whole matrix (rows end up with unequal population)."""
    n, k = w_bits.shape
    total = n * k
    keep = total - (sparsity_pct * total) // 100
    if keep == total:
        return np.ones((n, k), dtype=bool)
    if keep == 0:
        return np.zeros((n, k), dtype=bool)
    mag = (w_bits & np.uint16(0x7FFF)).astype(np.uint16).reshape(-1)
    kth = total - keep
    thr = np.partition(mag, kth)[kth]
    gt = mag > thr
    eq = mag == thr
    need = keep - int(gt.sum())
    rank = np.cumsum(eq, dtype=np.int64)
    return (gt | (eq & (rank <= need))).reshape(n, k)


def mask_2of4(w_bits: np.ndarray) -> np.ndarray:
    """Boolean mask keeping, in every aligned group of four columns, the two largest |w| (ties: lowest column)."""
    n, k = w_bits.shape
    if k % 4:
        raise ValueError("k_in must be a multiple of 4")
    mag = (w_bits & np.uint16(0x7FFF)).astype(np.int32).reshape(n, k // 4, 4)  # bf16 magnitudes order like their bits
    # stable descending sort inside the group: the lowest column wins among equals
    order = np.argsort(-mag, axis=-1, kind="stable")
    keep = np.zeros_like(mag, dtype=bool)
    np.put_along_axis(keep, order[..., :2], True, axis=-1)
    return keep.reshape(n, k)


# --------------------------------------------------------------------------- tensors


def _rng(cfg_id: int, layer: int, proj_id: int) -> np.random.Generator:
    return np.random.default_rng([SEED, int(cfg_id), int(layer), int(proj_id)])


def gen_weight_dense(cfg_id: int, layer: int, proj: str, n_out: int, k_in: int) -> np.ndarray:
    """Unpruned bf16 weight bits, W = 0.02 * z."""
    z = _rng(cfg_id, layer, PROJ[proj]).standard_normal((n_out, k_in), dtype=np.float32)
    z *= np.float32(0.02)
    return f32_to_bf16_bits(z)


def gen_weight(
    cfg_id: int,
    layer: int,
    proj: str,
    n_out: int,
    k_in: int,
    sparsity_pct: int,
    pattern: str = "row",
) -> np.ndarray:
    """Pruned bf16 weight bits: pruned entries are +0, kept entries are never zero."""
    w = gen_weight_dense(cfg_id, layer, proj, n_out, k_in)
    if pattern == "row":
        m = magnitude_mask_per_row(w, sparsity_pct)
    elif pattern == "global":
        m = magnitude_mask_global(w, sparsity_pct)
    elif pattern == "2:4":
        if sparsity_pct != 50:
            raise ValueError("the 2:4 pattern is 50 % sparse")
        m = mask_2of4(w)
    else:
        raise ValueError("pattern must be 'row', 'global' or '2:4'")
    w = np.where(m, w, np.uint16(0)).astype(np.uint16)
    # the sparsity pattern is the nonzero pattern: a kept +-0 would silently vanish
    if np.count_nonzero(w & np.uint16(0x7FFF)) != int(m.sum()):
        raise AssertionError("a kept weight is +-0; pick another seed")
    return w


def gen_x(cfg_id: int, layer: int, proj: str, k_tok: int, k_in: int) -> np.ndarray:
    """Activations, token-major [k_tok][k_in], bf16 bits, X = z."""
    z = _rng(cfg_id, layer, _X_BASE + PROJ[proj]).standard_normal((k_tok, k_in), dtype=np.float32)
    return f32_to_bf16_bits(z)


_LM_HEAD_ID = 300
_LM_H_ID = 301


def gen_lm_head(cfg_id: int, vocab: int, hidden: int) -> np.ndarray:
    """Dense (never pruned) LM-head weight bits [vocab][hidden], W = 0.02 * z, drawn in blocks of 8192 rows."""
    rng = _rng(cfg_id, 0, _LM_HEAD_ID)
    out = np.empty((vocab, hidden), dtype=np.uint16)
    for r0 in range(0, vocab, 8192):
        r1 = min(vocab, r0 + 8192)
        z = rng.standard_normal((r1 - r0, hidden), dtype=np.float32)
        z *= np.float32(0.02)
        out[r0:r1] = f32_to_bf16_bits(z)
    return out


def gen_final_hidden(cfg_id: int, k_tok: int, hidden: int) -> np.ndarray:
    """Final residual stream [k_tok][hidden] as float32, H = 3 * z (what the decoder stack hands to the head)."""
    z = _rng(cfg_id, 0, _LM_H_ID).standard_normal((k_tok, hidden), dtype=np.float32)
    return z * np.float32(3.0)


_KV_ID = 310


def gen_kv_history(cfg_id: int, layers: int, n_kv: int, max_pos: int, head_dim: int, n_hist: int):
    """Key and value caches [layers][n_kv][max_pos][head_dim] as bf16 bits: positions below n_hist hold a synthetic
    history (K = z, V = z: the size the keys and values of these stacks have), the rest is zero."""
    caches = []
    for which in (0, 1):
        c = np.zeros((layers, n_kv, max_pos, head_dim), dtype=np.uint16)
        for l in range(layers):
            z = _rng(cfg_id, l, _KV_ID + which).standard_normal((n_kv, n_hist, head_dim), dtype=np.float32)
            c[l, :, :n_hist] = f32_to_bf16_bits(z)
        caches.append(c)
    return caches[0], caches[1]


def gen_verify(
    cfg_id: int, batch: int, k: int, vocab: int, alpha: float, stream: int = 0
) -> Tuple[np.ndarray, np.ndarray]:
    """(draft [batch][k], target [batch][k+1]) int32 token ids."""
    if vocab < 2:
        raise ValueError("vocab must be >= 2")
    g = _rng(cfg_id, stream, _VERIFY_BASE)
    target = g.integers(0, vocab, size=(batch, k + 1), dtype=np.int64)
    match = g.random((batch, k)) < alpha
    u = g.integers(0, vocab - 1, size=(batch, k), dtype=np.int64)  # 0 .. vocab-2
    other = (target[:, :k] + 1 + u) % vocab  # never equal to target
    draft = np.where(match, target[:, :k], other)
    return draft.astype(np.int32), target.astype(np.int32)


# --------------------------------------------------------------------------- stacks


def layer_matrix_shapes(shape: StackShape) -> List[Tuple[str, int, int]]:
    """(projection, n_out, k_in) for the seven linears of one decoder block."""
    return [
        ("q", shape.q_out, shape.hidden),
        ("k", shape.kv_out, shape.hidden),
        ("v", shape.kv_out, shape.hidden),
        ("o", shape.hidden, shape.q_out),
        ("gate", shape.inter, shape.hidden),
        ("up", shape.inter, shape.hidden),
        ("down", shape.hidden, shape.inter),
    ]


def stack_matrices(shape: StackShape) -> Iterator[Tuple[int, str, int, int]]:
    """(layer, projection, n_out, k_in) over the whole stack, in execution order."""
    for layer in range(shape.layers):
        for proj, n_out, k_in in layer_matrix_shapes(shape):
            yield layer, proj, n_out, k_in
