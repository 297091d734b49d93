"""Pins for the magnitude-pruning oracle (Sec. 2.3: one-shot pruning at a uniform per-layer sparsity)."""
import numpy as np
import pytest

import sd2_workload as wl
from oracle import prune as opr


def _bits(vals):
    return wl.f32_to_bf16_bits(np.asarray(vals, dtype=np.float32))


def test_hand_case_rows():
    w = _bits([[1.0, -3.0, 2.0, 0.5, -2.0, 4.0, 0.25, -0.125] * 8])  # 64 columns, 50 % -> keep 32 per row
    out = wl.bf16_bits_to_f32(opr.prune_rows(w, 50))
    # per period of eight the magnitudes are 1, 3, 2, .5, 2, 4, .25, .125: kept are 3, 2, 2, 4 (and then 1 only if
    # needed); 32 of 64 = exactly the four largest of every period
    assert np.array_equal(out[0, :8], np.array([0, -3.0, 2.0, 0, -2.0, 4.0, 0, 0], dtype=np.float32))
    assert (out != 0).sum() == 32


def test_ties_go_to_the_lower_column():
    w = _bits([[1.0] * 64])
    out = opr.prune_rows(w, 75)  # keep 16 of 64 equal values: the first sixteen columns
    assert (out[0, :16] != 0).all() and not out[0, 16:].any()
    w24 = _bits([[2.0, 2.0, 2.0, 2.0, 1.0, 3.0, 3.0, 3.0]])
    assert wl.bf16_bits_to_f32(opr.prune_2of4(w24))[0].tolist() == [2.0, 2.0, 0, 0, 0, 3.0, 3.0, 0]


@pytest.mark.parametrize("pct", [50, 60, 70])
def test_counts_and_dominance(pct):
    w = wl.gen_weight_dense(95, 0, "q", 24, 320)
    out = opr.prune_rows(w, pct)
    kept = (out & 0x7FFF) != 0
    assert (kept.sum(axis=1) == 320 - (pct * 320) // 100).all()
    mag = (w & 0x7FFF).astype(np.int64)
    assert (np.where(kept, mag, 1 << 20).min(axis=1) >= np.where(kept, -1, mag).max(axis=1)).all()
    assert np.array_equal(out[kept], w[kept])  # kept entries keep their bits, sign included


def test_agrees_with_the_generators_masks():
    """Two independent implementations of the same rule (the generator vectorises it with partial sorts)."""
    w = wl.gen_weight_dense(96, 0, "q", 32, 384)
    for pct in (50, 60, 70):
        assert np.array_equal(opr.prune_rows(w, pct), np.where(wl.magnitude_mask_per_row(w, pct), w, 0))
    assert np.array_equal(opr.prune_2of4(w), np.where(wl.mask_2of4(w), w, 0))


def test_minus_zero_and_zero_rows():
    w = np.zeros((2, 64), dtype=np.uint16)
    w[0, 5] = 0x8000  # -0: magnitude zero; whatever is "kept" among zeros, the result holds no non-zero value
    out = opr.prune_rows(w, 50)
    assert not (out & 0x7FFF).any()
