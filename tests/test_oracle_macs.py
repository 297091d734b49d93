import os
from fractions import Fraction

import pytest

import sd2_workload as wl
from oracle import macs


def _golden(golden_dir):
    d = {}
    with open(os.path.join(golden_dir, "macs_abstract.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            d[k] = float(v)
    return d


def test_abstract_mac_reduction(golden_dir):
    g = _golden(golden_dir)
    s = wl.CONFIGS[3]["shape"]
    red = macs.mac_reduction(s.layers, s.hidden, s.q_out, s.kv_out, s.inter, s.vocab, 50)
    assert red == Fraction(1409286144, 3212574720)
    pct = float(red) * 100
    # the abstract prints the value rounded to two decimals (43.868 -> "43.87")
    assert round(pct, 2) == g["mac_reduction_percent_over"]


def test_counts_by_hand():
    s = wl.CONFIGS[3]["shape"]
    assert macs.decoder_linear_macs(s.layers, s.hidden, s.q_out, s.kv_out, s.inter) == 28 * 100663296
    assert macs.lm_head_macs(s.hidden, s.vocab) == 394002432
    # without the LM head the reduction would be exactly the sparsity
    assert Fraction(28 * 100663296 // 2, 28 * 100663296) == Fraction(1, 2)


def test_abstract_mal_ratios(golden_dir):
    g = _golden(golden_dir)
    assert round(g["mal_sd2_50_3b"] / g["mal_layer_pruned_50_3b"], 2) == g["mal_ratio_vs_layer_pruned"]
    assert abs((g["mal_dense_3b"] - g["mal_sd2_50_3b"]) / g["mal_dense_3b"] * 100 - g["mal_reduction_percent"]) < 0.02


def test_improvement_factor_eq3():
    assert macs.improvement_factor(4.16, 5, 0.05) == pytest.approx(3.328)
    assert macs.improvement_factor(4.0, 5, 0.0) == 4.0
    # a drafter as slow as the target can never win with k >= MAL
    assert macs.improvement_factor(4.16, 5, 1.0) < 1.0
