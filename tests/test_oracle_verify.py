import itertools
import os

import numpy as np
import pytest

import sd2_workload as wl
from oracle import verify as ov


def _hand_cases(golden_dir):
    cases = []
    with open(os.path.join(golden_dir, "verify_hand_cases.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            d, t, n, o = [p.split() for p in line.split("|")]
            cases.append(([int(v) for v in d], [int(v) for v in t], int(n[0]), [int(v) for v in o]))
    return cases


def test_hand_worked_cases(golden_dir):
    cases = _hand_cases(golden_dir)
    assert len(cases) == 5
    for d, t, n, o in cases:
        acc, out = ov.greedy_verify(np.array([d], dtype=np.int32).reshape(1, len(d)), np.array([t], dtype=np.int32))
        assert acc.tolist() == [n]
        assert out.tolist() == [o]


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_all_match_patterns(k):
    """Every one of the 2^k agree/disagree patterns; expected length = leading run of agreements."""
    pats = list(itertools.product([0, 1], repeat=k))
    target = np.arange(10, 10 + k + 1, dtype=np.int32)[None, :].repeat(len(pats), 0)
    draft = target[:, :k].copy()
    for r, p in enumerate(pats):
        for j, agree in enumerate(p):
            if not agree:
                draft[r, j] += 100
    acc, out = ov.greedy_verify(draft, target)
    for r, p in enumerate(pats):
        lead = 0
        for agree in p:
            if not agree:
                break
            lead += 1
        assert acc[r] == lead
        assert out[r, :lead].tolist() == target[r, :lead].tolist()
        assert out[r, lead] == target[r, lead]
        assert (out[r, lead + 1:] == -1).all()


def test_invariants_and_closed_form_mean():
    k, alpha = 5, 0.85
    draft, target = wl.gen_verify(5, 200000, k, 128256, alpha)
    acc, out = ov.greedy_verify(draft, target, vocab=128256)
    assert acc.min() >= 0 and acc.max() <= k
    rows = np.arange(acc.size)
    assert np.array_equal(out[rows, acc], target[rows, acc])
    short = acc < k
    assert (draft[rows[short], acc[short]] != target[rows[short], acc[short]]).all()
    for j in range(k):
        sel = acc > j
        assert np.array_equal(out[sel, j], draft[sel, j])
    emitted = acc + 1
    mean = emitted.mean()
    expect = ov.expected_emitted(alpha, k)
    assert expect == pytest.approx(4.1519, abs=1e-3)
    # std of emitted <= 2, 200k samples -> 4 sigma ~ 0.018
    assert abs(mean - expect) < 0.02


def test_closed_form_values():
    assert ov.expected_emitted(0.80, 5) == pytest.approx(3.68928, abs=1e-5)
    assert ov.expected_emitted(0.90, 5) == pytest.approx(4.68559, abs=1e-5)
    assert ov.expected_emitted(1.0, 5) == 6.0
    assert ov.expected_emitted(0.0, 5) == 1.0


def test_range_check():
    with pytest.raises(ValueError):
        ov.greedy_verify(np.array([[5]]), np.array([[5, 7]]), vocab=7)
    with pytest.raises(ValueError):
        ov.greedy_verify(np.array([[5, 1]]), np.array([[5, 7]]))
