"""Pins for the linear oracle: none of them re-uses the oracle's own formula."""
from fractions import Fraction

import numpy as np
import pytest

import sd2_workload as wl
from oracle import linear as ol
from oracle.bf16 import bits_to_f64


def _bits_of_ints(a):
    """bf16 bit patterns of small integers (exactly representable when |a| <= 256)."""
    return wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def _bf16_fraction(bits: int) -> Fraction:
    """Exact rational value of a bf16 bit pattern, decoded by hand from the fields."""
    s = -1 if bits & 0x8000 else 1
    e = (bits >> 7) & 0xFF
    m = bits & 0x7F
    if e == 0:
        return s * Fraction(m, 128) * Fraction(1, 2 ** 126)
    return s * (1 + Fraction(m, 128)) * (Fraction(2) ** (e - 127))


def test_bits_to_f64_against_field_decoding():
    rng = np.random.default_rng(1)
    bits = rng.integers(0, 0x7F80, size=200, dtype=np.uint16)  # finite, positive
    bits[::2] |= 0x8000
    got = bits_to_f64(bits)
    for b, g in zip(bits.tolist(), got.tolist()):
        assert Fraction(g) == _bf16_fraction(b)


def test_bruteforce_8x8_exact_rational():
    rng = np.random.default_rng(2)
    for trial in range(5):
        w_int = rng.integers(-9, 10, size=(8, 8))
        w_int[rng.random((8, 8)) < 0.5] = 0
        x_int = rng.integers(-7, 8, size=(3, 8))
        # dyadic scaling keeps everything exactly representable
        w_bits = _bits_of_ints(w_int * 0.25)
        x_bits = _bits_of_ints(x_int * 0.5)
        y = ol.sparse_linear(w_bits, x_bits)
        for t in range(3):
            for n in range(8):
                exact = sum(Fraction(int(w_int[n, c]), 4) * Fraction(int(x_int[t, c]), 2)
                            for c in range(8) if w_int[n, c] != 0)
                assert Fraction(float(y[t, n])) == exact


def test_exact_integer_reference_nonsquare():
    """Independent big-integer evaluation on a non-square case (catches transposes / dropped terms)."""
    w_bits = wl.gen_weight(9, 0, "q", 24, 64, 50)
    x_bits = wl.gen_x(9, 0, "q", 3, 64)
    y = ol.sparse_linear(w_bits, x_bits)
    assert y.shape == (3, 24)
    for t in range(3):
        for n in range(24):
            exact = sum(_bf16_fraction(int(w_bits[n, c])) * _bf16_fraction(int(x_bits[t, c]))
                        for c in range(64))
            scale = sum(abs(_bf16_fraction(int(w_bits[n, c])) * _bf16_fraction(int(x_bits[t, c])))
                        for c in range(64))
            assert abs(Fraction(float(y[t, n])) - exact) <= Fraction(64 * 2.3e-16) * scale


def test_masked_dense_equals_kept_column_loop():
    w_bits = wl.gen_weight(9, 1, "gate", 96, 256, 60)
    x_bits = wl.gen_x(9, 1, "gate", 5, 256)
    a = ol.sparse_linear(w_bits, x_bits)
    b = ol.sparse_linear_rowloop(w_bits, x_bits)
    assert ol.rel_l2(a, b) <= 1e-15


def test_explicit_mask_argument_prunes():
    """A mask given separately from the values must act exactly like zeroing the weights."""
    dense = wl.gen_weight_dense(9, 2, "o", 40, 128)
    m = wl.magnitude_mask_per_row(dense, 50)
    pruned = np.where(m, dense, 0).astype(np.uint16)
    x_bits = wl.gen_x(9, 2, "o", 2, 128)
    assert np.array_equal(ol.sparse_linear(dense, x_bits, mask=m), ol.sparse_linear(pruned, x_bits))
    # and it changes the answer (the mask is not ignored)
    assert ol.rel_l2(ol.sparse_linear(dense, x_bits), ol.sparse_linear(pruned, x_bits)) > 1e-2


def test_zero_sparsity_is_plain_matmul_fp32_crosscheck():
    dense = wl.gen_weight(9, 3, "up", 32, 128, 0)
    assert np.count_nonzero(dense) == dense.size
    x_bits = wl.gen_x(9, 3, "up", 4, 128)
    y = ol.sparse_linear(dense, x_bits)
    # textbook triple loop in Python floats (fp64), different code path and summation order
    w = wl.bf16_bits_to_f32(dense).astype(float)
    x = wl.bf16_bits_to_f32(x_bits).astype(float)
    ref = [[sum(w[n][c] * x[t][c] for c in range(128)) for n in range(32)] for t in range(4)]
    assert ol.rel_l2(y, np.array(ref)) < 1e-14


def test_one_hot_input_returns_masked_column():
    w_bits = wl.gen_weight(9, 4, "down", 48, 64, 50)
    for c in (0, 17, 63):
        x = np.zeros((1, 64), dtype=np.float32)
        x[0, c] = 1.0
        y = ol.sparse_linear(w_bits, wl.f32_to_bf16_bits(x))
        assert np.array_equal(y[0], wl.bf16_bits_to_f32(w_bits[:, c]).astype(np.float64))


def test_linearity_on_exact_inputs():
    rng = np.random.default_rng(5)
    w_bits = wl.gen_weight(9, 5, "q", 16, 64, 50)
    x1 = rng.integers(-8, 9, size=(2, 64)).astype(np.float32)
    x2 = rng.integers(-8, 9, size=(2, 64)).astype(np.float32)
    f = lambda x: ol.sparse_linear(w_bits, wl.f32_to_bf16_bits(x))
    assert np.allclose(f(x1 + x2), f(x1) + f(x2), rtol=0, atol=1e-12)
    assert np.allclose(f(4 * x1), 4 * f(x1), rtol=0, atol=0)


def test_negative_zero_counts_as_pruned():
    w = _bits_of_ints([[1.0, 2.0], [3.0, 4.0]])
    w[0, 1] = 0x8000
    assert ol.nonzero_mask(w).tolist() == [[True, False], [True, True]]


def test_rel_l2_definition():
    assert ol.rel_l2([3.0, 4.0], [3.0, 4.0]) == 0.0
    assert ol.rel_l2([0.0, 0.0], [3.0, 4.0]) == pytest.approx(1.0)
    assert ol.rel_l2([3.0, 4.0 + 5e-3], [3.0, 4.0]) == pytest.approx(1e-3)


def test_f64x_variant_against_exact_rationals_and_the_bit_input_variant():
    """sparse_linear_f64x takes activations as float64 values instead of bf16 bits.  Pin 1: exact rational brute
    force with activations that are NOT bf16 values (thirds of integers scaled by a power of two are not needed:
    quarters and eighths of small integers are exact in float64 and in Fraction alike).  Pin 2: on bf16-exact
    activations it must equal the bit-input variant exactly.  Pin 3: a transposed operand or a dropped mask fails."""
    rng = np.random.default_rng(41)
    w_int = rng.integers(-9, 10, size=(6, 10))
    w_int[rng.random((6, 10)) < 0.5] = 0
    w_bits = _bits_of_ints(w_int)
    x = rng.integers(-40, 41, size=(3, 10)).astype(np.float64) / 8.0   # multiples of 1/8: exact in binary
    got = ol.sparse_linear_f64x(w_bits, x)
    assert got.shape == (3, 6)
    for t in range(3):
        for n in range(6):
            want = sum(_bf16_fraction(int(w_bits[n, c])) * Fraction(int(round(x[t, c] * 8)), 8) for c in range(10))
            assert Fraction(float(got[t, n])) == want
    # the mask argument prunes: brute force over the kept columns only
    mask = rng.random((6, 10)) < 0.5
    got_m = ol.sparse_linear_f64x(w_bits, x, mask)
    for t in range(3):
        for n in range(6):
            want = sum(_bf16_fraction(int(w_bits[n, c])) * Fraction(int(round(x[t, c] * 8)), 8) for c in range(10) if mask[n, c])
            assert Fraction(float(got_m[t, n])) == want
    # bf16-exact activations: identical to the variant that takes bits
    x_bits = _bits_of_ints(rng.integers(-20, 21, size=(4, 10)))
    assert np.array_equal(ol.sparse_linear_f64x(w_bits, bits_to_f64(x_bits)), ol.sparse_linear(w_bits, x_bits))
