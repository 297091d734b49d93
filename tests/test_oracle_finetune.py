"""Pins for the masked-gradient oracle (Sec. 2.4: gradients of pruned parameters are set to zero)."""
import numpy as np

import sd2_workload as wl
from oracle import bf16 as ob
from oracle import finetune as oft
from oracle import linear as ol


def _case():
    w = wl.gen_weight(81, 0, "q", 48, 320, 50)
    g = np.random.default_rng(81).standard_normal((48, 320)).astype(np.float32)
    return w, g


def test_equals_the_elementwise_product_with_the_0_1_mask_on_finite_gradients():
    w, g = _case()
    m = ol.nonzero_mask(w).astype(np.float32)
    assert np.array_equal(oft.mask_gradient(w, g), g * m + 0.0)  # + 0.0 turns the product's -0 into +0


def test_idempotent_and_keeps_exactly_the_kept_entries():
    w, g = _case()
    once = oft.mask_gradient(w, g)
    assert np.array_equal(oft.mask_gradient(w, once), once)
    kept = ol.nonzero_mask(w)
    assert np.array_equal(once[kept], g[kept]) and not once[~kept].any()
    assert not np.signbit(once[~kept]).any()  # +0, not -0


def test_non_finite_values_at_pruned_positions_vanish():
    w, g = _case()
    pruned = np.argwhere(~ol.nonzero_mask(w))
    g[tuple(pruned[0])] = np.nan
    g[tuple(pruned[1])] = np.inf
    out = oft.mask_gradient(w, g)
    assert np.isfinite(out).all()


def test_pruned_weights_stay_zero_under_sgd():
    """The statement of Sec. 2.4: with masked gradients the pruned parameters never move."""
    w, g = _case()
    w64 = ob.bits_to_f64(w)
    for step in range(3):
        w64 = oft.sgd_step(w64, w, g * (step + 1), lr=0.1)
    assert not w64[~ol.nonzero_mask(w)].any()
    assert (w64[ol.nonzero_mask(w)] != ob.bits_to_f64(w)[ol.nonzero_mask(w)]).any()
