"""Wide-verification regime (16 to 64 tokens in one call) at the 3B drafter's own matrix sizes, and element-wise
error bounds at full size.

Every output element is a sum of exact bf16 x bf16 products accumulated in fp32, in some order.  Whatever the order,
|y - exact| <= gamma_n * sum_c |w||x| with gamma_n ~ n * 2^-24 for n terms added one after the other; the kernels add
in blocks (matrix instructions over 32 columns, then slabs, then wavefronts), which is far tighter, so the bound
64 * 2^-24 * sum_c |w||x| holds with room to spare for up to 8960 terms and still catches a single wrong element
(a dropped or doubled value moves an element by about sum|w||x| / sqrt(n), four orders of magnitude above it)."""
import numpy as np
import pytest

import sd2_workload as wl
from oracle import linear as ol
from oracle.bf16 import bits_to_f64

pytestmark = pytest.mark.gpu
TOL = 1e-3


def _gu():
    import gpu_util
    return gpu_util


def _elementwise_bound(w_bits, x_bits):
    return 64.0 * 2.0 ** -24 * (np.abs(bits_to_f64(x_bits)) @ np.abs(bits_to_f64(w_bits)).T)


def _check(y, w, x, what):
    ref = ol.sparse_linear(w, x)
    assert not np.isnan(y).any(), what
    assert ol.rel_l2(y, ref) <= TOL, what
    excess = np.abs(y.astype(np.float64) - ref) - _elementwise_bound(w, x)
    assert excess.max() <= 0.0, f"{what}: element {np.unravel_index(np.argmax(excess), excess.shape)} off by more than the fp32 summation bound"


@pytest.fixture(scope="module")
def full_size_mats():
    """Fused gate+up (16384 x 3072) and down (3072 x 8192) of the 3B shape at 50 %, packed and uploaded once."""
    gu = _gu()
    gate_up = np.concatenate([wl.gen_weight(3, 1, "gate", 8192, 3072, 50), wl.gen_weight(3, 1, "up", 8192, 3072, 50)], axis=0)
    down = wl.gen_weight(3, 1, "down", 3072, 8192, 50)
    return {"gate_up": (gate_up, gu.SparseMat(gate_up), gu.DenseMat(gate_up)), "down": (down, gu.SparseMat(down), gu.DenseMat(down))}


@pytest.mark.parametrize("kernel", ["final", "partials"])
@pytest.mark.parametrize("k_tok", [5, 16, 32, 64])
@pytest.mark.parametrize("which", ["gate_up", "down"])
def test_full_size_linears_element_by_element(full_size_mats, which, k_tok, kernel, sd2_options):
    gu = _gu()
    sd2_options.set("linear_partials", 1 if kernel == "partials" else 0)
    w, sparse, dense = full_size_mats[which]
    x = wl.gen_x(3, 1, "gate" if which == "gate_up" else "down", k_tok, w.shape[1])
    _check(gu.run_linear(sparse, x), w, x, f"sparse {kernel} {which} k={k_tok}")
    if kernel == "final":
        _check(gu.run_linear(dense, x, sparse=False), w, x, f"dense {which} k={k_tok}")


@pytest.mark.parametrize("n,k,k_tok", [
    (96, 1280, 40),     # three token groups, one slab per wavefront
    (200, 3328, 64),    # four groups, 13 slabs: two slabs per wavefront, ragged rows
    (48, 8960, 17),     # 35 slabs: three per wavefront
    (64, 12288, 33),    # 48 slabs: four per wavefront
    (1040, 512, 64),    # more strips than one round per workgroup, ragged last strip
])
def test_wide_exact_integers(n, k, k_tok):
    """Small integers: every partial sum is exact in fp32, so the result must equal the oracle bit for bit whatever
    the order of the adds -- any slip in token-group indexing shows as a wrong integer."""
    gu = _gu()
    rng = np.random.default_rng([77, n, k, k_tok])
    w_int = rng.integers(-8, 9, size=(n, k))
    w_int[rng.random((n, k)) < 0.5] = 0
    x_int = rng.integers(-4, 5, size=(k_tok, k))
    wb = wl.f32_to_bf16_bits(w_int.astype(np.float32))
    xb = wl.f32_to_bf16_bits(x_int.astype(np.float32))
    y = gu.run_linear(gu.SparseMat(wb), xb)
    assert np.array_equal(y.astype(np.int64), x_int @ w_int.T)


@pytest.mark.parametrize("k_tok", [16, 17, 31, 48, 49, 64])
def test_wide_token_counts_on_both_kernels(k_tok, sd2_options):
    gu = _gu()
    w = wl.gen_weight(13, 3, "gate", 528, 3072, 50)
    x = wl.gen_x(13, 3, "gate", k_tok, 3072)
    mat = gu.SparseMat(w)
    for partials in (0, 1):
        sd2_options.set("linear_partials", partials)
        _check(gu.run_linear(mat, x), w, x, f"k={k_tok} partials={partials}")


@pytest.mark.parametrize("k_tok", [16, 40, 64])
def test_wide_mlp_block_with_the_gated_epilogue(k_tok):
    """gate|up with the gated product in the linear's own epilogue, then down: the 1B-shape block on 16 to 64 tokens."""
    import torch
    import paper_2504_08838_amd as sd2
    from oracle import stack as os_
    gu = _gu()
    hidden, inter = 2048, 8192
    wg, wu, wd = (wl.gen_weight(2, 1, p, *sh, 50) for p, sh in (("gate", (inter, hidden)), ("up", (inter, hidden)), ("down", (hidden, inter))))
    x_bits = wl.gen_x(2, 1, "gate", k_tok, hidden)
    ref, _ = os_.mlp_block(wg, wu, wd, x_bits)
    g_u, dn = gu.SparseMat(np.concatenate([wg, wu], axis=0)), gu.SparseMat(wd)
    x = gu.dev(x_bits)
    y = torch.full((k_tok, hidden), float("nan"), dtype=torch.float32, device="cuda")
    nb = sd2.mlp_workspace_size(g_u.m, dn.m, k_tok)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    sd2.sparse_mlp_forward(g_u.m, dn.m, x.data_ptr(), k_tok, y.data_ptr(), ws.data_ptr(), nb, gu.stream_ptr())
    torch.cuda.synchronize()
    # end to end through one bf16 rounding point: a few products within fp32 error of a rounding boundary may round the other way
    assert ol.rel_l2(y.cpu().numpy(), ref) <= 2e-3


@pytest.mark.parametrize("k_tok", [16, 64])
def test_wide_two_layers_at_3b_width_link_by_link(k_tok):
    """Two layers of the 3B shape on 16 and 64 tokens: every linear and every glue step against the oracle on the GPU's
    own recorded inputs (the wide regime runs as one launch per linear and glue step)."""
    from types import SimpleNamespace
    from test_gpu_stack import _verify_steps, _weights
    from oracle import stack as os_
    gu = _gu()
    shape = SimpleNamespace(**{**wl.CONFIGS[3]["shape"].__dict__, "layers": 2})
    get = _weights(shape, 3)
    h_in = wl.gen_x(3, 0, "q", k_tok, shape.hidden)
    model = gu.build_model(shape, get)
    h_out, x, src = gu.run_forward_trace(model, h_in, shape)
    _verify_steps(shape, get, h_in, h_out, x, src)
    plain = gu.run_forward(model, h_in, shape.hidden)      # the non-recording entry point (fused epilogues) agrees
    assert ol.rel_l2(plain, h_out) <= 5e-3
    assert ol.rel_l2(plain, os_.drafter_forward(shape, get, h_in)) <= 5e-3
