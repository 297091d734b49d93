"""2:4 semi-structured linears (blob format 3, structured-sparse matrix instruction) against the oracle.

The oracle is the same masked-dense definition as for unstructured sparsity: the 2:4 matrix simply is a bf16 matrix
with exact zeros (Sec. 2.4), so `oracle.linear.sparse_linear` applies unchanged; bar 1e-3 relative L2 per output tensor."""
from types import SimpleNamespace

import numpy as np
import pytest

import sd2_workload as wl
from oracle import linear as ol
from oracle import stack as os_

pytestmark = pytest.mark.gpu

TOL = 1e-3
NM24 = 3


def _run(w, x):
    import gpu_util as gu
    return gu.run_linear(gu.SparseMat(w, NM24), x, sparse=True)


@pytest.mark.parametrize(
    "n,k,k_tok",
    [
        (512, 512, 1),       # two slabs: four wavefronts, two of them idle
        (512, 512, 5),
        (100, 768, 5),       # ragged last strip, three slabs
        (48, 64, 3),         # a quarter of a slab
        (3072, 3072, 5),     # o / q of the 3B shape: 12 wavefronts, one slab each
        (2048, 3072, 16),    # a full token block
        (1024, 8192, 8),     # down of the 3B shape: 16 wavefronts, two slabs each
        (256, 8960, 5),      # down of the 1.5B shape: 35 slabs, three per wavefront, ragged last slab
        (272, 1536, 7),      # six slabs on eight wavefronts
        (2048, 2048, 17),    # more than one token block
        (640, 3072, 40),
        (16384, 3072, 5),    # fused gate+up of the 3B shape at full size
    ],
)
def test_linear_matches_oracle(n, k, k_tok):
    w = wl.gen_weight(51, 0, "q", n, k, 50, pattern="2:4")
    x = wl.gen_x(51, 0, "q", k_tok, k)
    y = _run(w, x)
    ref = ol.sparse_linear(w, x)
    assert np.isfinite(y).all()
    assert ol.rel_l2(y, ref) <= TOL


def test_exact_on_small_integers():
    """Every product and partial sum is exactly representable: the result must be exact, which pins the operand
    layout (a wrong column index or a swapped pair would change an integer)."""
    rng = np.random.default_rng(7)
    n, k, k_tok = 64, 512, 6
    wi = rng.integers(-4, 5, size=(n, k)).astype(np.float32)
    # impose 2:4 with every admissible pattern, including groups of one value and empty groups
    keep = np.zeros((n, k // 4, 4), dtype=bool)
    pats = [(0, 1), (0, 2), (0, 3), (1, 2), (1, 3), (2, 3), (0,), (1,), (2,), (3,), ()]
    choice = rng.integers(0, len(pats), size=(n, k // 4))
    for pi, pat in enumerate(pats):
        for c in pat:
            keep[..., c] |= choice == pi
    wi = np.where(keep.reshape(n, k), wi, 0.0).astype(np.float32)
    xi = rng.integers(-3, 4, size=(k_tok, k)).astype(np.float32)
    w, x = wl.f32_to_bf16_bits(wi), wl.f32_to_bf16_bits(xi)
    y = _run(w, x)
    assert np.array_equal(y, (xi.astype(np.float64) @ wi.astype(np.float64).T).astype(np.float32))


def test_zero_matrix_and_single_values():
    n, k = 32, 256
    w = np.zeros((n, k), dtype=np.uint16)
    x = wl.gen_x(52, 0, "q", 4, k)
    assert not _run(w, x).any()
    w[3, 77] = 0x3F80   # 1.0: y[t][3] = x[t][77]
    w[31, 255] = 0xC000  # -2.0
    y = _run(w, x)
    xf = wl.bf16_bits_to_f32(x)
    expect = np.zeros((4, n), dtype=np.float32)
    expect[:, 3] = xf[:, 77]
    expect[:, 31] = -2.0 * xf[:, 255]
    assert np.array_equal(y, expect)


def test_run_to_run_determinism():
    w = wl.gen_weight(53, 0, "q", 1024, 3072, 50, pattern="2:4")
    x = wl.gen_x(53, 0, "q", 5, 3072)
    assert np.array_equal(_run(w, x), _run(w, x))  # fixed summation order, no atomics


@pytest.fixture(params=["single-launch", "multi-launch"])
def forward_path(request, sd2_options):
    """Both forwards: the persistent kernel (its 2:4 variant) and the chain of one launch per linear and glue step."""
    if request.param == "multi-launch":
        sd2_options.set("forward_multi", 1)
    else:
        sd2_options.set("forward_multi", 0)
    return request.param


def _stack24(shape, seed):
    table = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(shape)}
    cache = {}

    def get(layer, proj):
        if (layer, proj) not in cache:
            cache[(layer, proj)] = wl.gen_weight(seed, layer, proj, table[proj][0], table[proj][1], 50, pattern="2:4")
        return cache[(layer, proj)]

    return get


@pytest.mark.parametrize("k_tok", [1, 5, 8])
def test_stack_of_2of4_linears_end_to_end(k_tok, forward_path):
    """Every decoder linear in format 3 (two layers of a reduced 3B-like shape)."""
    import gpu_util as gu
    shape = SimpleNamespace(layers=2, hidden=1024, q_out=1024, kv_out=256, inter=2048, n_heads=8, n_kv=2, head_dim=128)
    get = _stack24(shape, 54)
    h_in = wl.gen_x(54, 0, "q", k_tok, shape.hidden)
    ref = os_.drafter_forward(shape, get, h_in)
    model = gu.build_model(shape, get, sparse=True, fmt=NM24)
    out = gu.run_forward(model, h_in, shape.hidden)
    assert np.isfinite(out).all()
    assert ol.rel_l2(out, ref) <= 5e-3  # end to end over rounding points; each linear is inside 1e-3 (below)


@pytest.mark.parametrize("which", ["small-3-layers", "llama3b-2-layers"])
def test_stack_of_2of4_linears_link_by_link(which, forward_path):
    """Every linear and glue step against the oracle on the GPU's own recorded inputs (bar 1e-3 per linear)."""
    import gpu_util as gu
    from test_gpu_stack import _verify_steps
    if which == "small-3-layers":
        shape = SimpleNamespace(layers=3, hidden=768, q_out=768, kv_out=256, inter=1536, n_heads=6, n_kv=2, head_dim=128)
    else:
        shape = SimpleNamespace(**{**wl.CONFIGS[3]["shape"].__dict__, "layers": 2})
    get = _stack24(shape, 55)
    h_in = wl.gen_x(55, 0, "q", 5, shape.hidden)
    model = gu.build_model(shape, get, sparse=True, fmt=NM24)
    h_out, x, src = gu.run_forward_trace(model, h_in, shape)
    assert np.isfinite(h_out).all()
    _verify_steps(shape, get, h_in, h_out, x, src)
