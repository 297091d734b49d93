"""Parity of the HIP linears (through the C ABI) against the fp64 oracle.

Bar: relative L2 error <= 1e-3 per output tensor (bf16 inputs, fp32 accumulation); in practice the
error is ~1e-6 because bf16 x bf16 products are exact in fp32 and only the summation order differs.
"""
import numpy as np
import pytest

import sd2_workload as wl
from oracle import linear as ol

pytestmark = pytest.mark.gpu
TOL = 1e-3


@pytest.fixture(autouse=True, params=["final", "partials", "partials-vector-alu"])
def linear_kernel(request, sd2_options):
    """Every case runs on the sparse kernels: the one that adds the slabs up inside the workgroup (up to 16 tokens), the
    one that leaves a partial result per slab for a second launch, and the latter's measurement variant that multiplies
    on the vector ALU instead of the matrix cores (up to 8 tokens; wider cases fall back to the matrix cores)."""
    sd2_options.set("linear_partials", {"final": 0, "partials": 1, "partials-vector-alu": 2}[request.param])
    return request.param


def _gu():
    import gpu_util
    return gpu_util


def _ints(a):
    return wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def test_mfma_lane_layout_exact_small_integers():
    """All partial sums are exact in fp32, so any wrong lane/column mapping shows as a hard mismatch."""
    gu = _gu()
    rng = np.random.default_rng(7)
    w = rng.integers(-4, 5, size=(48, 320)).astype(np.float32)
    w[rng.random(w.shape) < 0.5] = 0
    x = rng.integers(-3, 4, size=(5, 320)).astype(np.float32)
    wb, xb = _ints(w), _ints(x)
    ref = ol.sparse_linear(wb, xb)
    y = gu.run_linear(gu.SparseMat(wb), xb)
    assert np.array_equal(y.astype(np.float64), ref)
    y = gu.run_linear(gu.DenseMat(wb), xb, sparse=False)
    assert np.array_equal(y.astype(np.float64), ref)


def test_bruteforce_8x8_padded():
    gu = _gu()
    rng = np.random.default_rng(8)
    w = np.zeros((8, 64), dtype=np.float32)
    w[:, :8] = rng.integers(-9, 10, size=(8, 8)) * 0.25
    w[rng.random(w.shape) < 0.5] = 0
    x = np.zeros((3, 64), dtype=np.float32)
    x[:, :8] = rng.integers(-7, 8, size=(3, 8)) * 0.5
    wb, xb = _ints(w), _ints(x)
    y = gu.run_linear(gu.SparseMat(wb), xb)
    assert np.array_equal(y.astype(np.float64), ol.sparse_linear(wb, xb))


@pytest.mark.parametrize("k_tok", [1, 5])
def test_cfg1_single_linear(k_tok):
    gu = _gu()
    w = wl.gen_weight(1, 0, "q", 512, 512, 50)
    x = wl.gen_x(1, 0, "q", k_tok, 512)
    ref = ol.sparse_linear(w, x)
    ys = gu.run_linear(gu.SparseMat(w), x)
    yd = gu.run_linear(gu.DenseMat(w), x, sparse=False)
    assert ol.rel_l2(ys, ref) <= TOL and ol.rel_l2(yd, ref) <= TOL
    assert ol.rel_l2(ys, ref) < 1e-5


@pytest.mark.parametrize("n,k,pct,k_tok,pattern", [
    (1000, 832, 50, 5, "row"),      # ragged rows (not a multiple of 16), ragged last slab
    (1000, 832, 60, 3, "row"),
    (520, 1536, 70, 8, "row"),
    (2048, 2048, 50, 5, "global"),  # unequal rows
    (333, 64, 50, 1, "row"),        # n_out not a multiple of 4: scalar stores
    (64, 8960, 66, 5, "row"),
    (256, 3072, 75, 16, "row"),
    (256, 3072, 50, 17, "row"),     # two token groups
    (128, 1024, 50, 33, "row"),     # three token groups (runs as four)
    (128, 1024, 50, 64, "row"),
    (8192, 3072, 50, 5, "row"),     # several tiles per wavefront: exercises the prefetch pipeline
    (8192, 3072, 30, 5, "row"),     # dense tiles: the large LDS staging variant
    (2048, 1024, 0, 8, "row"),      # nothing pruned
])
def test_shapes_and_sparsities(n, k, pct, k_tok, pattern):
    gu = _gu()
    w = wl.gen_weight(13, 0, "gate", n, k, pct, pattern=pattern)
    x = wl.gen_x(13, 0, "gate", k_tok, k)
    ref = ol.sparse_linear(w, x)
    ys = gu.run_linear(gu.SparseMat(w), x)
    assert not np.isnan(ys).any()
    assert ol.rel_l2(ys, ref) <= TOL
    yd = gu.run_linear(gu.DenseMat(w), x, sparse=False)
    assert ol.rel_l2(yd, ref) <= TOL


def test_degenerate_patterns():
    gu = _gu()
    w = wl.gen_weight(13, 1, "q", 96, 512, 50)
    w[3, :] = 0; w[16:32, :] = 0; w[:, 256:] = 0; w[40, :256] = 0x3F80
    x = wl.gen_x(13, 1, "q", 5, 512)
    assert ol.rel_l2(gu.run_linear(gu.SparseMat(w), x), ol.sparse_linear(w, x)) <= TOL
    z = np.zeros((32, 256), dtype=np.uint16)                       # everything pruned
    y = gu.run_linear(gu.SparseMat(z), wl.gen_x(13, 2, "q", 2, 256))
    assert (y == 0).all()


def test_zero_sparsity_matches_dense_kernel():
    gu = _gu()
    w = wl.gen_weight(13, 3, "up", 256, 1024, 0)
    x = wl.gen_x(13, 3, "up", 5, 1024)
    ys = gu.run_linear(gu.SparseMat(w), x)
    yd = gu.run_linear(gu.DenseMat(w), x, sparse=False)
    ref = ol.sparse_linear(w, x)
    assert ol.rel_l2(ys, ref) <= TOL and ol.rel_l2(yd, ref) <= TOL
    assert ol.rel_l2(ys, yd) < 1e-5


def test_run_to_run_determinism():
    gu = _gu()
    w = wl.gen_weight(13, 4, "down", 512, 2048, 50)
    x = wl.gen_x(13, 4, "down", 5, 2048)
    mat = gu.SparseMat(w)
    first = gu.run_linear(mat, x)
    for _ in range(5):
        assert np.array_equal(gu.run_linear(mat, x), first)


def test_cfg2_mlp_block():
    import torch
    import paper_2504_08838_amd as sd2
    from oracle import stack as os_
    gu = _gu()
    hid, inter, k_tok = 2048, 8192, 5
    wg = wl.gen_weight(2, 0, "gate", inter, hid, 50)
    wu = wl.gen_weight(2, 0, "up", inter, hid, 50)
    wd = wl.gen_weight(2, 0, "down", hid, inter, 50)
    x = wl.gen_x(2, 0, "gate", k_tok, hid)
    ref, m_ref = os_.mlp_block(wg, wu, wd, x)
    gate_up = gu.SparseMat(np.concatenate([wg, wu], axis=0))
    down = gu.SparseMat(wd)
    # stand-alone linears at full size against the oracle
    assert ol.rel_l2(gu.run_linear(gate_up, x), np.concatenate([ol.sparse_linear(wg, x), ol.sparse_linear(wu, x)], axis=1)) <= TOL
    xd, y = gu.dev(x), torch.empty((k_tok, hid), dtype=torch.float32, device="cuda")
    nb = sd2.mlp_workspace_size(gate_up.m, down.m, k_tok)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    sd2.sparse_mlp_forward(gate_up.m, down.m, xd.data_ptr(), k_tok, y.data_ptr(), ws.data_ptr(), nb, gu.stream_ptr())
    torch.cuda.synchronize()
    assert ol.rel_l2(y.cpu().numpy(), ref) <= TOL
