"""The allocation-free sparse linear (partial sums in the library's static device array) against sd2_sparse_linear."""
import numpy as np
import pytest
import torch

import paper_2504_08838_amd as sd2
import sd2_workload as wl
from oracle import linear as ol

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _both(n_out, k_in, k_tok, seed):
    w = wl.gen_weight(seed, 0, "down", n_out, k_in, 50)
    x_bits = wl.gen_x(seed, 0, "down", k_tok, k_in)
    mat = gu.SparseMat(w)
    assert sd2.linear_workspace_size(mat.m, k_tok) > 0, "the case must be one that needs partial sums"
    y_ref = gu.run_linear(mat, x_bits, sparse=True)
    x = gu.dev(x_bits)
    y = torch.full((k_tok, n_out), float("nan"), dtype=torch.float32, device="cuda")
    sd2.sparse_linear_static(mat.m, x.data_ptr(), k_tok, y.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    return y.cpu().numpy(), y_ref, ol.sparse_linear(w, x_bits)


def test_static_scratch_linear_two_calls_in_a_row():
    # 35 slabs: beyond what the kernel with final results takes, so the per-slab partial sums are used; the second
    # call is smaller in every dimension and finds the first call's partial sums still in the array
    for n_out, k_in, k_tok, seed in ((208, 8960, 8, 71), (40, 8704, 3, 72)):
        y, y_ref, y_oracle = _both(n_out, k_in, k_tok, seed)
        assert np.array_equal(y, y_ref), "same kernels, same order of the adds: bit-identical"
        assert ol.rel_l2(y, y_oracle) <= 1e-3


def test_static_scratch_linear_rejects_what_the_array_cannot_hold():
    limit = sd2.static_scratch_bytes()
    assert limit == 8 << 20
    w = wl.gen_weight(73, 0, "down", 1024, 8960, 50)
    mat = gu.SparseMat(w)
    k_tok = 64
    assert sd2.linear_workspace_size(mat.m, k_tok) > limit
    x = gu.dev(wl.gen_x(73, 0, "down", k_tok, 8960))
    y = torch.zeros((k_tok, 1024), dtype=torch.float32, device="cuda")
    with pytest.raises(sd2.SD2Error) as e:
        sd2.sparse_linear_static(mat.m, x.data_ptr(), k_tok, y.data_ptr(), gu.stream_ptr())
    assert e.value.status == -4
    torch.cuda.synchronize()
    assert float(y.abs().max()) == 0.0  # nothing was enqueued
