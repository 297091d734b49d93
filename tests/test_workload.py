import numpy as np
import pytest

import sd2_workload as wl


def test_bf16_rounding_known_values():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 0.0], dtype=np.float32)
    assert wl.f32_to_bf16_bits(x).tolist() == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC020, 0x0000]
    b = np.array([0x3F80, 0xC020, 0x0001], dtype=np.uint16)
    assert wl.bf16_bits_to_f32(b).tolist() == [1.0, -2.5, float(np.float32(2.0 ** -133))]


@pytest.mark.parametrize("k,pcts,expect", [
    (512, (50,), (256,)), (2048, (50,), (1024,)), (8192, (50,), (4096,)), (3072, (50,), (1536,)),
    (1536, (50, 60, 70), (768, 615, 461)), (8960, (50, 60, 70), (4480, 3584, 2688)),
    (1536, (66, 75), (523, 384)),
])
def test_keep_counts(k, pcts, expect):
    assert tuple(wl.n_keep(k, p) for p in pcts) == expect


def test_cfg1_mask_properties():
    w = wl.gen_weight(1, 0, "q", 512, 512, 50)
    nz = w != 0
    assert nz.sum() == 131072
    assert (nz.sum(1) == 256).all()
    dense = wl.gen_weight_dense(1, 0, "q", 512, 512)
    mag = (dense & 0x7FFF).astype(np.int32)
    kept_min = np.where(nz, mag, 1 << 20).min(1)
    pruned_max = np.where(~nz, mag, -1).max(1)
    assert (kept_min >= pruned_max).all()
    assert np.array_equal(w[nz], dense[nz])           # kept values untouched


def test_total_nnz_of_stacks_by_arithmetic():
    def total(shape, pct):
        return sum(n * wl.n_keep(k, pct) for _, _, n, k in wl.stack_matrices(shape))
    assert total(wl.CONFIGS[3]["shape"], 50) == 1409286144
    assert total(wl.CONFIGS[4]["shape"], 50) == 655097856
    mlp = 2 * 8192 * wl.n_keep(2048, 50) + 2048 * wl.n_keep(8192, 50)
    assert mlp == 25165824


def test_tie_rule_lowest_columns_kept():
    row = np.full((1, 64), 0x3C00, dtype=np.uint16)
    row[0, ::2] |= 0x8000                              # signs must not matter
    m = wl.magnitude_mask_per_row(row, 75)
    assert m[0, :16].all() and not m[0, 16:].any()
    row[0, 40] = 0x3C01                                # one larger magnitude jumps the queue
    m = wl.magnitude_mask_per_row(row, 75)
    assert m[0, 40] and m[0, :15].all() and m.sum() == 16 and not m[0, 15]


def test_global_pattern_is_unbalanced_but_same_density():
    w = wl.gen_weight(9, 0, "gate", 128, 256, 50, pattern="global")
    nz = w != 0
    assert nz.sum() == 128 * 256 // 2
    assert nz.sum(1).min() < 128 < nz.sum(1).max()


def test_determinism_and_stream_separation():
    a = wl.gen_weight(2, 0, "gate", 64, 128, 50)
    assert np.array_equal(a, wl.gen_weight(2, 0, "gate", 64, 128, 50))
    assert not np.array_equal(a, wl.gen_weight(2, 0, "up", 64, 128, 50))
    assert not np.array_equal(a, wl.gen_weight(2, 1, "gate", 64, 128, 50))
    x = wl.gen_x(2, 0, "gate", 5, 128)
    assert x.shape == (5, 128) and x.dtype == np.uint16


def test_verify_inputs():
    d, t = wl.gen_verify(5, 4096, 5, 128256, 0.85)
    assert d.shape == (4096, 5) and t.shape == (4096, 6) and d.dtype == np.int32
    assert d.min() >= 0 and d.max() < 128256 and t.min() >= 0 and t.max() < 128256
    frac = (d == t[:, :5]).mean()
    assert abs(frac - 0.85) < 0.01


def test_stack_shapes():
    s = wl.CONFIGS[3]["shape"]
    per_layer = sum(n * k for _, n, k in wl.layer_matrix_shapes(s))
    assert per_layer == 100663296
    assert s.n_heads * s.head_dim == s.q_out and s.n_kv * s.head_dim == s.kv_out
    q = wl.CONFIGS[4]["shape"]
    assert q.n_heads * q.head_dim == q.q_out and q.n_kv * q.head_dim == q.kv_out
    assert len(list(wl.stack_matrices(s))) == 196
