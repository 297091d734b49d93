"""Format 3 (2:4 semi-structured): the mask generator, the reference packer written from docs/FORMAT.md, and the
library's packer against it.  The 2:4 pattern is the one the paper evaluates next to unstructured sparsity (Sec. 3)."""
import numpy as np
import pytest

import paper_2504_08838_amd as sd2
import sd2_workload as wl
from oracle import pack_ref as pr

NM24 = 3


def _w(n, k, seed=41):
    return wl.gen_weight(seed, 0, "q", n, k, 50, pattern="2:4")


def test_mask_keeps_the_two_largest_of_every_four():
    w = wl.gen_weight_dense(41, 0, "q", 64, 256)
    m = wl.mask_2of4(w)
    assert (m.reshape(64, 64, 4).sum(-1) == 2).all()
    mag = (w & 0x7FFF).astype(np.int32).reshape(64, 64, 4)
    kept_min = np.where(m.reshape(64, 64, 4), mag, 1 << 20).min(-1)
    pruned_max = np.where(m.reshape(64, 64, 4), -1, mag).max(-1)
    assert (kept_min >= pruned_max).all()


def test_mask_tie_rule_lowest_columns_win():
    w = np.full((2, 8), 0x3C00, dtype=np.uint16)  # all equal magnitudes
    m = wl.mask_2of4(w)
    assert m.tolist() == [[True, True, False, False] * 2] * 2
    w[0, 3] = 0x4000  # one larger value: it and the lowest of the rest
    assert wl.mask_2of4(w)[0, :4].tolist() == [True, False, False, True]


@pytest.mark.parametrize("n,k", [(16, 64), (40, 320), (33, 256), (100, 768), (7, 64)])
def test_reference_round_trip_and_header(n, k):
    w = _w(n, k)
    blob = pr.pack24(w)
    h = pr.header(blob)
    assert h["format"] == NM24 and h["n_out"] == n and h["k_in"] == k
    assert h["total_bytes"] == 128 + 4608 * h["n_tiles"] == blob.size
    assert h["useful_bytes"] == 9 * n * k // 8 and h["nnz"] == n * k // 2
    assert np.array_equal(pr.unpack24(blob), w)


def test_groups_with_fewer_than_two_values_and_minus_zero():
    w = _w(32, 256)
    w[:, ::3] = 0            # many groups now hold one value or none
    w[5, 8:12] = 0x8000      # a group of minus zeros: stored as an empty group
    blob = pr.pack24(w)
    expect = np.where((w & 0x7FFF) != 0, w, 0).astype(np.uint16)
    assert np.array_equal(pr.unpack24(blob), expect)
    # stored columns of a one-value group: {0,1} when the value sits in column 0, else {0,c}
    one = np.zeros((16, 64), dtype=np.uint16)
    one[0, 0], one[1, 5], one[2, 11] = 0x3F80, 0x3F80, 0x3F80
    b = pr.pack24(one)
    idx = b[128 + 4096:128 + 4608].view("<u8")
    # row r is lane r (a = 0); groups 0, 1 are p = 0, 1 of step 0; group 2 belongs to lane 32 + r (a = 2, p = 0)
    assert (int(idx[0]) >> 0) & 15 == 0b0100          # (0, 1)
    assert (int(idx[1]) >> 4) & 15 == 0b0100          # column 5 = group 1, c = 1 -> (0, 1)
    assert (int(idx[34]) >> 0) & 15 == 0b1100         # column 11 = group 2, c = 3 -> (0, 3)


def test_not_2of4_is_rejected():
    w = wl.gen_weight_dense(41, 0, "q", 16, 64)
    with pytest.raises(ValueError):
        pr.pack24(w)
    with pytest.raises(sd2.SD2Error) as e:
        sd2.pack_sparse(w, NM24)
    assert e.value.status == -3


@pytest.mark.parametrize("n,k", [(16, 64), (40, 320), (33, 256), (100, 768), (7, 64), (512, 1536)])
def test_library_packer_is_byte_identical_to_the_reference(n, k):
    w = _w(n, k, seed=42)
    if n == 40:
        w[:, ::5] = 0
    ref = pr.pack24(w)
    blob = sd2.pack_sparse(w, NM24)
    assert blob.size == ref.size == sd2.pack_sparse_size(w, NM24)
    assert np.array_equal(blob, ref)
    sd2.blob_validate(blob)
    info = sd2.blob_info(blob)
    assert info.format == NM24 and info.nnz == int(((w & 0x7FFF) != 0).sum())
    assert np.array_equal(sd2.unpack_sparse(blob, n, k), np.where((w & 0x7FFF) != 0, w, 0))


def test_corrupt_blobs_are_rejected():
    w = _w(32, 256)
    blob = sd2.pack_sparse(w, NM24)
    bad = blob.copy()
    bad[128 + 4096] ^= 0x0F  # stored columns of lane 0, groups 0: now descending or equal
    with pytest.raises(sd2.SD2Error):
        sd2.blob_validate(bad)
    with pytest.raises(sd2.SD2Error):
        sd2.blob_info(blob[:-1])  # truncated
    short = blob.copy()
    short[72:80] = np.frombuffer(np.uint64(blob.size + 16).tobytes(), dtype=np.uint8)  # total_bytes too large
    with pytest.raises(sd2.SD2Error):
        sd2.blob_info(short)


def test_auto_never_chooses_format_3():
    w = _w(16, 64)
    assert sd2.blob_info(sd2.pack_sparse(w, 0)).format == 1
