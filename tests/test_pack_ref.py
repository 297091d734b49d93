"""Bit-exactness pins for the packed format, on the oracle-side packer."""
import numpy as np
import pytest

import sd2_workload as wl
from oracle import pack_ref


def _canonical(w):
    nz = (w & 0x7FFF) != 0
    rc = np.argwhere(nz)
    return rc[:, 0], rc[:, 1], w[nz]


@pytest.mark.parametrize("n,k", [(16, 64), (100, 192), (520, 832), (33, 1024)])
def test_decoded_set_is_canonical(n, k):
    w = wl.gen_weight(12, 0, "q", n, k, 50)
    blob = pack_ref.pack(w)
    rows, cols, bits = pack_ref.decode_entries(blob)
    order = np.lexsort((cols, rows))
    r0, c0, b0 = _canonical(w)
    assert np.array_equal(rows[order], r0) and np.array_equal(cols[order], c0) and np.array_equal(bits[order], b0)
    assert np.array_equal(pack_ref.unpack(blob), w)


def test_header_sizes_and_offsets():
    w = wl.gen_weight(12, 1, "q", 100, 192, 50)
    h = pack_ref.header(pack_ref.pack(w))
    assert (h["n_strips"], h["n_slabs"], h["n_tiles"]) == (7, 1, 7)
    assert h["dir_off"] == 128 and h["mask_off"] == 128 + 48 * 7 and h["val_off"] == h["mask_off"] + 512 * 7
    assert h["nnz"] == int((w != 0).sum()) and h["useful_bytes"] == 2 * h["nnz"] + 100 * 192 // 8


def test_stress_patterns_roundtrip():
    w = wl.gen_weight(12, 2, "q", 70, 512, 50)
    w[3, :] = 0                       # empty row
    w[16:32, :] = 0                   # empty strip
    w[:, 256:512] = 0                 # empty slab
    w[40, :256] = 0x3F80              # fully dense row segment
    w[5, 7] = 0x8000                  # -0 is pruned and comes back as +0
    blob = pack_ref.pack(w)
    back = pack_ref.unpack(blob)
    expect = w.copy(); expect[5, 7] = 0
    assert np.array_equal(back, expect)
    assert pack_ref.header(blob)["nnz"] == int(((w & 0x7FFF) != 0).sum())


def test_zero_sparsity_gives_all_ones_masks():
    w = wl.gen_weight(12, 3, "q", 32, 256, 0)
    blob = pack_ref.pack(w)
    h = pack_ref.header(blob)
    masks = blob[h["mask_off"]:h["val_off"]]
    assert (masks == 0xFF).all()
    vals = blob[h["val_off"]:h["total_bytes"] - 16].view("<u2")
    # stream order within a tile: super-step, nibble, lane (= 16 * (col group) + row), column in nibble
    t = w[:16].reshape(16, 4, 4, 4, 4).transpose(1, 3, 2, 0, 4).reshape(-1)   # row q g h c -> q h g row c
    assert np.array_equal(vals[:t.size], t)
    d = blob[h["dir_off"]:h["dir_off"] + 48]
    assert d[8:40].view("<u2").tolist() == [256 * i for i in range(16)] and d[4:8].view("<u4")[0] == 4096


def test_value_run_padding_and_directory():
    w = np.zeros((16, 64), dtype=np.uint16)
    w[0, 0] = 0x3F80; w[1, 1] = 0x4000; w[2, 63] = 0x4040
    blob = pack_ref.pack(w)
    h = pack_ref.header(blob)
    d = blob[h["dir_off"]:h["dir_off"] + 48]
    assert d[0:8].view("<u4").tolist() == [0, 3]
    # runs: (q0,h0) holds cols 0..3 of every lane -> two values; the third sits in (q0,h3) of lane 48+2
    assert d[8:40].view("<u2").tolist() == [0, 2, 2, 2] + [3] * 12 and not d[40:].any()
    vals = blob[h["val_off"]:h["total_bytes"]].view("<u2")
    assert vals.size == 8 + 8 and vals[:3].tolist() == [0x3F80, 0x4000, 0x4040] and not vals[3:].any()
    masks = blob[h["mask_off"]:h["val_off"]].view("<u2").reshape(64, 4)
    assert masks[0, 0] == 1 and masks[1, 0] == 2 and masks[48 + 2, 0] == 0x8000 and masks.astype(bool).sum() == 3


def test_checksum_detects_changes():
    w = wl.gen_weight(12, 4, "q", 32, 128, 50)
    blob = pack_ref.pack(w)
    h = pack_ref.header(blob)
    assert pack_ref.checksum(blob[128:]) == h["checksum"]
    b2 = blob.copy(); b2[200] ^= 1
    assert pack_ref.checksum(b2[128:]) != h["checksum"]
    b3 = blob.copy(); b3[[300, 304]] = b3[[304, 300]]
    if not np.array_equal(b3, blob):
        assert pack_ref.checksum(b3[128:]) != h["checksum"]
