"""The library's C++ packer against the oracle-side packer and the format's pins (no GPU needed)."""
import numpy as np
import pytest

import paper_2504_08838_amd as sd2
import sd2_workload as wl
from oracle import pack_ref

CASES = [(16, 64), (100, 192), (520, 832), (33, 1024), (512, 512)]


@pytest.mark.parametrize("n,k", CASES)
@pytest.mark.parametrize("pct", [50, 75, 0])
def test_byte_identical_to_reference_packer(n, k, pct):
    w = wl.gen_weight(12, 0, "q", n, k, pct)
    a = sd2.pack_sparse(w, 1)
    b = pack_ref.pack(w)
    assert a.tobytes() == b.tobytes()
    assert sd2.pack_sparse_size(w, 1) == b.size


@pytest.mark.parametrize("pattern,pct", [("row", 50), ("row", 70), ("global", 60), ("row", 0)])
def test_roundtrip_and_canonical_set(pattern, pct):
    w = wl.gen_weight(12, 1, "gate", 200, 448, pct, pattern=pattern)
    blob = sd2.pack_sparse(w)
    sd2.blob_validate(blob)
    assert np.array_equal(sd2.unpack_sparse(blob, 200, 448), w)
    rows, cols, bits = pack_ref.decode_entries(blob)     # independent decoder reads the C++ blob
    order = np.lexsort((cols, rows))
    rc = np.argwhere(w != 0)
    assert np.array_equal(rows[order], rc[:, 0]) and np.array_equal(cols[order], rc[:, 1])
    assert np.array_equal(bits[order], w[w != 0])
    info = sd2.blob_info(blob)
    assert info.nnz == int((w != 0).sum()) and info.total_bytes == blob.size
    assert info.useful_bytes == 2 * info.nnz + 200 * 448 // 8


def test_stress_patterns():
    w = wl.gen_weight(12, 2, "q", 70, 512, 50)
    w[3, :] = 0; w[16:32, :] = 0; w[:, 256:512] = 0; w[40, :256] = 0x3F80; w[5, 7] = 0x8000
    blob = sd2.pack_sparse(w, 1)
    assert blob.tobytes() == pack_ref.pack(w).tobytes()
    expect = w.copy(); expect[5, 7] = 0
    assert np.array_equal(sd2.unpack_sparse(blob, 70, 512), expect)


def test_geometry_and_overhead():
    w = wl.gen_weight(12, 5, "gate", 1024, 3072, 50)
    info = sd2.blob_info(sd2.pack_sparse(w))
    assert (info.n_strips, info.n_slabs, info.n_tiles) == (64, 12, 768)
    assert 2048 <= info.max_tile_nnz <= 2400
    # directory + padding cost about 1 % on top of values and mask bits
    assert info.total_bytes <= 1.02 * info.useful_bytes


def test_error_paths():
    w = wl.gen_weight(12, 3, "q", 32, 128, 50)
    E = sd2.SD2Error
    with pytest.raises(E) as e:
        sd2.pack_sparse(np.zeros((4, 100), dtype=np.uint16))
    assert e.value.status == -2                                   # k_in not a multiple of 64
    with pytest.raises(E) as e:
        sd2.pack_sparse(w, 2)
    assert e.value.status == -8                                   # index format reserved
    with pytest.raises(E) as e:
        sd2.pack_sparse(w, 7)
    assert e.value.status == -3
    with pytest.raises(E) as e:
        sd2.pack_sparse(w, 1, out=np.empty(64, dtype=np.uint8))
    assert e.value.status == -4
    blob = sd2.pack_sparse(w)
    with pytest.raises(E) as e:
        sd2.unpack_sparse(blob, 32, 192)
    assert e.value.status == -2
    assert sd2.lib().sd2_pack_sparse(None, 32, 128, 1, None, 0, None) == -1
    assert sd2.strerror(-5) == "corrupt blob" and sd2.strerror(0) == "ok"


def test_corruption_is_detected():
    w = wl.gen_weight(12, 4, "q", 64, 256, 50)
    blob = sd2.pack_sparse(w)
    E = sd2.SD2Error
    for pos in (0, 5, 13, 17, 21, 29, 33, 41, 49, 73, 95):                     # header fields
        b = blob.copy(); b[pos] ^= 0x40
        with pytest.raises(E):
            sd2.blob_validate(b)
    info = sd2.blob_info(blob)
    for pos in (130, int(info.mask_off) + 3, int(info.val_off) + 9, blob.size - 1):
        b = blob.copy(); b[pos] ^= 0x01
        with pytest.raises(E) as e:
            sd2.blob_validate(b)
        assert e.value.status == -5
    with pytest.raises(E):
        sd2.blob_validate(blob[:-16])                              # truncated
    with pytest.raises(E):
        sd2.blob_info(blob[:64])
