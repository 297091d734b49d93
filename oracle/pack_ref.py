"""Reference packer/unpacker for the SD2B blob, written from docs/FORMAT.md alone.

Second, independent implementation of the byte format: the library's C++
packer must produce the same bytes.  The sparse representation itself is not
specified by the paper (Sec. 1 and Sec. 3.3 only say that a compressed
representation and its metadata are needed); the layout is this build's.
"""

import numpy as np

MAGIC = 0x42324453
HEADER = 128


def _ceil_div(a, b):
    return -(-a // b)


def checksum(payload: np.ndarray) -> int:
    w = np.frombuffer(payload.tobytes(), dtype="<u4").astype(np.uint64)
    s1 = int(w.sum(dtype=np.uint64)) & 0xFFFFFFFF
    idx = np.arange(1, w.size + 1, dtype=np.uint64)
    s2 = int((w * idx).sum(dtype=np.uint64)) & 0xFFFFFFFF
    rot = ((s2 << 16) | (s2 >> 16)) & 0xFFFFFFFF
    return s1 ^ rot


def _tile_view(a, n_ur, R, n_uc, Mu):
    """[n_ur*R*16][n_uc*Mu*256] -> axes (uc, ur, m, r, q, g, i, b)."""
    a = a.reshape(n_ur, R, 16, n_uc, Mu, 4, 4, 16)  # ur r i uc m q g b
    return a.transpose(3, 0, 4, 1, 5, 6, 2, 7)  # uc ur m r q g i b


def pack(w_bits: np.ndarray, strips_per_unit: int, slabs_per_unit: int) -> np.ndarray:
    """Return the blob (numpy uint8) for bf16 bit matrix ``w_bits`` [n_out][k_in]."""
    w_bits = np.ascontiguousarray(w_bits, dtype=np.uint16)
    n_out, k_in = w_bits.shape
    if n_out < 1 or k_in < 64 or k_in % 64:
        raise ValueError("k_in must be a positive multiple of 64")
    R, Mu = int(strips_per_unit), int(slabs_per_unit)
    n_strips, n_slabs = _ceil_div(n_out, 16), _ceil_div(k_in, 256)
    n_ur, n_uc = _ceil_div(n_strips, R), _ceil_div(n_slabs, Mu)
    n_units = n_ur * n_uc
    rows_p, cols_p = n_ur * R * 16, n_uc * Mu * 256

    wp = np.zeros((rows_p, cols_p), dtype=np.uint16)
    wp[:n_out, :k_in] = w_bits
    present = (wp & np.uint16(0x7FFF)) != 0

    pv = _tile_view(present, n_ur, R, n_uc, Mu)  # uc ur m r q g i b
    wv = _tile_view(wp, n_ur, R, n_uc, Mu)

    # masks: per (uc, ur, m, r) block -> lane l = g*16+i -> 4 words q
    weights = (np.uint32(1) << np.arange(16, dtype=np.uint32))
    words = (pv.astype(np.uint32) * weights).sum(axis=-1).astype("<u2")  # uc ur m r q g i
    masks = np.ascontiguousarray(words.transpose(0, 1, 2, 3, 5, 6, 4))  # uc ur m r g i q

    # values: stream order (uc, ur | m, r, q, g, i, b)
    pu = np.ascontiguousarray(pv).reshape(n_units, -1)
    wu = np.ascontiguousarray(wv).reshape(n_units, -1)
    nnz_u = pu.sum(axis=1, dtype=np.int64)
    padded_u = _ceil_div(nnz_u, 8) * 8
    starts = np.concatenate([[0], np.cumsum(padded_u // 8)])
    n_val = int(padded_u.sum())
    vals = np.zeros(n_val + 8, dtype="<u2")
    for u in range(n_units):
        s = int(starts[u]) * 8
        vals[s:s + int(nnz_u[u])] = wu[u][pu[u]]

    directory = np.zeros((_ceil_div(8 * n_units, 16) * 16) // 4, dtype="<u4")
    directory[0:2 * n_units:2] = starts[:-1].astype(np.uint32)
    directory[1:2 * n_units:2] = nnz_u.astype(np.uint32)

    dir_off = HEADER
    mask_off = dir_off + directory.nbytes
    val_off = mask_off + 512 * R * Mu * n_units
    total = val_off + vals.nbytes
    nnz = int(nnz_u.sum())

    payload = np.concatenate([
        directory.view(np.uint8), masks.reshape(-1).view(np.uint8), vals.view(np.uint8)])
    assert payload.size == total - HEADER and masks.nbytes == 512 * R * Mu * n_units

    hdr = np.zeros(HEADER, dtype=np.uint8)
    h32 = hdr.view("<u4")
    h32[0:12] = [MAGIC, 1, 1, n_out, k_in, n_strips, n_slabs, R, Mu, n_ur, n_uc, n_units]
    h64 = hdr.view("<u8")
    h64[6] = nnz
    h64[7] = dir_off
    h64[8] = mask_off
    h64[9] = val_off
    h64[10] = total
    h64[11] = 2 * nnz + (n_out * k_in) // 8
    h32[24] = checksum(payload)
    return np.concatenate([hdr, payload])


def header(blob: np.ndarray) -> dict:
    b = np.ascontiguousarray(blob, dtype=np.uint8)
    h32 = b[:HEADER].view("<u4")
    h64 = b[:HEADER].view("<u8")
    names = ["magic", "version", "format", "n_out", "k_in", "n_strips", "n_slabs",
             "strips_per_unit", "slabs_per_unit", "n_unit_rows", "n_unit_cols", "n_units"]
    d = {n: int(h32[i]) for i, n in enumerate(names)}
    d.update(nnz=int(h64[6]), dir_off=int(h64[7]), mask_off=int(h64[8]), val_off=int(h64[9]),
             total_bytes=int(h64[10]), useful_bytes=int(h64[11]), checksum=int(h32[24]))
    return d


def decode_entries(blob: np.ndarray):
    """Walk the blob position by position (slow, literal): -> rows, cols, value bits in stream order."""
    b = np.ascontiguousarray(blob, dtype=np.uint8)
    h = header(b)
    if h["magic"] != MAGIC or h["version"] != 1 or h["format"] != 1:
        raise ValueError("not an SD2B v1 bitmask blob")
    R, Mu = h["strips_per_unit"], h["slabs_per_unit"]
    directory = b[h["dir_off"]:h["dir_off"] + 8 * h["n_units"]].view("<u4").reshape(-1, 2)
    masks = b[h["mask_off"]:h["val_off"]].view("<u2").reshape(h["n_units"], Mu, R, 64, 4)
    vals = b[h["val_off"]:h["total_bytes"]].view("<u2")
    rows, cols, bits = [], [], []
    for uc in range(h["n_unit_cols"]):
        for ur in range(h["n_unit_rows"]):
            u = uc * h["n_unit_rows"] + ur
            p = int(directory[u, 0]) * 8
            p0 = p
            for m in range(Mu):
                for r in range(R):
                    for q in range(4):
                        for l in range(64):
                            word = int(masks[u, m, r, l, q])
                            while word:
                                bit = (word & -word).bit_length() - 1
                                word &= word - 1
                                rows.append(16 * (ur * R + r) + (l % 16))
                                cols.append(256 * (uc * Mu + m) + 64 * q + 16 * (l // 16) + bit)
                                bits.append(int(vals[p]))
                                p += 1
            if p - p0 != int(directory[u, 1]):
                raise ValueError("directory nnz disagrees with masks")
    return (np.array(rows, dtype=np.int64), np.array(cols, dtype=np.int64),
            np.array(bits, dtype=np.uint16))


def unpack(blob: np.ndarray) -> np.ndarray:
    h = header(blob)
    rows, cols, bits = decode_entries(blob)
    w = np.zeros((h["n_out"], h["k_in"]), dtype=np.uint16)
    w[rows, cols] = bits
    return w
