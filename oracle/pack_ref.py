"""Reference packer/unpacker for the SD2B blob, written from docs/FORMAT.md alone.

Second, independent implementation of the byte format: the library's C++
packer must produce the same bytes.  The sparse representation itself is not
specified by the paper (Sec. 1 and Sec. 3.3 only say that a compressed
representation and its metadata are needed); the layout is this build's.
"""

import numpy as np

MAGIC = 0x42324453
HEADER = 128
DIR_ENTRY = 48


def _ceil_div(a, b):
    return -(-a // b)


def checksum(payload: np.ndarray) -> int:
    w = np.frombuffer(payload.tobytes(), dtype="<u4").astype(np.uint64)
    s1 = int(w.sum(dtype=np.uint64)) & 0xFFFFFFFF
    idx = np.arange(1, w.size + 1, dtype=np.uint64)
    s2 = int((w * idx).sum(dtype=np.uint64)) & 0xFFFFFFFF
    rot = ((s2 << 16) | (s2 >> 16)) & 0xFFFFFFFF
    return s1 ^ rot


def _tile_view(a, n_strips, n_slabs):
    """[n_strips*16][n_slabs*256] -> axes (slab, strip, q, g, i, h, c): g = lane div 16, i = lane mod 16."""
    a = a.reshape(n_strips, 16, n_slabs, 4, 4, 4, 4)  # strip i slab q g h c
    return a.transpose(2, 0, 3, 4, 1, 5, 6)  # slab strip q g i h c


def pack(w_bits: np.ndarray) -> np.ndarray:
    """Return the blob (numpy uint8) for bf16 bit matrix ``w_bits`` [n_out][k_in]."""
    w_bits = np.ascontiguousarray(w_bits, dtype=np.uint16)
    n_out, k_in = w_bits.shape
    if n_out < 1 or k_in < 64 or k_in % 64:
        raise ValueError("k_in must be a positive multiple of 64")
    n_strips, n_slabs = _ceil_div(n_out, 16), _ceil_div(k_in, 256)
    n_tiles = n_strips * n_slabs

    wp = np.zeros((n_strips * 16, n_slabs * 256), dtype=np.uint16)
    wp[:n_out, :k_in] = w_bits
    present = (wp & np.uint16(0x7FFF)) != 0
    pv = _tile_view(present, n_strips, n_slabs)  # slab strip q g i h c
    wv = _tile_view(wp, n_strips, n_slabs)

    # masks: lane l = g*16 + i, word q, bit b = 4h + c
    weights = (np.uint32(1) << np.arange(16, dtype=np.uint32)).reshape(4, 4)
    words = (pv.astype(np.uint32) * weights).sum(axis=(-1, -2)).astype("<u2")  # slab strip q g i
    masks = np.ascontiguousarray(words.transpose(0, 1, 3, 4, 2))  # slab strip g i q

    # value stream order inside a tile: (q, h, l = (g, i), c)
    order = (0, 1, 2, 5, 3, 4, 6)  # slab strip q h g i c
    pt = np.ascontiguousarray(pv.transpose(order)).reshape(n_tiles, 16, 256)  # tile, run (q,h), lane*4+c
    wt = np.ascontiguousarray(wv.transpose(order)).reshape(n_tiles, 16, 256)
    run_nnz = pt.sum(axis=2, dtype=np.int64)  # [tile][16]
    nnz_t = run_nnz.sum(axis=1)
    base = np.cumsum(run_nnz, axis=1) - run_nnz
    padded = _ceil_div(nnz_t, 8) * 8
    starts = np.concatenate([[0], np.cumsum(padded // 8)])
    vals = np.zeros(int(padded.sum()) + 8, dtype="<u2")
    flat_p = pt.reshape(n_tiles, -1)
    flat_w = wt.reshape(n_tiles, -1)
    for t in range(n_tiles):
        s = int(starts[t]) * 8
        vals[s:s + int(nnz_t[t])] = flat_w[t][flat_p[t]]

    directory = np.zeros((n_tiles, DIR_ENTRY), dtype=np.uint8)
    directory[:, 0:4] = starts[:-1].astype("<u4").reshape(-1, 1).view(np.uint8)
    directory[:, 4:8] = nnz_t.astype("<u4").reshape(-1, 1).view(np.uint8)
    directory[:, 8:40] = np.ascontiguousarray(base.astype("<u2")).view(np.uint8)

    dir_off = HEADER
    mask_off = dir_off + DIR_ENTRY * n_tiles
    val_off = mask_off + 512 * n_tiles
    total = val_off + vals.nbytes
    nnz = int(nnz_t.sum())
    payload = np.concatenate([directory.reshape(-1), masks.reshape(-1).view(np.uint8), vals.view(np.uint8)])
    assert payload.size == total - HEADER

    hdr = np.zeros(HEADER, dtype=np.uint8)
    h32 = hdr.view("<u4")
    h32[0:9] = [MAGIC, 2, 1, n_out, k_in, n_strips, n_slabs, n_tiles, int(nnz_t.max())]
    h64 = hdr.view("<u8")
    h64[5] = nnz
    h64[6] = dir_off
    h64[7] = mask_off
    h64[8] = val_off
    h64[9] = total
    h64[10] = 2 * nnz + (n_out * k_in) // 8
    h32[22] = checksum(payload)
    return np.concatenate([hdr, payload])


def header(blob: np.ndarray) -> dict:
    b = np.ascontiguousarray(blob, dtype=np.uint8)
    h32 = b[:HEADER].view("<u4")
    h64 = b[:HEADER].view("<u8")
    names = ["magic", "version", "format", "n_out", "k_in", "n_strips", "n_slabs", "n_tiles", "max_tile_nnz"]
    d = {n: int(h32[i]) for i, n in enumerate(names)}
    d.update(nnz=int(h64[5]), dir_off=int(h64[6]), mask_off=int(h64[7]), val_off=int(h64[8]),
             total_bytes=int(h64[9]), useful_bytes=int(h64[10]), checksum=int(h32[22]))
    return d


def decode_entries(blob: np.ndarray):
    """Walk the blob position by position (slow, literal): -> rows, cols, value bits in stream order."""
    b = np.ascontiguousarray(blob, dtype=np.uint8)
    h = header(b)
    if h["magic"] != MAGIC or h["version"] != 2 or h["format"] != 1:
        raise ValueError("not an SD2B v2 bitmask blob")
    n_strips = h["n_strips"]
    directory = b[h["dir_off"]:h["mask_off"]].reshape(h["n_tiles"], DIR_ENTRY)
    masks = b[h["mask_off"]:h["val_off"]].view("<u2").reshape(h["n_tiles"], 64, 4)
    vals = b[h["val_off"]:h["total_bytes"]].view("<u2")
    rows, cols, bits = [], [], []
    for t in range(h["n_tiles"]):
        slab, strip = divmod(t, n_strips)
        start = int(directory[t, 0:4].view("<u4")[0]) * 8
        nnz_t = int(directory[t, 4:8].view("<u4")[0])
        base = directory[t, 8:40].view("<u2")
        p = start
        for q in range(4):
            for hh in range(4):
                if p - start != int(base[4 * q + hh]):
                    raise ValueError("run base disagrees with masks")
                for l in range(64):
                    nib = (int(masks[t, l, q]) >> (4 * hh)) & 15
                    for c in range(4):
                        if nib >> c & 1:
                            rows.append(16 * strip + (l % 16))
                            cols.append(256 * slab + 64 * q + 16 * (l // 16) + 4 * hh + c)
                            bits.append(int(vals[p]))
                            p += 1
        if p - start != nnz_t:
            raise ValueError("directory nnz disagrees with masks")
    return (np.array(rows, dtype=np.int64), np.array(cols, dtype=np.int64),
            np.array(bits, dtype=np.uint16))


def unpack(blob: np.ndarray) -> np.ndarray:
    h = header(blob)
    rows, cols, bits = decode_entries(blob)
    w = np.zeros((h["n_out"], h["k_in"]), dtype=np.uint16)
    w[rows, cols] = bits
    return w


# --------------------------------------------------------------------------- format 3: 2:4 semi-structured
# Written from the "Format 3" section of docs/FORMAT.md alone.

TILE24 = 4608


def _group_of(a: int, p: int) -> int:
    return 8 * (a % 2) + 2 * (a // 2) + 4 * (p // 2) + (p % 2)


def _stored_pair(nz):
    """Columns (c0 < c1) a group stores, given the sorted list of its non-zero columns."""
    if len(nz) > 2:
        raise ValueError("matrix is not 2:4")
    if len(nz) == 2:
        return nz[0], nz[1]
    if len(nz) == 0:
        return 0, 1
    return (0, 1) if nz[0] == 0 else (0, nz[0])


def pack24(w_bits: np.ndarray) -> np.ndarray:
    """Blob of format 3 for a 2:4 matrix (literal loops over groups vectorised over rows)."""
    w_bits = np.ascontiguousarray(w_bits, dtype=np.uint16)
    n_out, k_in = w_bits.shape
    if n_out < 1 or k_in < 64 or k_in % 64:
        raise ValueError("k_in must be a positive multiple of 64")
    n_strips, n_slabs = _ceil_div(n_out, 16), _ceil_div(k_in, 256)
    n_tiles = n_strips * n_slabs
    wp = np.zeros((n_strips * 16, n_slabs * 256), dtype=np.uint16)
    wp[:n_out, :k_in] = w_bits
    grp = wp.reshape(n_strips * 16, n_slabs * 64, 4)
    nzm = (grp & np.uint16(0x7FFF)) != 0
    cnt = nzm.sum(axis=-1)
    if (cnt > 2).any():
        raise ValueError("matrix is not 2:4")
    # stored columns per group from the table of the 11 admissible non-zero patterns
    c0 = np.zeros(cnt.shape, dtype=np.int64)
    c1 = np.ones(cnt.shape, dtype=np.int64)
    code = (nzm * np.array([1, 2, 4, 8])).sum(axis=-1)
    for pat in range(16):
        nz = [c for c in range(4) if pat >> c & 1]
        if len(nz) > 2:
            continue
        a, b = _stored_pair(nz)
        sel = code == pat
        c0[sel], c1[sel] = a, b
    v0 = np.take_along_axis(grp, c0[..., None], axis=-1)[..., 0]
    v1 = np.take_along_axis(grp, c1[..., None], axis=-1)[..., 0]
    v0 = np.where((v0 & np.uint16(0x7FFF)) != 0, v0, np.uint16(0))  # a stored column that is zero holds +0
    v1 = np.where((v1 & np.uint16(0x7FFF)) != 0, v1, np.uint16(0))

    payload = np.zeros((n_tiles, TILE24), dtype=np.uint8)
    vals = payload[:, :4096].view("<u2").reshape(n_tiles, 4, 64, 8)  # tile, q, lane, slot
    idx = np.zeros((n_tiles, 64), dtype=np.uint64)
    for slab in range(n_slabs):
        for strip in range(n_strips):
            t = slab * n_strips + strip
            rows = slice(16 * strip, 16 * strip + 16)
            for q in range(4):
                for a in range(4):
                    lanes = slice(16 * a, 16 * a + 16)  # lane = 16 a + (row mod 16)
                    for p in range(4):
                        g = 64 * slab + 16 * q + _group_of(a, p)
                        vals[t, q, lanes, 2 * p] = v0[rows, g]
                        vals[t, q, lanes, 2 * p + 1] = v1[rows, g]
                        idx[t, lanes] |= (c0[rows, g].astype(np.uint64) << np.uint64(16 * q + 4 * p)) | (
                            c1[rows, g].astype(np.uint64) << np.uint64(16 * q + 4 * p + 2))
    payload[:, 4096:] = idx.astype("<u8").view(np.uint8).reshape(n_tiles, 512)
    payload = payload.reshape(-1)

    nnz_tile = cnt.reshape(n_strips, 16, n_slabs, 64).sum(axis=(1, 3))
    nnz = int(cnt.sum())
    total = HEADER + TILE24 * n_tiles
    hdr = np.zeros(HEADER, dtype=np.uint8)
    h32 = hdr.view("<u4")
    h32[0:9] = [MAGIC, 2, 3, n_out, k_in, n_strips, n_slabs, n_tiles, int(nnz_tile.max())]
    h64 = hdr.view("<u8")
    h64[5] = nnz
    h64[6] = 0
    h64[7] = 0
    h64[8] = HEADER
    h64[9] = total
    h64[10] = 9 * n_out * k_in // 8
    h32[22] = checksum(payload)
    return np.concatenate([hdr, payload])


def unpack24(blob: np.ndarray) -> np.ndarray:
    """Position by position (slow, literal)."""
    b = np.ascontiguousarray(blob, dtype=np.uint8)
    h = header(b)
    if h["magic"] != MAGIC or h["version"] != 2 or h["format"] != 3:
        raise ValueError("not a format-3 blob")
    n_out, k_in, n_strips = h["n_out"], h["k_in"], h["n_strips"]
    w = np.zeros((n_out, k_in), dtype=np.uint16)
    for t in range(h["n_tiles"]):
        slab, strip = divmod(t, n_strips)
        tile = b[HEADER + TILE24 * t:HEADER + TILE24 * (t + 1)]
        vals = tile[:4096].view("<u2").reshape(4, 64, 8)
        idx = tile[4096:].view("<u8")
        for q in range(4):
            for lane in range(64):
                row = 16 * strip + lane % 16
                for v in range(8):
                    c = (int(idx[lane]) >> (16 * q + 2 * v)) & 3
                    col = 256 * slab + 64 * q + 4 * _group_of(lane // 16, v // 2) + c
                    bits = int(vals[q, lane, v])
                    if bits & 0x7FFF:
                        if row >= n_out or col >= k_in:
                            raise ValueError("value outside the matrix")
                        w[row, col] = bits
    return w
