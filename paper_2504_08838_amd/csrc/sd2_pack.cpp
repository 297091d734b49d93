// Host side of libsd2: packer, unpacker, blob checks.
// The sparse representation is this build's (the paper, Sec. 1 / Sec. 3.3, only asks
// for a compressed representation with little metadata); docs/FORMAT.md is normative.
#include <string.h>

#include "sd2_format.h"

namespace sd2 {

uint32_t checksum_words(const uint8_t* p, size_t bytes) {
    uint32_t s1 = 0, s2 = 0;
    size_t n = bytes / 4;
    for (size_t i = 0; i < n; ++i) {
        uint32_t w;
        memcpy(&w, p + 4 * i, 4);
        s1 += w;
        s2 += (uint32_t)(i + 1) * w;
    }
    return s1 ^ ((s2 << 16) | (s2 >> 16));
}

static int fill_geometry(int32_t n_out, int32_t k_in, Header* h) {
    if (n_out < 1 || k_in < 64 || (k_in % 64) != 0) return SD2_ERR_SHAPE;
    if ((uint64_t)n_out * (uint64_t)k_in > (1ull << 36)) return SD2_ERR_SHAPE;
    memset(h, 0, sizeof(*h));
    h->magic = kMagic;
    h->version = kVersion;
    h->format = SD2_FORMAT_BITMASK;
    h->n_out = (uint32_t)n_out;
    h->k_in = (uint32_t)k_in;
    h->n_strips = ceil_div(h->n_out, kStripRows);
    h->n_slabs = ceil_div(h->k_in, kSlabCols);
    h->n_tiles = h->n_strips * h->n_slabs;
    h->dir_off = kHeaderBytes;
    h->mask_off = h->dir_off + (uint64_t)kDirEntryBytes * h->n_tiles;
    h->val_off = h->mask_off + (uint64_t)kTileMaskBytes * h->n_tiles;
    return SD2_OK;
}

static inline bool present(uint16_t b) { return (b & 0x7FFFu) != 0; }

// Walks the tiles in stream order; counts always, writes when `out` is given.
static void walk(const uint16_t* w, Header* h, uint8_t* out) {
    DirEntry* dir = out ? reinterpret_cast<DirEntry*>(out + h->dir_off) : nullptr;
    uint16_t* masks = out ? reinterpret_cast<uint16_t*>(out + h->mask_off) : nullptr;
    uint16_t* vals = out ? reinterpret_cast<uint16_t*>(out + h->val_off) : nullptr;
    uint64_t nnz = 0, pos = 0;  // pos: value index (multiple of 8 at tile starts)
    uint32_t max_nnz = 0;
    for (uint32_t slab = 0; slab < h->n_slabs; ++slab) {
        for (uint32_t strip = 0; strip < h->n_strips; ++strip) {
            const uint32_t t = slab * h->n_strips + strip;
            const uint64_t start = pos;
            const uint32_t row0 = kStripRows * strip, col0 = kSlabCols * slab;
            uint16_t word[64][4];
            memset(word, 0, sizeof(word));
            DirEntry de;
            memset(&de, 0, sizeof(de));
            for (uint32_t q = 0; q < 4; ++q) {
                for (uint32_t hh = 0; hh < 4; ++hh) {
                    de.base[4 * q + hh] = (uint16_t)(pos - start);
                    for (uint32_t l = 0; l < 64; ++l) {
                        const uint32_t row = row0 + (l & 15);
                        const uint32_t c = col0 + 64 * q + 16 * (l >> 4) + 4 * hh;
                        if (row >= h->n_out || c >= h->k_in) continue;
                        const uint16_t* src = w + (size_t)row * h->k_in + c;
                        for (uint32_t b = 0; b < 4; ++b) {
                            if (present(src[b])) {
                                word[l][q] |= (uint16_t)(1u << (4 * hh + b));
                                if (vals) vals[pos] = src[b];
                                ++pos;
                            }
                        }
                    }
                }
            }
            const uint64_t n_t = pos - start;
            nnz += n_t;
            if (n_t > max_nnz) max_nnz = (uint32_t)n_t;
            const uint64_t padded = round_up(n_t, 8);
            if (vals)
                for (uint64_t i = pos; i < start + padded; ++i) vals[i] = 0;
            pos = start + padded;
            if (out) {
                de.val_start = (uint32_t)(start / 8);
                de.nnz = (uint32_t)n_t;
                memcpy(&dir[t], &de, sizeof(de));
                memcpy(masks + (size_t)t * 256, word, sizeof(word));
            }
        }
    }
    h->nnz = nnz;
    h->max_tile_nnz = max_nnz;
    h->total_bytes = h->val_off + 2 * pos + 16;
    h->useful_bytes = 2 * nnz + (uint64_t)h->n_out * h->k_in / 8;
}

int parse_header(const void* blob, size_t blob_bytes, Header* h) {
    if (!blob || !h) return SD2_ERR_NULL;
    if (blob_bytes < kHeaderBytes) return SD2_ERR_BLOB;
    memcpy(h, blob, sizeof(*h));
    if (h->magic != kMagic || h->version != kVersion) return SD2_ERR_BLOB;
    if (h->format == SD2_FORMAT_NM24) return nm24_check_header(h, blob_bytes);
    if (h->format != SD2_FORMAT_BITMASK) return SD2_ERR_FORMAT;
    Header g;
    if (h->n_out > 0x7fffffffu || h->k_in > 0x7fffffffu ||
        fill_geometry((int32_t)h->n_out, (int32_t)h->k_in, &g) != SD2_OK)
        return SD2_ERR_BLOB;
    if (g.n_strips != h->n_strips || g.n_slabs != h->n_slabs || g.n_tiles != h->n_tiles ||
        g.dir_off != h->dir_off || g.mask_off != h->mask_off || g.val_off != h->val_off)
        return SD2_ERR_BLOB;
    if (h->total_bytes > blob_bytes || h->total_bytes < h->val_off + 16 || (h->total_bytes % 16) != 0)
        return SD2_ERR_BLOB;
    if (h->nnz > (uint64_t)h->n_out * h->k_in || h->max_tile_nnz > 4096 || h->max_tile_nnz > h->nnz)
        return SD2_ERR_BLOB;
    if (h->useful_bytes != 2 * h->nnz + (uint64_t)h->n_out * h->k_in / 8) return SD2_ERR_BLOB;
    // the value section must hold every value plus per-tile padding and the 16-byte tail
    const uint64_t val_bytes = h->total_bytes - h->val_off - 16;
    if (val_bytes < 2 * h->nnz || val_bytes > 2 * h->nnz + 14ull * h->n_tiles) return SD2_ERR_BLOB;
    if (h->zero0) return SD2_ERR_BLOB;
    for (int i = 0; i < 9; ++i)
        if (h->zero[i]) return SD2_ERR_BLOB;
    return SD2_OK;
}

void info_from_header(const Header& h, sd2_blob_info_t* o) {
    memset(o, 0, sizeof(*o));
    o->format = (int32_t)h.format;
    o->n_out = (int32_t)h.n_out;
    o->k_in = (int32_t)h.k_in;
    o->n_strips = (int32_t)h.n_strips;
    o->n_slabs = (int32_t)h.n_slabs;
    o->n_tiles = (int32_t)h.n_tiles;
    o->max_tile_nnz = (int32_t)h.max_tile_nnz;
    o->nnz = h.nnz;
    o->total_bytes = h.total_bytes;
    o->useful_bytes = h.useful_bytes;
    o->mask_off = h.mask_off;
    o->val_off = h.val_off;
    o->checksum = h.checksum;
}

}  // namespace sd2

using namespace sd2;

extern "C" {

int sd2_pack_sparse_size(const uint16_t* w, int32_t n_out, int32_t k_in, int32_t format, size_t* bytes_out) {
    if (!w || !bytes_out) return SD2_ERR_NULL;
    if (format == SD2_FORMAT_INDEX16) return SD2_ERR_UNSUPPORTED;
    if (format == SD2_FORMAT_NM24) {
        Header h;
        int rc = nm24_fill_geometry(n_out, k_in, &h);
        if (rc != SD2_OK) return rc;
        if ((rc = nm24_walk(w, &h, nullptr)) != SD2_OK) return rc;
        *bytes_out = (size_t)h.total_bytes;
        return SD2_OK;
    }
    if (format != SD2_FORMAT_AUTO && format != SD2_FORMAT_BITMASK) return SD2_ERR_FORMAT;
    Header h;
    int rc = fill_geometry(n_out, k_in, &h);
    if (rc != SD2_OK) return rc;
    walk(w, &h, nullptr);
    *bytes_out = (size_t)h.total_bytes;
    return SD2_OK;
}

int sd2_pack_sparse(const uint16_t* w, int32_t n_out, int32_t k_in, int32_t format, void* blob, size_t blob_bytes,
                    size_t* bytes_written) {
    if (!w || !blob) return SD2_ERR_NULL;
    if (format == SD2_FORMAT_INDEX16) return SD2_ERR_UNSUPPORTED;
    if (format == SD2_FORMAT_NM24) {
        Header h;
        int rc = nm24_fill_geometry(n_out, k_in, &h);
        if (rc != SD2_OK) return rc;
        if ((rc = nm24_walk(w, &h, nullptr)) != SD2_OK) return rc;
        if (blob_bytes < h.total_bytes) return SD2_ERR_BUFFER;
        uint8_t* out = static_cast<uint8_t*>(blob);
        memset(out, 0, (size_t)h.total_bytes);
        nm24_walk(w, &h, out);
        h.checksum = checksum_words(out + kHeaderBytes, (size_t)(h.total_bytes - kHeaderBytes));
        memcpy(out, &h, sizeof(h));
        if (bytes_written) *bytes_written = (size_t)h.total_bytes;
        return SD2_OK;
    }
    if (format != SD2_FORMAT_AUTO && format != SD2_FORMAT_BITMASK) return SD2_ERR_FORMAT;
    Header h;
    int rc = fill_geometry(n_out, k_in, &h);
    if (rc != SD2_OK) return rc;
    walk(w, &h, nullptr);
    if (blob_bytes < h.total_bytes) return SD2_ERR_BUFFER;
    uint8_t* out = static_cast<uint8_t*>(blob);
    memset(out, 0, kHeaderBytes);
    walk(w, &h, out);
    memset(out + h.total_bytes - 16, 0, 16);
    h.checksum = checksum_words(out + kHeaderBytes, (size_t)(h.total_bytes - kHeaderBytes));
    memcpy(out, &h, sizeof(h));
    if (bytes_written) *bytes_written = (size_t)h.total_bytes;
    return SD2_OK;
}

int sd2_blob_info(const void* blob, size_t blob_bytes, sd2_blob_info_t* out) {
    if (!blob || !out) return SD2_ERR_NULL;
    Header h;
    int rc = parse_header(blob, blob_bytes, &h);
    if (rc != SD2_OK) return rc;
    info_from_header(h, out);
    return SD2_OK;
}

int sd2_blob_validate(const void* blob, size_t blob_bytes) {
    Header h;
    int rc = parse_header(blob, blob_bytes, &h);
    if (rc != SD2_OK) return rc;
    const uint8_t* p = static_cast<const uint8_t*>(blob);
    if (checksum_words(p + kHeaderBytes, (size_t)(h.total_bytes - kHeaderBytes)) != h.checksum)
        return SD2_ERR_BLOB;
    if (h.format == SD2_FORMAT_NM24) return nm24_decode(blob, h, nullptr);
    const DirEntry* dir = reinterpret_cast<const DirEntry*>(p + h.dir_off);
    const uint16_t* masks = reinterpret_cast<const uint16_t*>(p + h.mask_off);
    uint64_t next = 0, nnz = 0;
    uint32_t max_nnz = 0;
    for (uint32_t t = 0; t < h.n_tiles; ++t) {
        const uint16_t* tm = masks + (size_t)t * 256;
        const uint32_t strip = t % h.n_strips, slab = t / h.n_strips;
        uint32_t run = 0;
        for (uint32_t q = 0; q < 4; ++q)
            for (uint32_t hh = 0; hh < 4; ++hh) {
                if (dir[t].base[4 * q + hh] != run) return SD2_ERR_BLOB;
                for (uint32_t l = 0; l < 64; ++l) {
                    const uint32_t nib = (tm[l * 4 + q] >> (4 * hh)) & 15u;
                    run += (uint32_t)__builtin_popcount(nib);
                    // a set bit must lie inside the matrix (ragged last strip or slab)
                    const uint32_t row = kStripRows * strip + (l & 15);
                    const uint32_t c = kSlabCols * slab + 64 * q + 16 * (l >> 4) + 4 * hh;
                    if (nib && (row >= h.n_out || c + (31u - (uint32_t)__builtin_clz(nib)) >= h.k_in)) return SD2_ERR_BLOB;
                }
            }
        if (dir[t].nnz != run || dir[t].val_start != next || dir[t].zero[0] || dir[t].zero[1]) return SD2_ERR_BLOB;
        next += round_up(run, 8) / 8;
        nnz += run;
        if (run > max_nnz) max_nnz = run;
    }
    if (nnz != h.nnz || max_nnz != h.max_tile_nnz || h.val_off + 16 * next + 16 != h.total_bytes) return SD2_ERR_BLOB;
    return SD2_OK;
}

int sd2_unpack_sparse(const void* blob, size_t blob_bytes, uint16_t* w_out, int32_t n_out, int32_t k_in) {
    if (!w_out) return SD2_ERR_NULL;
    int rc = sd2_blob_validate(blob, blob_bytes);
    if (rc != SD2_OK) return rc;
    Header h;
    parse_header(blob, blob_bytes, &h);
    if ((uint32_t)n_out != h.n_out || (uint32_t)k_in != h.k_in) return SD2_ERR_SHAPE;
    if (h.format == SD2_FORMAT_NM24) return nm24_decode(blob, h, w_out);
    const uint8_t* p = static_cast<const uint8_t*>(blob);
    const DirEntry* dir = reinterpret_cast<const DirEntry*>(p + h.dir_off);
    const uint16_t* masks = reinterpret_cast<const uint16_t*>(p + h.mask_off);
    const uint16_t* vals = reinterpret_cast<const uint16_t*>(p + h.val_off);
    memset(w_out, 0, (size_t)n_out * k_in * 2);
    for (uint32_t t = 0; t < h.n_tiles; ++t) {
        const uint32_t strip = t % h.n_strips, slab = t / h.n_strips;
        const uint16_t* tm = masks + (size_t)t * 256;
        uint64_t pos = (uint64_t)dir[t].val_start * 8;
        for (uint32_t q = 0; q < 4; ++q)
            for (uint32_t hh = 0; hh < 4; ++hh)
                for (uint32_t l = 0; l < 64; ++l) {
                    const uint32_t nib = (tm[l * 4 + q] >> (4 * hh)) & 15u;
                    const uint32_t row = kStripRows * strip + (l & 15);
                    const uint32_t c = kSlabCols * slab + 64 * q + 16 * (l >> 4) + 4 * hh;
                    for (uint32_t b = 0; b < 4; ++b)
                        if ((nib >> b) & 1u) {
                            if (row >= h.n_out || c + b >= h.k_in) return SD2_ERR_BLOB;
                            w_out[(size_t)row * h.k_in + c + b] = vals[pos++];
                        }
                }
    }
    return SD2_OK;
}

}  // extern "C"
