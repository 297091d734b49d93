// Host side of libsd2, format 3: the 2:4 semi-structured blob (docs/FORMAT.md, "Format 3").
// The paper evaluates 2:4 drafters next to unstructured ones (Sec. 3, Sec. 3.3); a tile here is
// already the operand layout of the structured-sparse matrix instruction, so the device side
// needs no decode at all.
#include <string.h>

#include "sd2_format.h"

namespace sd2 {

static inline bool present(uint16_t b) { return (b & 0x7FFFu) != 0; }
static inline uint32_t group_of(uint32_t a, uint32_t p) { return 8 * (a & 1) + 2 * (a >> 1) + 4 * (p >> 1) + (p & 1); }

int nm24_fill_geometry(int32_t n_out, int32_t k_in, Header* h) {
    if (n_out < 1 || k_in < 64 || (k_in % 64) != 0) return SD2_ERR_SHAPE;
    if ((uint64_t)n_out * (uint64_t)k_in > (1ull << 36)) return SD2_ERR_SHAPE;
    memset(h, 0, sizeof(*h));
    h->magic = kMagic;
    h->version = kVersion;
    h->format = SD2_FORMAT_NM24;
    h->n_out = (uint32_t)n_out;
    h->k_in = (uint32_t)k_in;
    h->n_strips = ceil_div(h->n_out, kStripRows);
    h->n_slabs = ceil_div(h->k_in, kSlabCols);
    h->n_tiles = h->n_strips * h->n_slabs;
    h->dir_off = 0;
    h->mask_off = 0;
    h->val_off = kHeaderBytes;
    h->total_bytes = kHeaderBytes + (uint64_t)kNm24TileBytes * h->n_tiles;
    h->useful_bytes = 9ull * h->n_out * h->k_in / 8;
    return SD2_OK;
}

// Counts always, writes the tiles when `out` is given.  SD2_ERR_FORMAT if a group holds more than two values.
int nm24_walk(const uint16_t* w, Header* h, uint8_t* out) {
    uint64_t nnz = 0;
    uint32_t max_nnz = 0;
    for (uint32_t slab = 0; slab < h->n_slabs; ++slab)
        for (uint32_t strip = 0; strip < h->n_strips; ++strip) {
            const uint32_t t = slab * h->n_strips + strip;
            uint8_t* tile = out ? out + h->val_off + (size_t)kNm24TileBytes * t : nullptr;
            uint32_t n_t = 0;
            for (uint32_t l = 0; l < 64; ++l) {
                const uint32_t row = kStripRows * strip + (l & 15), a = l >> 4;
                uint64_t idx = 0;
                for (uint32_t q = 0; q < 4; ++q)
                    for (uint32_t p = 0; p < 4; ++p) {
                        const uint32_t col = kSlabCols * slab + 64 * q + 4 * group_of(a, p);
                        uint16_t v[4] = {0, 0, 0, 0};
                        if (row < h->n_out && col < h->k_in) memcpy(v, w + (size_t)row * h->k_in + col, 8);
                        uint32_t nz[4], n = 0;
                        for (uint32_t c = 0; c < 4; ++c)
                            if (present(v[c])) nz[n++] = c;
                        if (n > 2) return SD2_ERR_FORMAT;
                        uint32_t c0 = 0, c1 = 1;
                        if (n == 2) {
                            c0 = nz[0];
                            c1 = nz[1];
                        } else if (n == 1 && nz[0] != 0) {
                            c1 = nz[0];
                        }
                        n_t += n;
                        idx |= ((uint64_t)c0 << (16 * q + 4 * p)) | ((uint64_t)c1 << (16 * q + 4 * p + 2));
                        if (tile) {
                            const uint16_t s0 = present(v[c0]) ? v[c0] : (uint16_t)0, s1 = present(v[c1]) ? v[c1] : (uint16_t)0;
                            uint8_t* dst = tile + (size_t)(64 * q + l) * 16 + 4 * p;
                            memcpy(dst, &s0, 2);
                            memcpy(dst + 2, &s1, 2);
                        }
                    }
                if (tile) memcpy(tile + 4096 + 8 * l, &idx, 8);
            }
            nnz += n_t;
            if (n_t > max_nnz) max_nnz = n_t;
        }
    h->nnz = nnz;
    h->max_tile_nnz = max_nnz;
    return SD2_OK;
}

// Header fields of a format-3 blob against its geometry (the caller has checked magic, version and format).
int nm24_check_header(const Header* h, size_t blob_bytes) {
    Header g;
    if (h->n_out > 0x7fffffffu || h->k_in > 0x7fffffffu ||
        nm24_fill_geometry((int32_t)h->n_out, (int32_t)h->k_in, &g) != SD2_OK)
        return SD2_ERR_BLOB;
    if (g.n_strips != h->n_strips || g.n_slabs != h->n_slabs || g.n_tiles != h->n_tiles || h->dir_off != 0 ||
        h->mask_off != 0 || g.val_off != h->val_off || g.total_bytes != h->total_bytes ||
        g.useful_bytes != h->useful_bytes)
        return SD2_ERR_BLOB;
    if (h->total_bytes > blob_bytes) return SD2_ERR_BLOB;
    if (h->nnz > (uint64_t)h->n_out * h->k_in / 2 || h->max_tile_nnz > 2048 || h->max_tile_nnz > h->nnz) return SD2_ERR_BLOB;
    if (h->zero0) return SD2_ERR_BLOB;
    for (int i = 0; i < 9; ++i)
        if (h->zero[i]) return SD2_ERR_BLOB;
    return SD2_OK;
}

// Checks every group (ascending stored columns, nothing outside the matrix, counts) and, when w_out is given,
// writes the matrix.
int nm24_decode(const void* blob, const Header& h, uint16_t* w_out) {
    const uint8_t* p = static_cast<const uint8_t*>(blob);
    if (w_out) memset(w_out, 0, (size_t)h.n_out * h.k_in * 2);
    uint64_t nnz = 0;
    uint32_t max_nnz = 0;
    for (uint32_t t = 0; t < h.n_tiles; ++t) {
        const uint32_t strip = t % h.n_strips, slab = t / h.n_strips;
        const uint8_t* tile = p + h.val_off + (size_t)kNm24TileBytes * t;
        uint32_t n_t = 0;
        for (uint32_t l = 0; l < 64; ++l) {
            const uint32_t row = kStripRows * strip + (l & 15), a = l >> 4;
            uint64_t idx;
            memcpy(&idx, tile + 4096 + 8 * l, 8);
            for (uint32_t q = 0; q < 4; ++q)
                for (uint32_t pp = 0; pp < 4; ++pp) {
                    const uint32_t c0 = (uint32_t)(idx >> (16 * q + 4 * pp)) & 3u, c1 = (uint32_t)(idx >> (16 * q + 4 * pp + 2)) & 3u;
                    if (c0 >= c1) return SD2_ERR_BLOB;
                    uint16_t s[2];
                    memcpy(s, tile + (size_t)(64 * q + l) * 16 + 4 * pp, 4);
                    const uint32_t col = kSlabCols * slab + 64 * q + 4 * group_of(a, pp);
                    for (uint32_t j = 0; j < 2; ++j) {
                        if (!present(s[j])) {
                            if (s[j] != 0) return SD2_ERR_BLOB;  // a padding entry is +0
                            continue;
                        }
                        const uint32_t c = col + (j ? c1 : c0);
                        if (row >= h.n_out || c >= h.k_in) return SD2_ERR_BLOB;
                        if (w_out) w_out[(size_t)row * h.k_in + c] = s[j];
                        ++n_t;
                    }
                }
        }
        nnz += n_t;
        if (n_t > max_nnz) max_nnz = n_t;
    }
    if (nnz != h.nnz || max_nnz != h.max_tile_nnz) return SD2_ERR_BLOB;
    return SD2_OK;
}

}  // namespace sd2
