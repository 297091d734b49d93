// Byte layout of the SD2B blob (see docs/FORMAT.md) and small host helpers.
// Shared by the host packer and the device launch code of the library only.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "../../include/sd2.h"

namespace sd2 {

constexpr uint32_t kMagic = 0x42324453u;  // "SD2B"
constexpr uint32_t kVersion = 2;
constexpr size_t kHeaderBytes = 128;
constexpr int kStripRows = 16;       // rows of one MFMA tile
constexpr int kSlabCols = 256;       // columns of one tile = 4 super-steps of 64
constexpr int kTileMaskBytes = 512;  // 64 lanes x 4 x uint16
constexpr int kDirEntryBytes = 48;
constexpr int kNm24TileBytes = 4608;  // format 3: 4096 bytes of values + 512 bytes of column indices per tile

struct Header {
    uint32_t magic, version, format;
    uint32_t n_out, k_in, n_strips, n_slabs, n_tiles, max_tile_nnz, zero0;
    uint64_t nnz, dir_off, mask_off, val_off, total_bytes, useful_bytes;
    uint32_t checksum;
    uint32_t zero[9];
};
static_assert(sizeof(Header) == kHeaderBytes, "header must be 128 bytes");

struct DirEntry {
    uint32_t val_start;  // in 16-byte units from val_off
    uint32_t nnz;
    uint16_t base[16];   // values of the tile before run (q, h), index 4q + h
    uint32_t zero[2];
};
static_assert(sizeof(DirEntry) == kDirEntryBytes, "directory entry must be 48 bytes");

inline uint32_t ceil_div(uint32_t a, uint32_t b) { return (a + b - 1) / b; }
inline uint64_t round_up(uint64_t a, uint64_t b) { return (a + b - 1) / b * b; }

uint32_t checksum_words(const uint8_t* p, size_t bytes);
int parse_header(const void* blob, size_t blob_bytes, Header* h);
void info_from_header(const Header& h, sd2_blob_info_t* out);

// format 3 (2:4 semi-structured)
int nm24_fill_geometry(int32_t n_out, int32_t k_in, Header* h);
int nm24_walk(const uint16_t* w, Header* h, uint8_t* out);
int nm24_check_header(const Header* h, size_t blob_bytes);
int nm24_decode(const void* blob, const Header& h, uint16_t* w_out);

}  // namespace sd2
