// Device-side helpers shared by the gfx950 kernels of libsd2 (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sd2 {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct __attribute__((packed, aligned(4))) Tri32 {
    uint32_t a, b, c;
};

union Frag {
    uint32_t u[4];
    u32x4 q;
    bf16x8 v;
};

// Directory entry of one tile as stored in the blob.
struct DirEnt {
    uint32_t val_start;  // 16-byte units from the start of the value section
    uint32_t nnz;
    uint32_t base[8];    // 16 x uint16: values of the tile before run (q, h)
    uint32_t zero[2];
};

constexpr int kWavesPerBlock = 4;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round to nearest, ties to even (finite inputs)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// inclusive prefix sum over the 64 lanes of a wavefront
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x) {
    x += __builtin_amdgcn_update_dpp(0u, x, 0x111, 0xf, 0xf, true);  // row_shr:1
    x += __builtin_amdgcn_update_dpp(0u, x, 0x112, 0xf, 0xf, true);  // row_shr:2
    x += __builtin_amdgcn_update_dpp(0u, x, 0x114, 0xf, 0xf, true);  // row_shr:4
    x += __builtin_amdgcn_update_dpp(0u, x, 0x118, 0xf, 0xf, true);  // row_shr:8
    x += __builtin_amdgcn_update_dpp(0u, x, 0x142, 0xa, 0xf, true);  // row_bcast:15 -> rows 1,3
    x += __builtin_amdgcn_update_dpp(0u, x, 0x143, 0xc, 0xf, true);  // row_bcast:31 -> rows 2,3
    return x;
}

// exclusive prefix sum: shift the wave by one lane (lane 0 gets 0), then scan
__device__ __forceinline__ uint32_t wave_excl_scan(uint32_t x) {
    return wave_incl_scan(__builtin_amdgcn_update_dpp(0u, x, 0x138, 0xf, 0xf, true));  // wave_shr:1
}

// Byte-permute selectors that spread up to four compacted bf16 values over four columns.
// Entry [nib] = {selector for columns 0,1 ; selector for columns 2,3}; 0x0c yields a zero byte.
__device__ __forceinline__ uint2 make_expand_selector(uint32_t nib) {
    uint32_t sel[2] = {0u, 0u};
    uint32_t rank = 0;
    for (uint32_t p = 0; p < 4; ++p) {
        uint32_t lo = 0x0cu, hi = 0x0cu;
        if ((nib >> p) & 1u) {
            lo = 2u * rank;
            hi = 2u * rank + 1u;
            ++rank;
        }
        sel[p >> 1] |= (lo | (hi << 8)) << (16u * (p & 1u));
    }
    return make_uint2(sel[0], sel[1]);
}

// 16 consecutive bf16 of row `r` (of `n_rows`) starting at column `col`, or zeros outside.
__device__ __forceinline__ void load_row16(const uint16_t* __restrict__ p, int r, int n_rows, int col, int k_in,
                                           Frag& b0, Frag& b1) {
    if (r < n_rows && col < k_in) {
        const u32x4* q = reinterpret_cast<const u32x4*>(p + (size_t)r * k_in + col);
        b0.q = q[0];
        b1.q = q[1];
    } else {
        b0.q = u32x4{0, 0, 0, 0};
        b1.q = u32x4{0, 0, 0, 0};
    }
}

// Issue the loads of one tile: MAXCH coalesced 16-byte pieces per lane (clamped to the tile's
// own pieces, so no lane reads past the blob) and the lane's four 16-bit masks.
template <int MAXCH>
__device__ __forceinline__ void issue_tile(u32x4 (&st)[MAXCH], uint2& mk, const uint16_t* __restrict__ vals,
                                           const uint2* __restrict__ masks, uint32_t val_start, uint32_t nnz, int t,
                                           int lane) {
    const u32x4* __restrict__ src = reinterpret_cast<const u32x4*>(vals + (size_t)val_start * 8);
    const uint32_t n16 = (nnz * 2 + 8 + 15) / 16;  // 8 bytes of slack for the 12-byte windows
#pragma unroll
    for (int c = 0; c < MAXCH; ++c) st[c] = src[min((uint32_t)(c * 64 + lane), n16 - 1u)];
    mk = masks[(size_t)t * 64 + lane];
}

}  // namespace sd2
