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

// fp32 -> bf16, round to nearest, ties to even: the gfx950 packed conversion instruction
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return (uint16_t)(pack_bf16(f, 0.f) & 0xffffu); }

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

// Exclusive prefix sums of N values at once, stage by stage: the N cross-lane adds of a stage are independent, so they
// issue back to back instead of each waiting out the hazard slots behind the one before it.
template <int N>
__device__ __forceinline__ void wave_excl_scans(uint32_t (&x)[N]) {
#define SD2_SCAN_STAGE(ctrl, rmask) \
    _Pragma("unroll") for (int i = 0; i < N; ++i) x[i] += __builtin_amdgcn_update_dpp(0u, x[i], ctrl, rmask, 0xf, true)
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] = __builtin_amdgcn_update_dpp(0u, x[i], 0x138, 0xf, 0xf, true);  // wave_shr:1
    SD2_SCAN_STAGE(0x111, 0xf);  // row_shr:1
    SD2_SCAN_STAGE(0x112, 0xf);  // row_shr:2
    SD2_SCAN_STAGE(0x114, 0xf);  // row_shr:4
    SD2_SCAN_STAGE(0x118, 0xf);  // row_shr:8
    SD2_SCAN_STAGE(0x142, 0xa);  // row_bcast:15 -> rows 1,3
    SD2_SCAN_STAGE(0x143, 0xc);  // row_bcast:31 -> rows 2,3
#undef SD2_SCAN_STAGE
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

// Expands the tile staged in this wavefront's LDS buffer into its eight MFMA A operands and hands
// them, one 64-column super-step at a time, to use(q, f0, f1).
//
// Lane l owns row l % 16 and, in super-step q, columns 64q + 16(l / 16) + 0..15 as four nibbles of
// its 16-bit mask.  The values of run (q, h) = nibble h of every lane, in lane order, start at
// base[4q + h] (16-bit halves of the eight directory words); a lane's own values follow those of the
// lower lanes, whose count is an exclusive wave prefix sum of the nibble popcounts (four 8-bit fields
// scanned in one dword).  A 12-byte LDS window at the 4-byte-aligned address below the lane's first
// value, two byte-aligns and two byte-permutes with a selector looked up by the nibble put its (at most
// four) values into their columns and zeros elsewhere.  (A single 8-byte read at the 2-byte-aligned
// address is legal on gfx950 but measured far slower.)  The stream carries eight bytes of slack, so the
// window never leaves the buffer.
//
// The four scans run first and the LDS reads of STEPS super-steps are issued back to back before the
// first is consumed, so that a wavefront pays the LDS latency 4 / STEPS times per tile, not per nibble.
// First stage of the expansion: per super-step q, the four 8-bit exclusive prefix counts of its nibbles in ex[q].
__device__ __forceinline__ void expand_scans(uint2 mk, uint32_t (&ex)[4]) {
    // Nibble popcounts of a 32-bit mask word (two super-steps) at once: the classic pairwise sums give eight
    // 4-bit counts, two masks split them into bytes, and one byte permute per super-step lines up its four counts.
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        const uint32_t m = w ? mk.y : mk.x;
        uint32_t x = m - ((m >> 1) & 0x55555555u);
        x = (x & 0x33333333u) + ((x >> 2) & 0x33333333u);      // nibble n holds popcount(nibble n of m), 0..4
        const uint32_t even = x & 0x0f0f0f0fu;                 // bytes: counts of nibbles 0, 2, 4, 6
        const uint32_t odd = (x >> 4) & 0x0f0f0f0fu;           // bytes: counts of nibbles 1, 3, 5, 7
        // v_perm_b32(hi, lo, sel): selector byte 0..3 picks from lo, 4..7 from hi
        ex[2 * w] = __builtin_amdgcn_perm(odd, even, 0x05010400u);      // [n0, n1, n2, n3]
        ex[2 * w + 1] = __builtin_amdgcn_perm(odd, even, 0x07030602u);  // [n4, n5, n6, n7]
    }
    wave_excl_scans(ex);  // per nibble: values of lower lanes (<= 252, no carry); the four scans advance together
}

// Second stage: super-steps STEPS * part .. STEPS * part + STEPS - 1, handed to use(q, f0, f1).
template <int STEPS, typename F>
__device__ __forceinline__ void expand_part(int part, const uint8_t* __restrict__ bufb, const uint2* __restrict__ lut,
                                            const uint32_t (&base)[8], uint2 mk, const uint32_t (&ex)[4], F&& use) {
    static_assert(STEPS == 1 || STEPS == 2 || STEPS == 4, "super-steps whose LDS reads are batched");
    const uint32_t lds_base = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) uint8_t*)bufb;  // LDS byte address
    Tri32 tr[4 * STEPS];
    uint2 sel[4 * STEPS];
    uint32_t off[4 * STEPS];
#pragma unroll
    for (int i = 0; i < 4 * STEPS; ++i) {
        const int q = STEPS * part + (i >> 2), h = i & 3;
        const uint32_t m = (q >> 1) ? mk.y : mk.x;
        const uint32_t run_base = (base[(4 * q + h) >> 1] >> (16 * (h & 1))) & 0xffffu;
        // LDS address of the lane's first value: the run's start is scalar arithmetic, the lane adds its prefix
        // (the buffer is 4-byte aligned, so the low address bits are the byte offset's)
        off[i] = (lds_base + run_base * 2u) + __builtin_amdgcn_ubfe(ex[q], 8 * h, 8) * 2u;
        const __attribute__((address_space(3))) uint32_t* win =
            (const __attribute__((address_space(3))) uint32_t*)(uintptr_t)(off[i] & ~3u);
        tr[i].a = win[0];
        tr[i].b = win[1];
        tr[i].c = win[2];
        sel[i] = lut[__builtin_amdgcn_ubfe(m, 16 * (q & 1) + 4 * h, 4)];
    }
    Frag f[STEPS][2];
#pragma unroll
    for (int i = 0; i < 4 * STEPS; ++i) {
        const int h = i & 3;
        const uint32_t w0 = __builtin_amdgcn_alignbyte(tr[i].b, tr[i].a, off[i]);
        const uint32_t w1 = __builtin_amdgcn_alignbyte(tr[i].c, tr[i].b, off[i]);
        f[i >> 2][h >> 1].u[2 * (h & 1) + 0] = __builtin_amdgcn_perm(w1, w0, sel[i].x);
        f[i >> 2][h >> 1].u[2 * (h & 1) + 1] = __builtin_amdgcn_perm(w1, w0, sel[i].y);
    }
#pragma unroll
    for (int j = 0; j < STEPS; ++j) use(STEPS * part + j, f[j][0], f[j][1]);
}

template <int STEPS = 2, typename F>
__device__ __forceinline__ void expand_tile(const uint8_t* __restrict__ bufb, const uint2* __restrict__ lut,
                                            const uint32_t (&base)[8], uint2 mk, F&& use) {
    uint32_t ex[4];
    expand_scans(mk, ex);
#pragma unroll
    for (int part = 0; part < 4 / STEPS; ++part) expand_part<STEPS>(part, bufb, lut, base, mk, ex, use);
}

// The same request with the value stream written straight into LDS (no staging registers): piece c of the
// tile lands at lds_buf + c * 1024 bytes, 16 bytes per lane in lane order.  lds_buf is wave-uniform.  The
// data is in LDS once the wavefront's vector-memory counter has drained (s_waitcnt vmcnt(0)).
template <int MAXCH>
__device__ __forceinline__ void issue_tile_lds(uint32_t* lds_buf, uint2& mk, const uint16_t* __restrict__ vals,
                                               const uint2* __restrict__ tile_masks, uint32_t val_start, uint32_t nnz,
                                               int lane) {
    const u32x4* __restrict__ src = reinterpret_cast<const u32x4*>(vals + (size_t)val_start * 8);
    const uint32_t n16 = (nnz * 2 + 8 + 15) / 16;
#pragma unroll
    for (int c = 0; c < MAXCH; ++c)
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)(src + min((uint32_t)(c * 64 + lane), n16 - 1u)),
            (__attribute__((address_space(3))) void*)(lds_buf + c * 256), 16, 0, 0);
    mk = tile_masks[lane];
}

// Waits until every vector-memory operation of this wavefront has completed (loads returned, direct-to-LDS
// data written) without touching the other counters, and keeps the compiler from moving LDS reads above it.
__device__ __forceinline__ void wait_vector_memory() {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), expcnt and lgkmcnt unconstrained
    asm volatile("" ::: "memory");
}

}  // namespace sd2
