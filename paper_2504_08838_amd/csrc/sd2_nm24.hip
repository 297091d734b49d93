// libsd2 -- linear layer on a 2:4 semi-structured matrix (blob format 3) for gfx950.
//
// The paper evaluates 2:4 drafters next to unstructured ones (Sec. 3, Sec. 3.3).  With two values and
// two 2-bit column indices per group of four weights the matrix costs 1.125 bytes per dense weight,
// and the blob stores a tile exactly as v_smfmac_f32_16x16x64_bf16 wants its sparse operand: per
// step of 64 columns, 16 bytes of values per lane and a 16-bit index field.  So there is nothing to
// decode: a wavefront loads a tile with four 16-byte loads and one 8-byte load per lane (each load
// instruction reads one contiguous KiB) and issues four matrix instructions.
//
// One workgroup walks over 16-row strips; the contraction is split over its wavefronts by slab
// (256 columns): wavefront w owns slabs w, w + WAVES, ... and keeps their activation columns (the
// dense operand) in registers for the whole kernel.  Per strip the partial 16 x 16 blocks meet in
// LDS (double buffered, one barrier), four wavefronts add them in a fixed order and write y -- final
// values, no split-K partials in memory.
#include <algorithm>
#include <atomic>

#include "sd2_device.h"
#include "sd2_format.h"
#include "sd2_internal.h"

namespace sd2 {

typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 bf16x16;

struct Nm24Tile {
    u32x4 v[4];   // values of the four steps
    uint2 idx;    // column indices: steps 0, 1 in .x (16 bits each), steps 2, 3 in .y
};

union Frag16 {
    u32x4 q[2];
    bf16x16 v;
};

__device__ __forceinline__ void nm24_load(Nm24Tile& t, const uint8_t* __restrict__ tiles, size_t tile, int lane) {
    const uint8_t* p = tiles + tile * (size_t)kNm24TileBytes;
#pragma unroll
    for (int q = 0; q < 4; ++q) t.v[q] = *reinterpret_cast<const u32x4*>(p + (size_t)(64 * q + lane) * 16);
    t.idx = *reinterpret_cast<const uint2*>(p + 4096 + 8 * lane);
}

template <int SPW, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void nm24_linear_kernel(const uint8_t* __restrict__ tiles,
                                                                 const uint16_t* __restrict__ x, float* __restrict__ y,
                                                                 int n_out, int k_in, int k_tok, int n_strips, int n_slabs) {
    __shared__ float red[2 * WAVES * 256];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, gb = lane >> 4;
    const int my_strips = (n_strips - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    // this wavefront's slabs: wave + WAVES * j; a slab past the matrix contributes nothing and loads nothing
    int n_mine = 0;
#pragma unroll
    for (int j = 0; j < SPW; ++j) n_mine += (wave + WAVES * j < n_slabs) ? 1 : 0;

    // Flat tile order of the wavefront: strip by strip, its slabs within a strip.  D register sets form a ring:
    // set f mod D holds tile f and is refilled with tile f + D as soon as tile f has gone through the matrix
    // instructions, so D - 1 tiles are always in flight.  The loop is unrolled D times: set numbers are static.
    constexpr int D = SPW == 1 ? 3 : 2;
    auto tile_of = [&](int i, int j) { return (size_t)(wave + WAVES * j) * n_strips + ((int)blockIdx.x + i * (int)gridDim.x); };
    int ri = 0, rj = 0;  // the next tile to request
    auto request = [&](Nm24Tile& t) {
        if (ri < my_strips) {
            nm24_load(t, tiles, tile_of(ri, rj), lane);
            if (++rj == n_mine) {
                rj = 0;
                ++ri;
            }
        }
    };
    Nm24Tile set[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        set[d].v[0] = set[d].v[1] = set[d].v[2] = set[d].v[3] = u32x4{0u, 0u, 0u, 0u};
        set[d].idx = make_uint2(0u, 0u);
        if (n_mine > 0) request(set[d]);
    }

    // dense operand: lane (token n, block gb) holds columns 64 q + 16 gb + 0..15 of step q of each of its slabs
    const int tok = min(n, k_tok - 1);  // lanes past the last token repeat it; their results are never written
    Frag16 b[SPW][4];
#pragma unroll
    for (int j = 0; j < SPW; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = (wave + WAVES * j) * 256 + 64 * q + 16 * gb;
            if (col < k_in) {
                const u32x4* src = reinterpret_cast<const u32x4*>(x + (size_t)tok * k_in + col);
                b[j][q].q[0] = src[0];
                b[j][q].q[1] = src[1];
            } else {
                b[j][q].q[0] = b[j][q].q[1] = u32x4{0u, 0u, 0u, 0u};
            }
        }

    const int red_tok = lane >> 2, red_row = 4 * wave + (lane & 3);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    // The strip's partial block goes to LDS (double buffered, one barrier per strip); the first four wavefronts add
    // the blocks of all wavefronts in a fixed order: thread (wave rho, lane l) owns token l >> 2, row 4 rho + (l & 3).
    auto strip_end = [&](int i) {
        float* mine = red + (i & 1) * (WAVES * 256);
        *reinterpret_cast<f32x4*>(mine + wave * 256 + lane * 4) = acc;
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the block is in LDS; the tiles on their way stay in flight
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (wave < 4) {
            float v = 0.f;
#pragma unroll
            for (int ww = 0; ww < WAVES; ++ww) v += mine[ww * 256 + wave * 64 + lane];
            const int row = ((int)blockIdx.x + i * (int)gridDim.x) * 16 + red_row;
            if (row < n_out && red_tok < k_tok) y[(size_t)red_tok * n_out + row] = v;
        }
        acc = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    auto multiply = [&](const Nm24Tile& t, const Frag16 (&bj)[4]) {
        acc = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8, t.v[0]), bj[0].v, acc, (int)t.idx.x, 0, 0);
        acc = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8, t.v[1]), bj[1].v, acc, (int)t.idx.x, 0, 1);
        acc = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8, t.v[2]), bj[2].v, acc, (int)t.idx.y, 0, 0);
        acc = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8, t.v[3]), bj[3].v, acc, (int)t.idx.y, 0, 1);
    };

    if (n_mine == 0) {  // a wavefront without slabs still joins every barrier
#pragma unroll 1
        for (int i = 0; i < my_strips; ++i) strip_end(i);
        return;
    }
    const int n_flat = my_strips * n_mine;
    int i = 0, j = 0;
#pragma unroll 1
    for (int f0 = 0; f0 < n_flat; f0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (f0 + d < n_flat) {  // wave-uniform
                // the slab within the strip picks the dense operand: wave-uniform branches, static register numbers
                if (SPW == 1 || j == 0)
                    multiply(set[d], b[0]);
                else if (SPW == 2 || j == 1)
                    multiply(set[d], b[SPW > 1 ? 1 : 0]);
                else
                    multiply(set[d], b[SPW > 2 ? 2 : 0]);
                request(set[d]);
                if (++j == n_mine) {
                    j = 0;
                    strip_end(i);
                    ++i;
                }
            }
        }
    }
}

static int nm24_cu_count() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
        return n;
    return 256;
}

template <int SPW, int WAVES>
static hipError_t launch_nm24_t(const uint8_t* tiles, const uint16_t* x, float* y, int n_out, int k_in, int k_tok,
                                int n_strips, int n_slabs, hipStream_t s) {
    // as many workgroups as fit on the chip at once (registers and LDS decide how many per compute unit)
    static std::atomic<int> cached{0};  // threads that race here compute the same value
    int resident = cached.load(std::memory_order_relaxed);
    if (resident == 0) {
        int per_cu = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, nm24_linear_kernel<SPW, WAVES>, 64 * WAVES, 0) != hipSuccess ||
            per_cu < 1)
            per_cu = 1;
        resident = nm24_cu_count() * per_cu;
        cached.store(resident, std::memory_order_relaxed);
    }
    const int grid = std::min(n_strips, resident);
    hipLaunchKernelGGL((nm24_linear_kernel<SPW, WAVES>), dim3((unsigned)grid), dim3(64 * WAVES), 0, s, tiles, x, y, n_out, k_in,
                       k_tok, n_strips, n_slabs);
    return hipGetLastError();
}

// Slabs per wavefront and wavefronts per workgroup: the dense operand of a slab takes 32 registers, so three
// slabs per wavefront are only combined with at most 12 wavefronts (three per SIMD).
static bool nm24_shape(int n_slabs, int& spw, int& waves) {
    for (spw = 1; spw <= 3; ++spw) {
        const int need = (n_slabs + spw - 1) / spw;  // wavefronts that get a slab
        if (need <= (spw == 3 ? 12 : 16)) {
            waves = std::max(4, (need + 3) / 4 * 4);  // in steps of four (the first four also add the partials)
            return true;
        }
    }
    return false;
}

bool nm24_supported(int n_slabs) {
    int spw, waves;
    return n_slabs >= 1 && nm24_shape(n_slabs, spw, waves);
}

// y[t][n] for tokens [0, k_tok), k_tok <= 16: final values (every entry of y written).
hipError_t launch_nm24_linear(const MatArgs& m, const LinArgs& a, hipStream_t s) {
    int spw, waves;
    if (m.n_slabs < 1 || !nm24_shape(m.n_slabs, spw, waves) || a.k_tok < 1 || a.k_tok > 16) return hipErrorInvalidValue;
    const uint8_t* tiles = static_cast<const uint8_t*>(m.dir);  // format 3 has no directory: the tiles follow the header
#define SD2_NM24_CASE(S, W) \
    if (spw == S && waves == W) return launch_nm24_t<S, W>(tiles, a.x, a.out, m.n_out, m.k_in, a.k_tok, m.n_strips, m.n_slabs, s)
    SD2_NM24_CASE(1, 4);
    SD2_NM24_CASE(1, 8);
    SD2_NM24_CASE(1, 12);
    SD2_NM24_CASE(1, 16);
    SD2_NM24_CASE(2, 12);
    SD2_NM24_CASE(2, 16);
    SD2_NM24_CASE(3, 12);
#undef SD2_NM24_CASE
    return hipErrorInvalidValue;
}

}  // namespace sd2
