// gfx950 (CDNA4, MI355X) kernels of libsd2.
//
// Sparse linear.  A wavefront walks a contiguous range of 16x256 tiles of the packed matrix.
// While it decodes one tile out of its private LDS buffer, the compacted stream and the masks
// of its next tile are already in flight in registers (plain coalesced 16-byte loads that do not
// depend on the masks).  Decoding, per 16x64 step: every lane owns 16 columns of one row as four
// nibbles; a wave-wide exclusive prefix sum over the four nibble populations (one packed DPP
// scan) plus the per-run base from the tile directory gives the position of the lane's values in
// the stream; a 12-byte LDS window is byte-aligned and spread over the four columns with two
// byte-permutes whose selectors come from a 16-entry table; the dense 16x32 bf16 fragments go
// through v_mfma_f32_16x16x32_bf16 against the activations held in registers.  The MFMA is used
// for the multiply because the decode already leaves a dense fragment in registers and the vector
// ALU is the scarce unit here; HBM traffic is the compacted stream and nothing else.
#include <algorithm>
#include <atomic>

#include "sd2_device.h"
#include "sd2_internal.h"

#ifndef SD2_LINEAR_STEPS
#define SD2_LINEAR_STEPS 1  // super-steps per batch of LDS reads in the stand-alone kernel (16 waves per CU hide the rest)
#endif

namespace sd2 {

// One 16 x k_tok block of results: lane (n = lane & 15, g = lane >> 4) holds rows 4g..4g+3 of token n.
template <int TG>
__device__ __forceinline__ void store_tile(const f32x4 (&acc)[TG], float* __restrict__ out, int n_out, int k_tok,
                                           int strip, int slab, int lane) {
    const int n = lane & 15, g = lane >> 4;
    const int row = strip * 16 + 4 * g;
    float* base = out + (size_t)slab * k_tok * n_out;
#pragma unroll
    for (int tg = 0; tg < TG; ++tg) {
        const int tok = n + 16 * tg;
        if (tok >= k_tok) continue;
        float* dst = base + (size_t)tok * n_out + row;
        if ((n_out & 3) == 0) {
            if (row < n_out) *reinterpret_cast<float4*>(dst) = make_float4(acc[tg][0], acc[tg][1], acc[tg][2], acc[tg][3]);
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (row + v < n_out) dst[v] = acc[tg][v];
        }
    }
}

// ------------------------------------------------------------------ sparse linear

template <int MAXCH, int TG, bool PREFETCH>
__device__ __forceinline__ void sparse_tile(u32x4 (&st)[MAXCH], uint2& mk_next, DirEnt& de_cur, DirEnt& de_next,
                                            Frag (&b)[4][2], int& cur_slab, uint32_t* __restrict__ buf,
                                            const uint2* __restrict__ lut, const DirEnt* __restrict__ dir,
                                            const uint2* __restrict__ masks, const uint16_t* __restrict__ vals,
                                            const uint16_t* __restrict__ x, float* __restrict__ out, int n_out, int k_in,
                                            int k_tok, int n_strips, int n_tiles, int t, int lane) {
    const int n = lane & 15, g = lane >> 4;
    // the staged tile goes to this wave's LDS buffer (its loads were issued one tile ago)
#pragma unroll
    for (int c = 0; c < MAXCH; ++c) reinterpret_cast<u32x4*>(buf)[c * 64 + lane] = st[c];
    const uint2 mk = mk_next;
    const int strip = t % n_strips, slab = t / n_strips;
    const int col0 = slab * 256 + 16 * g;
    if (TG == 1 && slab != cur_slab) {
        cur_slab = slab;
#pragma unroll
        for (int q = 0; q < 4; ++q) load_row16(x, n, k_tok, col0 + 64 * q, k_in, b[q][0], b[q][1]);
    }
    if (PREFETCH) {
        issue_tile<MAXCH>(st, mk_next, vals, masks, de_next.val_start, de_next.nnz, t + 1, lane);
    }
    const DirEnt de = de_cur;
    de_cur = de_next;
    de_next = dir[min(t + 2, n_tiles - 1)];

    f32x4 acc[TG];
#pragma unroll
    for (int tg = 0; tg < TG; ++tg) acc[tg] = f32x4{0.f, 0.f, 0.f, 0.f};
    expand_tile<SD2_LINEAR_STEPS>(reinterpret_cast<const uint8_t*>(buf), lut, de.base, mk, [&](int q, const Frag& f0, const Frag& f1) {
        if (TG == 1) {
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0.v, b[q][0].v, acc[0], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f1.v, b[q][1].v, acc[0], 0, 0, 0);
        } else {
#pragma unroll
            for (int tg = 0; tg < TG; ++tg) {
                Frag x0, x1;
                load_row16(x, n + 16 * tg, k_tok, col0 + 64 * q, k_in, x0, x1);
                acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0.v, x0.v, acc[tg], 0, 0, 0);
                acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f1.v, x1.v, acc[tg], 0, 0, 0);
            }
        }
    });
    store_tile<TG>(acc, out, n_out, k_tok, strip, slab, lane);
}

// The same tile with the multiply on the vector ALU instead of the matrix cores (k_tok <= 8): the lane that owns 16
// columns of a row in a super-step reads the matching 16 activations of every token from the wavefront's copy of the
// slab's activation columns in LDS (the four lanes groups read four addresses: broadcasts) and adds the products with
// the packed bf16 dot-product instruction, fp32 sums; at the end of the tile the four column groups of a row are
// added across lanes.  It exists to put a number on the alternative to the matrix instruction; nothing selects it
// unless the caller asks for it.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
constexpr int kValuTok = 8;

template <int MAXCH, bool PREFETCH>
__device__ __forceinline__ void sparse_tile_valu(u32x4 (&st)[MAXCH], uint2& mk_next, DirEnt& de_cur, DirEnt& de_next,
                                                 int& cur_slab, uint32_t* __restrict__ buf, uint32_t* __restrict__ xs,
                                                 const uint2* __restrict__ lut, const DirEnt* __restrict__ dir,
                                                 const uint2* __restrict__ masks, const uint16_t* __restrict__ vals,
                                                 const uint16_t* __restrict__ x, float* __restrict__ out, int n_out, int k_in,
                                                 int k_tok, int n_strips, int n_tiles, int t, int lane) {
    const int n = lane & 15, g = lane >> 4;
#pragma unroll
    for (int c = 0; c < MAXCH; ++c) reinterpret_cast<u32x4*>(buf)[c * 64 + lane] = st[c];
    const uint2 mk = mk_next;
    const int strip = t % n_strips, slab = t / n_strips;
    if (slab != cur_slab) {  // this wavefront's copy of the slab's activation columns: [token][256] bf16
        cur_slab = slab;
#pragma unroll
        for (int it = 0; it < kValuTok / 2; ++it) {
            const int tok = 2 * it + (lane >> 5), piece = lane & 31, col = slab * 256 + 8 * piece;
            u32x4 v = u32x4{0, 0, 0, 0};
            if (tok < k_tok && col < k_in) v = *reinterpret_cast<const u32x4*>(x + (size_t)tok * k_in + col);
            reinterpret_cast<u32x4*>(xs)[tok * 32 + piece] = v;
        }
    }
    if (PREFETCH) issue_tile<MAXCH>(st, mk_next, vals, masks, de_next.val_start, de_next.nnz, t + 1, lane);
    const DirEnt de = de_cur;
    de_cur = de_next;
    de_next = dir[min(t + 2, n_tiles - 1)];

    float acc[kValuTok];
#pragma unroll
    for (int tok = 0; tok < kValuTok; ++tok) acc[tok] = 0.f;
    expand_tile<SD2_LINEAR_STEPS>(reinterpret_cast<const uint8_t*>(buf), lut, de.base, mk, [&](int q, const Frag& f0, const Frag& f1) {
#pragma unroll
        for (int tok = 0; tok < kValuTok; ++tok) {
            if (tok < k_tok) {
                Frag x0, x1;
                const u32x4* xr = reinterpret_cast<const u32x4*>(xs) + tok * 32 + 8 * q + 2 * g;
                x0.q = xr[0];
                x1.q = xr[1];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[tok] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, f0.u[e]), __builtin_bit_cast(bf16x2_t, x0.u[e]), acc[tok], false);
                    acc[tok] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, f1.u[e]), __builtin_bit_cast(bf16x2_t, x1.u[e]), acc[tok], false);
                }
            }
        }
    });
    float* base = out + (size_t)slab * k_tok * n_out;
    const int row = strip * 16 + n;
#pragma unroll
    for (int tok = 0; tok < kValuTok; ++tok) {
        if (tok < k_tok) {
            float v = acc[tok];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (g == (tok & 3) && row < n_out) base[(size_t)tok * n_out + row] = v;
        }
    }
}

template <int MAXCH>
__global__ __launch_bounds__(256) void sparse_linear_valu_kernel(const DirEnt* __restrict__ dir, const uint2* __restrict__ masks,
                                                                const uint16_t* __restrict__ vals,
                                                                const uint16_t* __restrict__ x, float* __restrict__ out,
                                                                int n_out, int k_in, int k_tok, int n_strips, int n_tiles,
                                                                int tiles_per_wave) {
    extern __shared__ uint32_t tile_smem[];  // per wavefront: the tile buffer, then [kValuTok][256] bf16 activations
    __shared__ uint2 lut[16];
    const int tid = threadIdx.x;
    if (tid < 16) lut[tid] = make_expand_selector((uint32_t)tid);
    __syncthreads();
    const int lane = tid & 63, wave = tid >> 6;
    const int gw = __builtin_amdgcn_readfirstlane((int)blockIdx.x * kWavesPerBlock + wave);
    const int t0 = gw * tiles_per_wave;
    const int t1 = min(t0 + tiles_per_wave, n_tiles);
    if (t0 >= t1) return;
    uint32_t* buf = tile_smem + wave * (MAXCH * 256 + kValuTok * 128);
    uint32_t* xs = buf + MAXCH * 256;
    u32x4 st[MAXCH];
    uint2 mk_next;
    DirEnt de_cur = dir[t0];
    DirEnt de_next = dir[min(t0 + 1, n_tiles - 1)];
    issue_tile<MAXCH>(st, mk_next, vals, masks, de_cur.val_start, de_cur.nnz, t0, lane);
    int cur_slab = -1;
#pragma unroll 1
    for (int t = t0; t < t1 - 1; ++t)
        sparse_tile_valu<MAXCH, true>(st, mk_next, de_cur, de_next, cur_slab, buf, xs, lut, dir, masks, vals, x, out, n_out, k_in,
                                      k_tok, n_strips, n_tiles, t, lane);
    sparse_tile_valu<MAXCH, false>(st, mk_next, de_cur, de_next, cur_slab, buf, xs, lut, dir, masks, vals, x, out, n_out, k_in,
                                   k_tok, n_strips, n_tiles, t1 - 1, lane);
}

template <int MAXCH, int TG>
__global__ __launch_bounds__(256) void sparse_linear_kernel(const DirEnt* __restrict__ dir, const uint2* __restrict__ masks,
                                                           const uint16_t* __restrict__ vals,
                                                           const uint16_t* __restrict__ x, float* __restrict__ out,
                                                           int n_out, int k_in, int k_tok, int n_strips, int n_tiles,
                                                           int tiles_per_wave) {
    extern __shared__ uint32_t tile_smem[];
    __shared__ uint2 lut[16];
    const int tid = threadIdx.x;
    if (tid < 16) lut[tid] = make_expand_selector((uint32_t)tid);
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    const int gw = __builtin_amdgcn_readfirstlane((int)blockIdx.x * kWavesPerBlock + wave);
    const int t0 = gw * tiles_per_wave;
    const int t1 = min(t0 + tiles_per_wave, n_tiles);
    if (t0 >= t1) return;
    uint32_t* buf = tile_smem + wave * (MAXCH * 256);

    u32x4 st[MAXCH];
    uint2 mk_next;
    DirEnt de_cur = dir[t0];
    DirEnt de_next = dir[min(t0 + 1, n_tiles - 1)];
    issue_tile<MAXCH>(st, mk_next, vals, masks, de_cur.val_start, de_cur.nnz, t0, lane);
    int cur_slab = -1;
    Frag b[4][2];
#pragma unroll 1
    for (int t = t0; t < t1 - 1; ++t)
        sparse_tile<MAXCH, TG, true>(st, mk_next, de_cur, de_next, b, cur_slab, buf, lut, dir, masks, vals, x, out, n_out,
                                     k_in, k_tok, n_strips, n_tiles, t, lane);
    sparse_tile<MAXCH, TG, false>(st, mk_next, de_cur, de_next, b, cur_slab, buf, lut, dir, masks, vals, x, out, n_out,
                                  k_in, k_tok, n_strips, n_tiles, t1 - 1, lane);
}

// ------------------------------------------------------------------ sparse linear, final results in one launch
//
// The same tiles, walked so that no partial sums leave the compute unit (k_tok <= 16).  A workgroup owns strips
// b, b + G, ...; the contraction of a strip is split over its wavefronts by slab: wavefront w owns slabs w, w + WAVES, ...
// (SPW of them) and sums their tiles of a strip in its accumulator.  The wavefronts' 16 x 16 blocks of a strip meet in
// LDS; every few strips a barrier that waits for LDS only lets the threads add them in a fixed order and write y.  A wavefront with one slab keeps that slab's activation columns in registers for the whole kernel; with
// more slabs it fetches them per tile (they stay in the caches).  The streams of the next two tiles are in flight in
// registers while the current one is expanded.
//
// More than 16 tokens (TG = 2..4 groups of 16): the tile is still expanded once, and each of its eight dense fragments
// goes through one matrix instruction per token group.  The activation columns of all groups no longer fit a
// wavefront's registers, so they are fetched per 64-column step (they stay in the caches: every wavefront of the chip
// reads the same [k_tok][k_in] array), one step ahead of the expansion that consumes them.
constexpr int kStripRound = 4;  // strip results (of 16 tokens each) between two workgroup barriers of the kernel below
// strips per round for TG token groups; the gated variant needs whole pairs in a round
constexpr int strip_round(int tg, bool gated) {
    const int r = kStripRound / tg > 0 ? kStripRound / tg : 1;
    return gated && (r & 1) ? r + 1 : r;
}

//
// GATED: the matrix is [gate; up] (two halves of n_out / 2 rows that share the input) and what leaves the kernel is the
// gated product bf16(silu(gate x) * (up x)), [k_tok][n_out / 2], written to y (as uint16): a workgroup then owns pairs
// of strips, strip p of the gate half and strip p of the up half, which sit side by side in a round's slots.
template <int MAXCH, int SPW, int WAVES, int TG, bool GATED = false>
__global__ __launch_bounds__(64 * WAVES) void sparse_strip_kernel(const DirEnt* __restrict__ dir, const uint2* __restrict__ masks,
                                                                 const uint16_t* __restrict__ vals,
                                                                 const uint16_t* __restrict__ x_all, float* __restrict__ y_all,
                                                                 int n_out, int k_in, int k_tok_all, int n_strips, int n_slabs) {
    extern __shared__ uint32_t strip_smem[];  // [WAVES][MAXCH * 256] tile buffers, then [kStripRound][WAVES][256] floats
    // More tokens than one pass takes: the grid's second dimension numbers the passes of 16 TG tokens each (the matrix is
    // streamed once per pass; a pass is this kernel on its own slice of the activations and of the results).
    const int pass = (int)blockIdx.y;
    const uint16_t* __restrict__ x = x_all + (size_t)pass * (16 * TG) * k_in;
    float* __restrict__ y = GATED ? reinterpret_cast<float*>(reinterpret_cast<uint16_t*>(y_all) + (size_t)pass * (16 * TG) * (n_out / 2))
                                  : y_all + (size_t)pass * (16 * TG) * n_out;
    const int k_tok = min(16 * TG, k_tok_all - pass * (16 * TG));
    __shared__ uint2 lut[16];
    const int tid = threadIdx.x;
    if (tid < 16) lut[tid] = make_expand_selector((uint32_t)tid);
    __syncthreads();
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    uint32_t* buf = strip_smem + wave * (MAXCH * 256);
    float* red = reinterpret_cast<float*>(strip_smem + WAVES * (MAXCH * 256));
    constexpr int kRound = strip_round(TG, GATED);  // strips per round: the slots of a round fit LDS
    // the strips this workgroup walks, in order: b, b + G, ... -- or, gated, the pairs (b, b + half), (b + G, b + G + half), ...
    const int n_units = GATED ? n_strips / 2 : n_strips;
    const int my_units = (n_units - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int my_strips = GATED ? 2 * my_units : my_units;
    auto strip_of = [&](int ord) {
        return GATED ? (int)blockIdx.x + (ord >> 1) * (int)gridDim.x + (ord & 1) * n_units : (int)blockIdx.x + ord * (int)gridDim.x;
    };
    int n_mine = 0;  // this wavefront's slabs: wave + WAVES * j
#pragma unroll
    for (int j = 0; j < SPW; ++j) n_mine += (wave + WAVES * j < n_slabs) ? 1 : 0;
    const int n_flat = my_strips * n_mine;  // its tiles, strip by strip
    auto tile_of = [&](int f) {
        const int i = f / max(n_mine, 1), j = f - i * max(n_mine, 1);
        return (wave + WAVES * j) * n_strips + strip_of(i);
    };

    // The strips are handled in rounds of kRound: every wavefront leaves its blocks of a strip (one per token group) in
    // the strip's slot, one barrier (LDS only: streams stay in flight) ends the round, and the threads share the adding:
    // entry e of a block is token 16 tg + ((e & 63) >> 2), row 4 (e >> 6) + (e & 3) of the strip.  A second barrier
    // frees the slots.
    f32x4 acc[TG];
#pragma unroll
    for (int tg = 0; tg < TG; ++tg) acc[tg] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto round_end = [&](int i_first, int n_in_round) {
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (GATED) {
            // a round holds whole pairs: slot 2 r is the gate strip, slot 2 r + 1 the up strip of pair r
            const int half_rows = n_out / 2;
            uint16_t* m_out = reinterpret_cast<uint16_t*>(y);
            for (int idx = tid; idx < (n_in_round / 2) * TG * 256; idx += 64 * WAVES) {
                const int e = idx & 255, tg = (idx >> 8) % TG, r = (idx >> 8) / TG;
                const float* slot = red + (size_t)(2 * r) * (WAVES * TG * 256) + tg * 256;
                float gv = 0.f, uv = 0.f;
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww) {
                    gv += slot[ww * (TG * 256) + e];
                    uv += slot[WAVES * TG * 256 + ww * (TG * 256) + e];
                }
                const int tok = 16 * tg + ((e & 63) >> 2);
                const int row = strip_of(i_first + 2 * r) * 16 + 4 * (e >> 6) + (e & 3);
                if (row < half_rows && tok < k_tok) m_out[(size_t)tok * half_rows + row] = f32_to_bf16(gv / (1.0f + expf(-gv)) * uv);
            }
        } else {
            for (int idx = tid; idx < n_in_round * TG * 256; idx += 64 * WAVES) {
                const int e = idx & 255, tg = (idx >> 8) % TG, r = (idx >> 8) / TG;
                const float* slot = red + (size_t)r * (WAVES * TG * 256) + tg * 256;
                float v = 0.f;
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww) v += slot[ww * (TG * 256) + e];
                const int tok = 16 * tg + ((e & 63) >> 2);
                const int row = strip_of(i_first + r) * 16 + 4 * (e >> 6) + (e & 3);
                if (row < n_out && tok < k_tok) y[(size_t)tok * n_out + row] = v;
            }
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    auto strip_done = [&](int i) {  // lane (n, g) holds rows 4g..4g+3 of token n: entry (16 g + n) * 4 + v of the block
#pragma unroll
        for (int tg = 0; tg < TG; ++tg) {
            *reinterpret_cast<f32x4*>(red + (size_t)(i % kRound) * (WAVES * TG * 256) + (wave * TG + tg) * 256 + lane * 4) = acc[tg];
            acc[tg] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        if ((i + 1) % kRound == 0 || i + 1 == my_strips) round_end(i - i % kRound, i % kRound + 1);
    };
    if (n_mine == 0) {  // a wavefront without slabs contributes zeros and joins every barrier
#pragma unroll 1
        for (int i = 0; i < my_strips; ++i) strip_done(i);
        return;
    }

    // Operand B in registers: always for one token group; for two groups when the wavefront owns a single slab (its
    // activation columns then never change).  Otherwise B is fetched per 64-column step (below).
    constexpr bool kBRegs = TG == 1 || (TG == 2 && SPW == 1);
    constexpr int kBG = kBRegs ? TG : 1;
    Frag b[kBG][4][2];
    auto load_b = [&](int slab) {
        const int col0 = slab * 256 + 16 * g;
#pragma unroll
        for (int tg = 0; tg < kBG; ++tg)
#pragma unroll
            for (int q = 0; q < 4; ++q) load_row16(x, n + 16 * tg, k_tok, col0 + 64 * q, k_in, b[tg][q][0], b[tg][q][1]);
    };
    if (kBRegs && SPW == 1) load_b(wave);

    // two tiles' streams are in flight in registers while a third is expanded
    u32x4 st[2][MAXCH];
    uint2 mkn[2];
    DirEnt den[2];
    auto request = [&](int slot, int f) {
        if (f < n_flat) {
            const int t = tile_of(f);
            den[slot] = dir[t];
            issue_tile<MAXCH>(st[slot], mkn[slot], vals, masks, den[slot].val_start, den[slot].nnz, t, lane);
        }
    };
    request(0, 0);
    request(1, 1);
    int j = 0, i = 0;
    auto consume = [&](int slot, int f) {
#pragma unroll
        for (int c = 0; c < MAXCH; ++c) reinterpret_cast<u32x4*>(buf)[c * 64 + lane] = st[slot][c];
        const uint2 mk = mkn[slot];
        const DirEnt de = den[slot];
        if (kBRegs) {
            if (SPW > 1) load_b(wave + WAVES * j);
            request(slot, f + 2);
            expand_tile<SD2_LINEAR_STEPS>(reinterpret_cast<const uint8_t*>(buf), lut, de.base, mk,
                                          [&](int q, const Frag& f0, const Frag& f1) {
#pragma unroll
                                              for (int tg = 0; tg < kBG; ++tg) {
                                                  acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0.v, b[tg][q][0].v, acc[tg], 0, 0, 0);
                                                  acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f1.v, b[tg][q][1].v, acc[tg], 0, 0, 0);
                                              }
                                          });
        } else {
            // operand B of step q for every token group, requested one step ahead of its use
            const int col0 = (wave + WAVES * j) * 256 + 16 * g;
            Frag bb[2][TG][2];
            auto load_bq = [&](int q) {
#pragma unroll
                for (int tg = 0; tg < TG; ++tg) load_row16(x, n + 16 * tg, k_tok, col0 + 64 * q, k_in, bb[q & 1][tg][0], bb[q & 1][tg][1]);
            };
            load_bq(0);
            request(slot, f + 2);
            expand_tile<1>(reinterpret_cast<const uint8_t*>(buf), lut, de.base, mk, [&](int q, const Frag& f0, const Frag& f1) {
                if (q < 3) load_bq(q + 1);
#pragma unroll
                for (int tg = 0; tg < TG; ++tg) {
                    acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0.v, bb[q & 1][tg][0].v, acc[tg], 0, 0, 0);
                    acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f1.v, bb[q & 1][tg][1].v, acc[tg], 0, 0, 0);
                }
            });
        }
        if (++j == n_mine) {
            j = 0;
            strip_done(i);
            ++i;
        }
    };
#pragma unroll 1
    for (int f = 0; f < n_flat; f += 2) {
        consume(0, f);
        if (f + 1 < n_flat) consume(1, f + 1);
    }
}

// ------------------------------------------------------------------ dense bf16 baseline
// Same tile walk, operand A read straight from the row-major matrix; the next tile's fragments
// are in flight while the current one goes through the MFMAs.

__device__ __forceinline__ void issue_dense_tile(Frag (&f)[4][2], const uint16_t* __restrict__ w, int n_out, int k_in,
                                                 int n_strips, int t, int lane) {
    const int strip = t % n_strips, slab = t / n_strips;
    const int row = strip * 16 + (lane & 15);
    const int col0 = slab * 256 + 16 * (lane >> 4);
#pragma unroll
    for (int q = 0; q < 4; ++q) load_row16(w, row, n_out, col0 + 64 * q, k_in, f[q][0], f[q][1]);
}

template <int TG>
__global__ __launch_bounds__(256) void dense_linear_kernel(const uint16_t* __restrict__ w, const uint16_t* __restrict__ x,
                                                          float* __restrict__ out, int n_out, int k_in, int k_tok,
                                                          int n_strips, int n_tiles, int tiles_per_wave) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int gw = __builtin_amdgcn_readfirstlane((int)blockIdx.x * kWavesPerBlock + (tid >> 6));
    const int t0 = gw * tiles_per_wave;
    const int t1 = min(t0 + tiles_per_wave, n_tiles);
    if (t0 >= t1) return;
    const int n = lane & 15, g = lane >> 4;
    Frag nxt[4][2], b[4][2];
    issue_dense_tile(nxt, w, n_out, k_in, n_strips, t0, lane);
    int cur_slab = -1;
#pragma unroll 1
    for (int t = t0; t < t1; ++t) {
        Frag f[4][2];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            f[q][0].q = nxt[q][0].q;
            f[q][1].q = nxt[q][1].q;
        }
        const int strip = t % n_strips, slab = t / n_strips;
        const int col0 = slab * 256 + 16 * g;
        if (TG == 1 && slab != cur_slab) {
            cur_slab = slab;
#pragma unroll
            for (int q = 0; q < 4; ++q) load_row16(x, n, k_tok, col0 + 64 * q, k_in, b[q][0], b[q][1]);
        }
        issue_dense_tile(nxt, w, n_out, k_in, n_strips, min(t + 1, t1 - 1), lane);
        f32x4 acc[TG];
#pragma unroll
        for (int tg = 0; tg < TG; ++tg) acc[tg] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (TG == 1) {
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[q][0].v, b[q][0].v, acc[0], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[q][1].v, b[q][1].v, acc[0], 0, 0, 0);
            } else {
#pragma unroll
                for (int tg = 0; tg < TG; ++tg) {
                    Frag x0, x1;
                    load_row16(x, n + 16 * tg, k_tok, col0 + 64 * q, k_in, x0, x1);
                    acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[q][0].v, x0.v, acc[tg], 0, 0, 0);
                    acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[q][1].v, x1.v, acc[tg], 0, 0, 0);
                }
            }
        }
        store_tile<TG>(acc, out, n_out, k_tok, strip, slab, lane);
    }
}

// ------------------------------------------------------------------ launch

static int device_cu_count() {
    static std::atomic<int> cached{0};  // threads that race here compute the same value
    int cus = cached.load(std::memory_order_relaxed);
    if (cus == 0) {
        int dev = 0, n = 0;
        cus = (hipGetDevice(&dev) == hipSuccess &&
               hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
                  ? n
                  : 256;
        cached.store(cus, std::memory_order_relaxed);
    }
    return cus;
}

// Tiles per wavefront: enough wavefronts to fill every CU a few times over, then longer ranges
// so that the prefetch of the next tile has something to overlap with.
static int tiles_per_wave_for(int n_tiles, int waves_per_cu) {
    const int target = device_cu_count() * waves_per_cu;
    return n_tiles <= target ? 1 : (n_tiles + target - 1) / target;
}

template <int MAXCH, int TG>
static hipError_t launch_sparse_t(const MatArgs& m, const LinArgs& a, hipStream_t s) {
    const int tpw = tiles_per_wave_for(m.n_tiles, 16);
    const int waves = (m.n_tiles + tpw - 1) / tpw;
    const dim3 grid((unsigned)((waves + kWavesPerBlock - 1) / kWavesPerBlock)), block(64 * kWavesPerBlock);
    const size_t lds = (size_t)kWavesPerBlock * MAXCH * 1024;
    hipLaunchKernelGGL((sparse_linear_kernel<MAXCH, TG>), grid, block, lds, s, static_cast<const DirEnt*>(m.dir), m.masks,
                       m.vals, a.x, a.out, m.n_out, m.k_in, a.k_tok, m.n_strips, m.n_tiles, tpw);
    return hipGetLastError();
}

template <int MAXCH>
static hipError_t launch_sparse_valu_t(const MatArgs& m, const LinArgs& a, hipStream_t s) {
    const int tpw = tiles_per_wave_for(m.n_tiles, 16);
    const int waves = (m.n_tiles + tpw - 1) / tpw;
    const dim3 grid((unsigned)((waves + kWavesPerBlock - 1) / kWavesPerBlock)), block(64 * kWavesPerBlock);
    const size_t lds = (size_t)kWavesPerBlock * (MAXCH * 1024 + kValuTok * 512);
    hipLaunchKernelGGL((sparse_linear_valu_kernel<MAXCH>), grid, block, lds, s, static_cast<const DirEnt*>(m.dir), m.masks,
                       m.vals, a.x, a.out, m.n_out, m.k_in, a.k_tok, m.n_strips, m.n_tiles, tpw);
    return hipGetLastError();
}

bool sparse_linear_valu_supported(const MatArgs& m, int k_tok) {
    return k_tok >= 1 && k_tok <= kValuTok && (m.k_in & 7) == 0 && m.max_tile_nnz * 2 + 8 <= 5 * 1024;
}

hipError_t launch_sparse_linear_valu(const MatArgs& m, const LinArgs& a, hipStream_t s) {
    if (!sparse_linear_valu_supported(m, a.k_tok)) return hipErrorInvalidValue;
    return launch_sparse_valu_t<5>(m, a, s);
}

// Slabs per wavefront and wavefronts per workgroup of the kernel that writes final results.  Up to 16 tokens: one
// slab per wavefront up to 16 slabs, two beyond (then with 16 wavefronts).  More tokens need more registers per
// wavefront, so at most 12 wavefronts share a compute unit and take up to four slabs each.  More than 32 (48) slabs
// or tiles too dense for the 5 KiB buffers go to the kernel with partial sums.
static bool strip_shape(int n_slabs, int tg, int& spw, int& waves) {
    if (n_slabs < 1 || tg < 1 || tg > 4) return false;
    if (tg == 1) {
        if (n_slabs > 32) return false;
        spw = n_slabs <= 16 ? 1 : 2;
    } else {
        if (n_slabs > 48) return false;
        spw = (n_slabs + 11) / 12;
    }
    const int need = (n_slabs + spw - 1) / spw;
    waves = std::max(4, (need + 3) / 4 * 4);
    return true;
}

bool sparse_strip_supported(const MatArgs& m, int k_tok) {
    int spw, waves;
    return k_tok >= 1 && k_tok <= 64 && (m.max_tile_nnz * 2 + 8 + 1023) / 1024 <= 5 &&
           strip_shape(m.n_slabs, (k_tok + 15) / 16, spw, waves);
}

template <int SPW, int WAVES, int TG, bool GATED = false>
static hipError_t launch_strip_t(const MatArgs& m, const LinArgs& a, hipStream_t s, int passes = 1) {
    constexpr int kCh = 5;
    constexpr int kRound = strip_round(TG, GATED);
    const size_t lds = (size_t)WAVES * kCh * 1024 + (size_t)kRound * TG * WAVES * 256 * sizeof(float);
    static std::atomic<int> cached{0};  // workgroups resident on the chip; threads that race here compute the same value
    int resident = cached.load(std::memory_order_acquire);
    if (resident == 0) {
        const void* fn = reinterpret_cast<const void*>(sparse_strip_kernel<kCh, SPW, WAVES, TG, GATED>);
        int per_cu = 0;
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return hipErrorInvalidValue;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 64 * WAVES, lds) != hipSuccess || per_cu < 1) per_cu = 1;
        resident = device_cu_count() * per_cu;
        cached.store(resident, std::memory_order_release);
    }
    const int grid = std::min(GATED ? m.n_strips / 2 : m.n_strips, resident);
    hipLaunchKernelGGL((sparse_strip_kernel<kCh, SPW, WAVES, TG, GATED>), dim3((unsigned)grid, (unsigned)passes), dim3(64 * WAVES), lds, s,
                       static_cast<const DirEnt*>(m.dir), m.masks, m.vals, a.x, a.out, m.n_out, m.k_in, a.k_tok, m.n_strips, m.n_slabs);
    return hipGetLastError();
}

// y[t][n] final (every entry written), k_tok <= 64; sparse_strip_supported(m, k_tok) must hold
hipError_t launch_sparse_strip_linear(const MatArgs& m, const LinArgs& a, hipStream_t s) {
    int spw, waves;
    const int tg = (a.k_tok + 15) / 16;
    if (!sparse_strip_supported(m, a.k_tok) || !strip_shape(m.n_slabs, tg, spw, waves)) return hipErrorInvalidValue;
    // (a matrix with at most one strip per compute unit is timed by its start-up, not by its stream: one pass then)
    const bool few_strips = m.n_strips <= device_cu_count();
    if (tg > 2 && spw == 1 && !few_strips) {
        // One slab per wavefront: two token groups' activation columns fit its registers for the whole kernel, more do
        // not, and fetching them per step costs more than streaming the matrix again: 32 tokens per pass.
        // (both passes in one launch: the grid's second dimension)
        if (waves == 4) return launch_strip_t<1, 4, 2>(m, a, s, 2);
        if (waves == 8) return launch_strip_t<1, 8, 2>(m, a, s, 2);
        if (waves == 12) return launch_strip_t<1, 12, 2>(m, a, s, 2);
        return hipErrorInvalidValue;
    }
#define SD2_STRIP_CASE(S, W, T) \
    if (spw == S && waves == W && tg == T) return launch_strip_t<S, W, T>(m, a, s)
    SD2_STRIP_CASE(1, 4, 1);
    SD2_STRIP_CASE(1, 8, 1);
    SD2_STRIP_CASE(1, 12, 1);
    SD2_STRIP_CASE(1, 16, 1);
    SD2_STRIP_CASE(2, 12, 1);
    SD2_STRIP_CASE(2, 16, 1);
    SD2_STRIP_CASE(1, 4, 2);
    SD2_STRIP_CASE(1, 8, 2);
    SD2_STRIP_CASE(1, 12, 2);
    SD2_STRIP_CASE(1, 4, 3);
    SD2_STRIP_CASE(1, 8, 3);
    SD2_STRIP_CASE(1, 12, 3);
    SD2_STRIP_CASE(1, 4, 4);
    SD2_STRIP_CASE(1, 8, 4);
    SD2_STRIP_CASE(1, 12, 4);
#define SD2_STRIP_WIDE(T) \
    SD2_STRIP_CASE(2, 8, T); \
    SD2_STRIP_CASE(2, 12, T); \
    SD2_STRIP_CASE(3, 12, T); \
    SD2_STRIP_CASE(4, 12, T)
    SD2_STRIP_WIDE(2);
    SD2_STRIP_WIDE(3);
    SD2_STRIP_WIDE(4);
#undef SD2_STRIP_WIDE
#undef SD2_STRIP_CASE
    return hipErrorInvalidValue;
}

// The gated product of a fused [gate; up] matrix in one launch: m_out [k_tok][n_out / 2] bf16 = bf16(silu(gate x) * (up x)).
// One slab per wavefront (k_in <= 3072 for more than 16 tokens, <= 4096 else), whole strips per half.
bool sparse_strip_gated_supported(const MatArgs& m, int k_tok) {
    int spw, waves;
    return sparse_strip_supported(m, k_tok) && strip_shape(m.n_slabs, std::min((k_tok + 15) / 16, 2), spw, waves) && spw == 1 &&
           m.n_out % 32 == 0;
}

hipError_t launch_sparse_strip_gated(const MatArgs& m, const uint16_t* x, int k_tok, uint16_t* m_out, hipStream_t s) {
    if (!sparse_strip_gated_supported(m, k_tok)) return hipErrorInvalidValue;
    int spw, waves;
    const int tg = std::min((k_tok + 15) / 16, 2);
    strip_shape(m.n_slabs, tg, spw, waves);
    const LinArgs a{x, k_tok, reinterpret_cast<float*>(m_out)};
    if (k_tok > 32) {  // 32 tokens per pass, as for the plain product; both passes in one launch
        if (waves == 4) return launch_strip_t<1, 4, 2, true>(m, a, s, 2);
        if (waves == 8) return launch_strip_t<1, 8, 2, true>(m, a, s, 2);
        if (waves == 12) return launch_strip_t<1, 12, 2, true>(m, a, s, 2);
        return hipErrorInvalidValue;
    }
#define SD2_GATED_CASE(W, T) \
    if (waves == W && tg == T) return launch_strip_t<1, W, T, true>(m, a, s)
    SD2_GATED_CASE(4, 1);
    SD2_GATED_CASE(8, 1);
    SD2_GATED_CASE(12, 1);
    SD2_GATED_CASE(16, 1);
    SD2_GATED_CASE(4, 2);
    SD2_GATED_CASE(8, 2);
    SD2_GATED_CASE(12, 2);
#undef SD2_GATED_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_sparse_linear(const MatArgs& m, const LinArgs& a, hipStream_t s) {
    const int tg = (a.k_tok + 15) / 16;
    // LDS pieces per tile: 2 bytes per value plus 8 bytes of slack, in 1 KiB chunks per wavefront
    const int chunks = (m.max_tile_nnz * 2 + 8 + 1023) / 1024;
    if (chunks <= 5) {
        if (tg == 1) return launch_sparse_t<5, 1>(m, a, s);
        if (tg == 2) return launch_sparse_t<5, 2>(m, a, s);
        return launch_sparse_t<5, 4>(m, a, s);
    }
    if (tg == 1) return launch_sparse_t<9, 1>(m, a, s);
    if (tg == 2) return launch_sparse_t<9, 2>(m, a, s);
    return launch_sparse_t<9, 4>(m, a, s);
}

template <int TG>
static hipError_t launch_dense_t(const MatArgs& m, const LinArgs& a, hipStream_t s) {
    const int tpw = tiles_per_wave_for(m.n_tiles, 16);
    const int waves = (m.n_tiles + tpw - 1) / tpw;
    const dim3 grid((unsigned)((waves + kWavesPerBlock - 1) / kWavesPerBlock)), block(64 * kWavesPerBlock);
    hipLaunchKernelGGL((dense_linear_kernel<TG>), grid, block, 0, s, m.w, a.x, a.out, m.n_out, m.k_in, a.k_tok, m.n_strips,
                       m.n_tiles, tpw);
    return hipGetLastError();
}

hipError_t launch_dense_linear(const MatArgs& m, const LinArgs& a, hipStream_t s) {
    const int tg = (a.k_tok + 15) / 16;
    if (tg == 1) return launch_dense_t<1>(m, a, s);
    if (tg == 2) return launch_dense_t<2>(m, a, s);
    return launch_dense_t<4>(m, a, s);
}

// ------------------------------------------------------------------ masked gradient (sparse fine-tuning)
// Sec. 2.4: the mask is fixed and the gradients of pruned parameters are set to zero.  One thread owns eight
// consecutive columns of a row (consecutive threads: consecutive chunks, so loads and stores are full runs); its
// eight mask bits are one byte of the blob's mask section (tile, lane, 64-column step).  Selection, not a product.
template <typename T>
__global__ __launch_bounds__(256) void mask_gradient_kernel(const uint16_t* __restrict__ masks, T* __restrict__ grad,
                                                            int n_out, int k_in, int n_strips) {
    const size_t chunks_per_row = (size_t)k_in / 8;
    const size_t n_chunks = (size_t)n_out * chunks_per_row;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_chunks; i += (size_t)gridDim.x * 256) {
        const uint32_t row = (uint32_t)(i / chunks_per_row), col = (uint32_t)(i % chunks_per_row) * 8;
        const uint32_t tile = (col >> 8) * (uint32_t)n_strips + (row >> 4);
        const uint32_t lane = (row & 15u) + 16u * ((col & 63u) >> 4), q = (col & 255u) >> 6;
        const uint32_t bits = ((uint32_t)masks[(size_t)tile * 256 + lane * 4 + q] >> (col & 8u)) & 0xffu;
        T* p = grad + (size_t)row * k_in + col;
        if (sizeof(T) == 4) {
            u32x4 lo = reinterpret_cast<u32x4*>(p)[0], hi = reinterpret_cast<u32x4*>(p)[1];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                lo[b] = (bits >> b) & 1u ? lo[b] : 0u;
                hi[b] = (bits >> (4 + b)) & 1u ? hi[b] : 0u;
            }
            reinterpret_cast<u32x4*>(p)[0] = lo;
            reinterpret_cast<u32x4*>(p)[1] = hi;
        } else {
            u32x4 v = *reinterpret_cast<u32x4*>(p);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const uint32_t keep = ((bits >> (2 * b)) & 1u ? 0x0000ffffu : 0u) | ((bits >> (2 * b + 1)) & 1u ? 0xffff0000u : 0u);
                v[b] &= keep;
            }
            *reinterpret_cast<u32x4*>(p) = v;
        }
    }
}

hipError_t launch_mask_gradient(const MatArgs& m, void* grad, bool bf16, hipStream_t s) {
    const size_t n_chunks = (size_t)m.n_out * (size_t)(m.k_in / 8);
    const unsigned grid = (unsigned)std::min<size_t>((n_chunks + 255) / 256, (size_t)device_cu_count() * 16);
    const uint16_t* masks = reinterpret_cast<const uint16_t*>(m.masks);
    if (bf16)
        hipLaunchKernelGGL(mask_gradient_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, masks, static_cast<uint16_t*>(grad),
                           m.n_out, m.k_in, m.n_strips);
    else
        hipLaunchKernelGGL(mask_gradient_kernel<uint32_t>, dim3(grid), dim3(256), 0, s, masks, static_cast<uint32_t*>(grad),
                           m.n_out, m.k_in, m.n_strips);
    return hipGetLastError();
}

// ------------------------------------------------------------------ drafting round: embedding rows, flag folding
// h_in[j] = E[id_j] for the round's window: id_0 = *start, id_j = drafts[j - 1].  Ids outside [0, vocab) are clamped
// (they cannot be reported from the device).  One workgroup per window position, 16 bytes per thread and step.
__global__ __launch_bounds__(256) void embed_window_kernel(const uint16_t* __restrict__ emb, int vocab, int hidden,
                                                           const int32_t* __restrict__ start,
                                                           const int32_t* __restrict__ drafts, uint16_t* __restrict__ h_in) {
    const int j = blockIdx.x;
    int id = j == 0 ? start[0] : drafts[j - 1];
    id = min(max(id, 0), vocab - 1);
    const u32x4* src = reinterpret_cast<const u32x4*>(emb + (size_t)id * hidden);
    u32x4* dst = reinterpret_cast<u32x4*>(h_in + (size_t)j * hidden);
    for (int c = threadIdx.x; c < hidden / 8; c += 256) dst[c] = src[c];
}

// *acc |= *flag (keeps a give-up flag of one forward beyond the next forward's set-up); flag == nullptr: *acc = 0
__global__ void fold_flag_kernel(const unsigned* __restrict__ flag, unsigned* __restrict__ acc) {
    if (threadIdx.x != 0) return;
    if (!flag)
        *acc = 0u;
    else if (*flag)
        *acc = 1u;
}

hipError_t launch_embed_window(const uint16_t* emb, int vocab, int hidden, const int32_t* start, const int32_t* drafts,
                               int n_tok, uint16_t* h_in, hipStream_t s) {
    hipLaunchKernelGGL(embed_window_kernel, dim3((unsigned)n_tok), dim3(256), 0, s, emb, vocab, hidden, start, drafts, h_in);
    return hipGetLastError();
}

hipError_t launch_fold_flag(const unsigned* flag, unsigned* acc, hipStream_t s) {
    hipLaunchKernelGGL(fold_flag_kernel, dim3(1), dim3(64), 0, s, flag, acc);
    return hipGetLastError();
}

// ------------------------------------------------------------------ one-shot magnitude pruning
// Sec. 2.3 prunes every decoder linear one-shot to a uniform sparsity.  Criterion here: weight magnitude; ties go
// to the lower column; pruned entries become +0.  bf16 magnitudes order like their low 15 bits, so the threshold
// of a row is found exactly by a two-level radix select (256 + 128 bins in LDS), and the ties at the threshold are
// resolved in column order with a prefix count: thread i owns the contiguous columns [i cpt, (i + 1) cpt).
constexpr int kPruneThreads = 256;
constexpr int kPruneMaxPerThread = 36;  // k_in <= 9216

__global__ __launch_bounds__(kPruneThreads) void prune_rows_kernel(uint16_t* __restrict__ w, int n_out, int k_in, int n_keep) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t scan[kPruneThreads];
    __shared__ uint32_t pick[2];  // chosen bin, entries strictly above it
    const int tid = threadIdx.x;
    const int cpt = k_in / kPruneThreads;  // k_in is a multiple of 256 here
    for (int row = blockIdx.x; row < n_out; row += gridDim.x) {
        uint16_t* wr = w + (size_t)row * k_in + (size_t)tid * cpt;
        uint16_t v[kPruneMaxPerThread];
#pragma unroll
        for (int i = 0; i < kPruneMaxPerThread; ++i) v[i] = i < cpt ? wr[i] : (uint16_t)0;
        uint32_t above = 0;  // entries with a magnitude above the bins examined so far
        uint32_t prefix = 0, prefix_mask = 0;  // magnitude bits fixed so far
        // level 0: bits 14..7 (256 bins); level 1: bits 6..0 (128 bins) among the entries of the chosen bin
#pragma unroll 1
        for (int level = 0; level < 2; ++level) {
            const int shift = level ? 0 : 7;
            const uint32_t bins = level ? 128u : 256u;
            hist[tid] = 0;
            __syncthreads();
#pragma unroll
            for (int i = 0; i < kPruneMaxPerThread; ++i)
                if (i < cpt) {
                    const uint32_t m = v[i] & 0x7fffu;
                    if ((m & prefix_mask) == prefix) atomicAdd(&hist[(m >> shift) & (bins - 1)], 1u);
                }
            __syncthreads();
            if (tid == 0) {  // walk down from the largest bin until n_keep entries are covered
                uint32_t acc = above, b = bins;
                while (b > 0 && acc + hist[b - 1] < (uint32_t)n_keep) acc += hist[--b];
                pick[0] = b > 0 ? b - 1 : 0u;  // the bin that holds the threshold
                pick[1] = acc;
            }
            __syncthreads();
            prefix |= pick[0] << shift;
            prefix_mask |= (bins - 1) << shift;
            above = pick[1];
            __syncthreads();
        }
        const uint32_t thr = prefix;                   // magnitude of the last kept entry
        const uint32_t ties_kept = (uint32_t)n_keep - above;  // entries equal to it that stay, in column order
        uint32_t mine = 0;
#pragma unroll
        for (int i = 0; i < kPruneMaxPerThread; ++i)
            if (i < cpt && (uint32_t)(v[i] & 0x7fffu) == thr) ++mine;
        scan[tid] = mine;
        __syncthreads();
        if (tid == 0) {  // exclusive prefix of the tie counts (256 entries: a serial pass is cheap next to the row's traffic)
            uint32_t run = 0;
            for (int t = 0; t < kPruneThreads; ++t) {
                const uint32_t c = scan[t];
                scan[t] = run;
                run += c;
            }
        }
        __syncthreads();
        uint32_t seen = scan[tid];
#pragma unroll
        for (int i = 0; i < kPruneMaxPerThread; ++i)
            if (i < cpt) {
                const uint32_t m = v[i] & 0x7fffu;
                bool keep = m > thr;
                if (m == thr) keep = seen++ < ties_kept;
                if (!keep) wr[i] = 0;
            }
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void prune_2of4_kernel(uint16_t* __restrict__ w, size_t n_groups) {
    for (size_t gidx = (size_t)blockIdx.x * 256 + threadIdx.x; gidx < n_groups; gidx += (size_t)gridDim.x * 256) {
        uint2 raw = reinterpret_cast<uint2*>(w)[gidx];
        uint32_t v[4] = {raw.x & 0xffffu, raw.x >> 16, raw.y & 0xffffu, raw.y >> 16};
        // rank of each entry: how many others beat it (larger magnitude, or equal magnitude at a lower column)
        uint32_t out[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t rank = 0;
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                const uint32_t mc = v[c] & 0x7fffu, mo = v[o] & 0x7fffu;
                rank += (o != c && (mo > mc || (mo == mc && o < c))) ? 1u : 0u;
            }
            out[c] = rank < 2 ? v[c] : 0u;
        }
        reinterpret_cast<uint2*>(w)[gidx] = make_uint2(out[0] | (out[1] << 16), out[2] | (out[3] << 16));
    }
}

hipError_t launch_prune_rows(uint16_t* w, int n_out, int k_in, int n_keep, hipStream_t s) {
    const unsigned grid = (unsigned)std::min(n_out, device_cu_count() * 8);
    hipLaunchKernelGGL(prune_rows_kernel, dim3(grid), dim3(kPruneThreads), 0, s, w, n_out, k_in, n_keep);
    return hipGetLastError();
}

hipError_t launch_prune_2of4(uint16_t* w, int n_out, int k_in, hipStream_t s) {
    const size_t n_groups = (size_t)n_out * (size_t)(k_in / 4);
    const unsigned grid = (unsigned)std::min<size_t>((n_groups + 255) / 256, (size_t)device_cu_count() * 16);
    hipLaunchKernelGGL(prune_2of4_kernel, dim3(grid), dim3(256), 0, s, w, n_groups);
    return hipGetLastError();
}

// ------------------------------------------------------------------ glue

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ part, int n_splits, size_t split_stride,
                                                             size_t n, float* __restrict__ y) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float acc = 0.f;
    for (int s = 0; s < n_splits; ++s) acc += part[(size_t)s * split_stride + i];
    y[i] = acc;
}

hipError_t launch_reduce_partials_strided(const float* part, int n_splits, size_t split_stride, size_t n, float* y,
                                          hipStream_t s) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, part, n_splits,
                       split_stride, n, y);
    return hipGetLastError();
}

hipError_t launch_reduce_partials(const float* part, int n_splits, size_t n, float* y, hipStream_t s) {
    return launch_reduce_partials_strided(part, n_splits, n, n, y, s);
}

// ------------------------------------------------------------------ static scratch for callers that cannot allocate
//
// Device memory that belongs to the library's code object: every GPU the library runs on holds its own copy of this
// array, at its own address, until the process ends.  In host code the array's name is only a handle for the
// symbol; the device address is looked up once per device (with that device current) and kept, and only that
// address is ever handed to kernels.  The contents survive from call to call; the linear that uses it overwrites
// every partial result it later reads, so nothing has to be cleared.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t static_scratch(void** ptr_out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> per_device[kMaxDevices];  // zero-initialised; threads that race here store the same address
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = per_device[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev].store(p, std::memory_order_release);
    }
    *ptr_out = p;
    return hipSuccess;
}

__device__ __forceinline__ float block_sum_256(float v, float* red) {
    const int tid = threadIdx.x;
    red[tid] = v;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off) red[tid] += red[tid + off];
        __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
}

// Sum of n_splits partial results, four independent chains so that the loads overlap.
__device__ __forceinline__ float sum_splits(const float* __restrict__ p, int n_splits, size_t stride) {
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    int s = 0;
    for (; s + 4 <= n_splits; s += 4) {
        a0 += p[(size_t)s * stride];
        a1 += p[(size_t)(s + 1) * stride];
        a2 += p[(size_t)(s + 2) * stride];
        a3 += p[(size_t)(s + 3) * stride];
    }
    for (; s < n_splits; ++s) a0 += p[(size_t)s * stride];
    return (a0 + a1) + (a2 + a3);
}

// Step 1 of the residual update: block (c, t) owns 256 columns of token t.  h is initialised from bf16 h_in or
// updated with the sum of the partials; the block's sum of squares goes to ssq[t][c].
__global__ __launch_bounds__(256) void residual_update_kernel(float* __restrict__ h, const uint16_t* __restrict__ h_in,
                                                             const float* __restrict__ part, int n_splits, int k_tok,
                                                             int hidden, float* __restrict__ ssq) {
    __shared__ float red[256];
    const int t = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    float v = 0.f;
    if (i < hidden) {
        const size_t at = (size_t)t * hidden + i;
        v = h_in ? bf16_to_f32(h_in[at]) : h[at] + sum_splits(part + at, n_splits, (size_t)k_tok * hidden);
        h[at] = v;
    }
    const float tot = block_sum_256(v * v, red);
    if (threadIdx.x == 0) ssq[(size_t)t * gridDim.x + blockIdx.x] = tot;
}

// Step 2: a = bf16(h / sqrt(mean(h^2) + 1e-5)), the mean taken from the per-block sums of step 1.
__global__ __launch_bounds__(256) void rmsnorm_apply_kernel(const float* __restrict__ h, const float* __restrict__ ssq,
                                                           int hidden, uint16_t* __restrict__ a) {
    const int t = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    float tot = 0.f;
    for (unsigned c = 0; c < gridDim.x; ++c) tot += ssq[(size_t)t * gridDim.x + c];  // same order in every thread
    const float inv = 1.0f / sqrtf(tot / (float)hidden + 1e-5f);
    if (i < hidden) a[(size_t)t * hidden + i] = f32_to_bf16(h[(size_t)t * hidden + i] * inv);
}

// Both steps in one launch for hidden <= 16384: one workgroup of 1024 threads per token keeps its columns in registers
// between the residual update, the sum of squares (cross-lane sums, then the 16 wavefronts' totals in a fixed order)
// and the normalisation.
constexpr int kRnThreads = 1024, kRnCols = 16;

__global__ __launch_bounds__(kRnThreads) void residual_norm_kernel(float* __restrict__ h, const uint16_t* __restrict__ h_in,
                                                                  const float* __restrict__ part, int n_splits, int k_tok,
                                                                  int hidden, uint16_t* __restrict__ a) {
    __shared__ float wave_tot[kRnThreads / 64];
    const int t = blockIdx.x, tid = threadIdx.x;
    float v[kRnCols];
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < kRnCols; ++j) {
        const int i = tid + j * kRnThreads;
        v[j] = 0.f;
        if (i < hidden) {
            const size_t at = (size_t)t * hidden + i;
            v[j] = h_in ? bf16_to_f32(h_in[at]) : h[at] + sum_splits(part + at, n_splits, (size_t)k_tok * hidden);
            h[at] = v[j];
            ss += v[j] * v[j];
        }
    }
    if (!a) return;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((tid & 63) == 0) wave_tot[tid >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kRnThreads / 64; ++w) tot += wave_tot[w];
    const float inv = 1.0f / sqrtf(tot / (float)hidden + 1e-5f);
#pragma unroll
    for (int j = 0; j < kRnCols; ++j) {
        const int i = tid + j * kRnThreads;
        if (i < hidden) a[(size_t)t * hidden + i] = f32_to_bf16(v[j] * inv);
    }
}

hipError_t launch_residual_rmsnorm(float* h, const uint16_t* h_in, const float* part, int n_splits, int k_tok,
                                   int hidden, uint16_t* a, float* ssq, hipStream_t s) {
    if (hidden <= kRnThreads * kRnCols) {
        hipLaunchKernelGGL(residual_norm_kernel, dim3((unsigned)k_tok), dim3(kRnThreads), 0, s, h, h_in, part, n_splits, k_tok, hidden, a);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)((hidden + 255) / 256), (unsigned)k_tok);
    hipLaunchKernelGGL(residual_update_kernel, grid, dim3(256), 0, s, h, h_in, part, n_splits, k_tok, hidden, ssq);
    if (a) hipLaunchKernelGGL(rmsnorm_apply_kernel, grid, dim3(256), 0, s, h, ssq, hidden, a);
    return hipGetLastError();
}

// Causal softmax attention among the k_tok <= 64 in-flight tokens: one workgroup of two wavefronts per (head, query
// token i).  Scores: lane j of each wavefront owns key j <= i and half of the head's dimensions (its key row is
// contiguous in memory: 16-byte loads), the halves meet in LDS; softmax over the 64 lanes of one wavefront by
// cross-lane maxima and sums; output: thread d owns dimension d and walks the values of tokens 0..i (coalesced).
__global__ __launch_bounds__(128) void inflight_attention_kernel(const float* __restrict__ part, int n_splits, int k_tok,
                                                                int q_out, int kv_out, int n_heads, int n_kv, int D,
                                                                uint16_t* __restrict__ ctx) {
    __shared__ __attribute__((aligned(16))) float sq[256];  // the query (head_dim <= 256)
    __shared__ float sc[2][64];                             // each wavefront's share of the scores
    __shared__ float sp[64];                                // probabilities
    const int head = blockIdx.x, i = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int grp = head / (n_heads / n_kv);
    const int n_out = q_out + 2 * kv_out;
    const size_t stride = (size_t)k_tok * n_out;
    for (int d = tid; d < D; d += 128) sq[d] = sum_splits(part + (size_t)i * n_out + head * D + d, n_splits, stride);
    __syncthreads();
    const int half = D / 2;  // a multiple of 4 (head_dim is a multiple of 8)
    float dot = 0.f;
    if (lane <= i) {
        const float* kr = part + (size_t)lane * n_out + q_out + grp * D + w * half;
        const float* qh = sq + w * half;
        if (n_splits == 1) {
            // final values: sixteen 16-byte loads of the key row in flight at a time -- a loop that uses each load before it
            // issues the next pays the latency of the caches sixteen times over
            for (int d0 = 0; d0 < half; d0 += 64) {
                float4 kk[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int d = d0 + 4 * u;
                    kk[u] = d < half ? *reinterpret_cast<const float4*>(kr + d) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int d = min(d0 + 4 * u, half - 4);  // (a clamped index multiplies zeros)
                    const float4 qq = *reinterpret_cast<const float4*>(qh + d);
                    dot += qq.x * kk[u].x + qq.y * kk[u].y + qq.z * kk[u].z + qq.w * kk[u].w;
                }
            }
        } else {  // partial sums of a split contraction
            for (int d = 0; d < half; d += 4) {
                float4 kk = *reinterpret_cast<const float4*>(kr + d);
                for (int sp_i = 1; sp_i < n_splits; ++sp_i) {
                    const float4 more = *reinterpret_cast<const float4*>(kr + (size_t)sp_i * stride + d);
                    kk.x += more.x;
                    kk.y += more.y;
                    kk.z += more.z;
                    kk.w += more.w;
                }
                const float4 qq = *reinterpret_cast<const float4*>(qh + d);
                dot += qq.x * kk.x + qq.y * kk.y + qq.z * kk.z + qq.w * kk.w;
            }
        }
    }
    sc[w][lane] = dot;
    __syncthreads();
    if (w == 0) {
        const bool on = lane <= i;
        const float s = on ? (sc[0][lane] + sc[1][lane]) * (1.0f / sqrtf((float)D)) : -INFINITY;
        float mx = s;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        const float e = on ? expf(s - mx) : 0.f;
        float sum = e;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        sp[lane] = e / sum;
    }
    __syncthreads();
    for (int d = tid; d < D; d += 128) {
        const float* vr = part + q_out + kv_out + grp * D + d;
        float o = 0.f;
        if (n_splits == 1) {  // final values: plain loads, sixteen in flight; the products are added in token order
            for (int j0 = 0; j0 <= i; j0 += 16) {
                float v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = j0 + u <= i ? vr[(size_t)(j0 + u) * n_out] : 0.f;
#pragma unroll
                for (int u = 0; u < 16; ++u) o += sp[min(j0 + u, 63)] * v[u];
            }
        } else {
            for (int j = 0; j <= i; ++j) o += sp[j] * sum_splits(vr + (size_t)j * n_out, n_splits, stride);
        }
        ctx[(size_t)i * q_out + head * D + d] = f32_to_bf16(o);
    }
}

hipError_t launch_inflight_attention(const float* part, int n_splits, int k_tok, int q_out, int kv_out, int n_heads,
                                     int n_kv, int head_dim, uint16_t* ctx, hipStream_t s) {
    if (k_tok < 1 || k_tok > 64 || head_dim < 8 || head_dim > 256 || head_dim % 8) return hipErrorInvalidValue;
    hipLaunchKernelGGL(inflight_attention_kernel, dim3((unsigned)n_heads, (unsigned)k_tok), dim3(128), 0, s, part, n_splits, k_tok,
                       q_out, kv_out, n_heads, n_kv, head_dim, ctx);
    return hipGetLastError();
}

// ------------------------------------------------------------------ decode step: rotary embedding, key/value cache
//
// The drafter conditions every candidate on the prompt and the candidates before it (Sec. 2); for the Llama / Qwen
// decoders of Sec. 3 that is rotary position embedding on queries and keys and attention over the cached keys and
// values of all earlier positions.  Half-split pairing: dimension i < D/2 of a head rotates with dimension i + D/2 by
// the angle position * theta^(-2 i / D).  The cache holds bf16: rotated keys, plain values.

// cos and sin of the angles of the call's tokens, [k_tok][D/2].  Double precision: positions reach thousands of
// radians, where a float product has already lost the low bits of the angle.
__global__ __launch_bounds__(256) void rope_table_kernel(int pos0, int k_tok, int D, double theta, float2* __restrict__ table) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int half = D / 2;
    if (idx >= k_tok * half) return;
    const int t = idx / half, i = idx % half;
    const double ang = (double)(pos0 + t) * pow(theta, -2.0 * (double)i / (double)D);
    table[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

hipError_t launch_rope_table(int pos0, int k_tok, int head_dim, double theta, float2* table, hipStream_t s) {
    const int n = k_tok * (head_dim / 2);
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, pos0, k_tok, head_dim, theta, table);
    return hipGetLastError();
}

// Block (head slot, token): slots below n_heads are query heads (summed from the split-K partials, rotated, kept as
// fp32 in q_rot [k_tok][q_out]); the others are key/value heads (key rotated, both rounded to bf16 and written to
// position pos0 + token of the layer's caches [n_kv][max_pos][D]).  Thread i < D/2 owns the pair (i, i + D/2).
__global__ __launch_bounds__(128) void rope_append_kernel(const float* __restrict__ part, int n_splits, int k_tok, int q_out,
                                                         int kv_out, int n_heads, int D, const float2* __restrict__ table,
                                                         int pos0, int max_pos, float* __restrict__ q_rot,
                                                         uint16_t* __restrict__ k_cache, uint16_t* __restrict__ v_cache) {
    const int slot = blockIdx.x, t = blockIdx.y, i = threadIdx.x, half = D / 2;
    if (i >= half) return;
    const int n_out = q_out + 2 * kv_out;
    const size_t stride = (size_t)k_tok * n_out;
    const float* row = part + (size_t)t * n_out;
    const float2 cs = table[t * half + i];
    if (slot < n_heads) {
        const float lo = sum_splits(row + slot * D + i, n_splits, stride);
        const float hi = sum_splits(row + slot * D + half + i, n_splits, stride);
        float* dst = q_rot + (size_t)t * q_out + slot * D;
        dst[i] = lo * cs.x - hi * cs.y;
        dst[half + i] = hi * cs.x + lo * cs.y;
    } else {
        const int g = slot - n_heads;
        const float lo = sum_splits(row + q_out + g * D + i, n_splits, stride);
        const float hi = sum_splits(row + q_out + g * D + half + i, n_splits, stride);
        const float v0 = sum_splits(row + q_out + kv_out + g * D + i, n_splits, stride);
        const float v1 = sum_splits(row + q_out + kv_out + g * D + half + i, n_splits, stride);
        const size_t at = ((size_t)g * max_pos + (size_t)(pos0 + t)) * D;
        k_cache[at + i] = f32_to_bf16(lo * cs.x - hi * cs.y);
        k_cache[at + half + i] = f32_to_bf16(hi * cs.x + lo * cs.y);
        v_cache[at + i] = f32_to_bf16(v0);
        v_cache[at + half + i] = f32_to_bf16(v1);
    }
}

hipError_t launch_rope_append(const float* part, int n_splits, int k_tok, int q_out, int kv_out, int n_heads, int n_kv,
                              int head_dim, const float2* table, int pos0, int max_pos, float* q_rot, uint16_t* k_cache,
                              uint16_t* v_cache, hipStream_t s) {
    if (head_dim < 2 || head_dim > 256 || (head_dim & 1)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rope_append_kernel, dim3((unsigned)(n_heads + n_kv), (unsigned)k_tok), dim3(128), 0, s, part, n_splits,
                       k_tok, q_out, kv_out, n_heads, head_dim, table, pos0, max_pos, q_rot, k_cache, v_cache);
    return hipGetLastError();
}

constexpr int kAttMaxRep = 8;  // query heads per key/value head

constexpr int kAttWaves = 16;  // wavefronts per attention block

// LDS of the attention kernel in floats: scores [rep][n_max], per-wavefront partial outputs [waves][rep][D], inverse sums
static size_t cached_attention_lds(int rep, int D, int n_max) {
    return ((size_t)rep * n_max + (size_t)kAttWaves * rep * D + kAttMaxRep) * sizeof(float);
}

__device__ __forceinline__ void bf16x8_to_f32(const u32x4 w, float (&f)[8]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = __uint_as_float(w[e] << 16);
        f[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
}

// Block (key/value head g, token t): the rep query heads of the group attend to cache positions 0 .. pos0 + t.
// A cache row (one position, D = 8 LPR bf16) is read by LPR consecutive lanes, 16 bytes each, so a wavefront reads
// 64 / LPR consecutive positions = one contiguous KiB per load instruction, and the block's sixteen wavefronts
// cover 1024 / LPR positions per pass; four passes of loads are in flight at once.  Scores: each lane multiplies its eight
// dimensions with the queries it holds in registers, the LPR lanes of a row add up across lanes.  Softmax: one
// wavefront per head over the scores in LDS.  Values: each lane accumulates its eight dimensions over the rows it
// reads; the row slots of a wavefront add up across lanes, the wavefronts through LDS.
template <int LPR, int REP>
__global__ __launch_bounds__(64 * kAttWaves) void cached_attention_kernel(const float* __restrict__ q_rot, const uint16_t* __restrict__ k_cache,
                                                              const uint16_t* __restrict__ v_cache, int max_pos, int pos0,
                                                              int n_max, int q_out, int rep, uint16_t* __restrict__ ctx) {
    constexpr int D = 8 * LPR, RPW = 64 / LPR, RPI = kAttWaves * RPW, UNR = 4;
    extern __shared__ float smem[];
    const int g = blockIdx.x, t = blockIdx.y, tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int piece = lane % LPR, slot = wave * RPW + lane / LPR;  // 16-byte piece of a row, row slot within a pass
    const int n = pos0 + t + 1;
    float* sc = smem;                        // [rep][n_max]
    float* so = sc + (size_t)rep * n_max;    // [waves][rep][D]
    float* sinv = so + kAttWaves * rep * D;  // [kAttMaxRep]
    const u32x4* kg = reinterpret_cast<const u32x4*>(k_cache + (size_t)g * max_pos * D) + piece;
    const u32x4* vg = reinterpret_cast<const u32x4*>(v_cache + (size_t)g * max_pos * D) + piece;
    const float scale = 1.0f / sqrtf((float)D);

    float qr[REP][8];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        const float* src = q_rot + (size_t)t * q_out + ((size_t)g * rep + min(r, rep - 1)) * D + 8 * piece;
        const f32x4 lo = *reinterpret_cast<const f32x4*>(src), hi = *reinterpret_cast<const f32x4*>(src + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            qr[r][e] = lo[e] * scale;
            qr[r][4 + e] = hi[e] * scale;
        }
    }
    for (int j0 = 0; j0 < n; j0 += RPI * UNR) {
        u32x4 w[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int j = j0 + u * RPI + slot;
            w[u] = j < n ? kg[(size_t)j * LPR] : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int j = j0 + u * RPI + slot;
            float kf[8];
            bf16x8_to_f32(w[u], kf);
#pragma unroll
            for (int r = 0; r < REP; ++r) {
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) dot += kf[e] * qr[r][e];
#pragma unroll
                for (int o = 1; o < LPR; o <<= 1) dot += __shfl_xor(dot, o);
                if (piece == 0 && j < n && r < rep) sc[(size_t)r * n_max + j] = dot;
            }
        }
    }
    __syncthreads();
    for (int r = wave; r < rep; r += kAttWaves) {
        float* row = sc + (size_t)r * n_max;
        float mx = -3.0e38f;
        for (int j = lane; j < n; j += 64) mx = fmaxf(mx, row[j]);
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        float sum = 0.f;
        for (int j = lane; j < n; j += 64) {
            const float e = expf(row[j] - mx);
            row[j] = e;
            sum += e;
        }
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        if (lane == 0) sinv[r] = 1.0f / sum;
    }
    __syncthreads();
    float acc[REP][8];
#pragma unroll
    for (int r = 0; r < REP; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
    for (int j0 = 0; j0 < n; j0 += RPI * UNR) {
        u32x4 w[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int j = j0 + u * RPI + slot;
            w[u] = j < n ? vg[(size_t)j * LPR] : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int j = j0 + u * RPI + slot;
            if (j < n) {
                float vf[8];
                bf16x8_to_f32(w[u], vf);
#pragma unroll
                for (int r = 0; r < REP; ++r) {
                    const float p = sc[(size_t)min(r, rep - 1) * n_max + j];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[r][e] += p * vf[e];
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < REP; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[r][e];
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) v += __shfl_xor(v, o);
            if (lane < LPR && r < rep) so[(wave * rep + r) * D + 8 * piece + e] = v;
        }
    __syncthreads();
    for (int idx = tid; idx < rep * D; idx += 64 * kAttWaves) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < kAttWaves; ++w) o += so[w * rep * D + idx];
        ctx[(size_t)t * q_out + (size_t)g * rep * D + idx] = f32_to_bf16(o * sinv[idx / D]);
    }
}

bool cached_attention_supported(int n_heads, int n_kv, int head_dim, int max_pos) {
    if (n_kv < 1 || n_heads % n_kv || n_heads / n_kv > kAttMaxRep) return false;
    if (head_dim != 64 && head_dim != 128 && head_dim != 256) return false;
    return max_pos >= 1 && cached_attention_lds(n_heads / n_kv, head_dim, max_pos) <= 160 * 1024 - 256;
}

template <int LPR, int REP>
static hipError_t launch_cached_attention_t(const float* q_rot, const uint16_t* k_cache, const uint16_t* v_cache, int max_pos,
                                            int pos0, int k_tok, int q_out, int rep, int n_kv, uint16_t* ctx, hipStream_t s) {
    static std::atomic<bool> lds_raised{false};  // once, at the first call (a warm-up call precedes any graph capture)
    if (!lds_raised.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(cached_attention_kernel<LPR, REP>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256);
        if (e != hipSuccess) return e;
        lds_raised.store(true, std::memory_order_release);
    }
    const int n_max = pos0 + k_tok;
    hipLaunchKernelGGL((cached_attention_kernel<LPR, REP>), dim3((unsigned)n_kv, (unsigned)k_tok), dim3(64 * kAttWaves),
                       cached_attention_lds(rep, 8 * LPR, n_max), s, q_rot, k_cache, v_cache, max_pos, pos0, n_max, q_out, rep, ctx);
    return hipGetLastError();
}

hipError_t launch_cached_attention(const float* q_rot, const uint16_t* k_cache, const uint16_t* v_cache, int max_pos, int pos0,
                                   int k_tok, int q_out, int n_heads, int n_kv, int head_dim, uint16_t* ctx, hipStream_t s) {
    if (!cached_attention_supported(n_heads, n_kv, head_dim, max_pos) || pos0 < 0 || pos0 + k_tok > max_pos)
        return hipErrorInvalidValue;
    const int rep = n_heads / n_kv;
    // register arrays are sized for 4 or 8 query heads per key/value head
#define SD2_ATT_CASE(L) \
    if (head_dim == 8 * L) \
        return rep <= 4 ? launch_cached_attention_t<L, 4>(q_rot, k_cache, v_cache, max_pos, pos0, k_tok, q_out, rep, n_kv, ctx, s) \
                        : launch_cached_attention_t<L, 8>(q_rot, k_cache, v_cache, max_pos, pos0, k_tok, q_out, rep, n_kv, ctx, s)
    SD2_ATT_CASE(8);
    SD2_ATT_CASE(16);
    SD2_ATT_CASE(32);
#undef SD2_ATT_CASE
    return hipErrorInvalidValue;
}

__global__ __launch_bounds__(256) void silu_mul_kernel(const float* __restrict__ part, int n_splits, int k_tok, int inter,
                                                      uint16_t* __restrict__ mo) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t n = (size_t)k_tok * inter;
    if (i >= n) return;
    const int t = (int)(i / inter), j = (int)(i % inter);
    const size_t stride = (size_t)k_tok * 2 * inter;
    float gsum = 0.f, usum = 0.f;
    for (int s = 0; s < n_splits; ++s) {
        const float* p = part + (size_t)s * stride + (size_t)t * 2 * inter;
        gsum += p[j];
        usum += p[inter + j];
    }
    const float act = gsum / (1.0f + expf(-gsum));
    mo[i] = f32_to_bf16(act * usum);
}

hipError_t launch_silu_mul(const float* part, int n_splits, int k_tok, int inter, uint16_t* m, hipStream_t s) {
    const size_t n = (size_t)k_tok * inter;
    hipLaunchKernelGGL(silu_mul_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, part, n_splits, k_tok, inter, m);
    return hipGetLastError();
}

// ------------------------------------------------------------------ verification (Eq. 2)

__global__ __launch_bounds__(64) void greedy_verify_kernel(const int32_t* __restrict__ draft, const int32_t* __restrict__ target,
                                                          int batch, int k, int32_t* __restrict__ accepted,
                                                          int32_t* __restrict__ out_tokens) {
    const int b = blockIdx.x * 64 + threadIdx.x;
    if (b >= batch) return;
    const int32_t* d = draft + (size_t)b * k;
    const int32_t* t = target + (size_t)b * (k + 1);
    int32_t* o = out_tokens + (size_t)b * (k + 1);
    int n = 0;
    while (n < k && d[n] == t[n]) {
        o[n] = d[n];
        ++n;
    }
    o[n] = t[n];
    for (int j = n + 1; j <= k; ++j) o[j] = -1;
    accepted[b] = n;
}

hipError_t launch_greedy_verify(const int32_t* draft, const int32_t* target, int batch, int k, int32_t* accepted,
                                int32_t* out_tokens, hipStream_t s) {
    if (batch == 0) return hipSuccess;
    hipLaunchKernelGGL(greedy_verify_kernel, dim3((unsigned)((batch + 63) / 64)), dim3(64), 0, s, draft, target, batch, k,
                       accepted, out_tokens);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void calibration_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(blocks), dim3(256), 0, s, static_cast<u32x4*>(dst),
                       static_cast<const u32x4*>(src), n16);
    return hipGetLastError();
}

// Pure read stream: every lane reads 16 bytes per step, eight steps in flight, and folds them into a checksum; one
// word per workgroup leaves the chip.  Its rate is what a kernel that only reads can reach on this part.
constexpr int kReadBlocks = 256 * 8;

__global__ __launch_bounds__(256) void calibration_read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
    __shared__ uint32_t part[4];
    const size_t stride = (size_t)gridDim.x * 256;
    u32x4 acc = {0u, 0u, 0u, 0u};
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    for (; i < n16; i += stride) acc ^= src[i];
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x ^= (uint32_t)__shfl_xor((int)x, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

hipError_t launch_calibration_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s) {
    hipLaunchKernelGGL(calibration_read_kernel, dim3(kReadBlocks), dim3(256), 0, s, static_cast<const u32x4*>(src), bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace sd2
