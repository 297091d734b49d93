// libsd2 -- the drafter's LM head with the greedy choice fused in (gfx950).
//
// Eq. 1 (Sec. 2.1) draws each draft token from the drafter's distribution; greedy drafting takes
// the largest logit.  The head is the one linear that is never pruned (Sec. 2.3, Sec. 3.2), so it
// is a plain dense [vocab][hidden] bf16 matrix streamed once per call: pure HBM traffic.
//
// One workgroup of 8 wavefronts per compute unit walks over 16-row strips of the matrix.  Inside a
// workgroup the contraction is split eight ways: wavefront w owns the 128-column chunks w, w+8, ...
// of every strip, and keeps the matching slice of the normalised activations (operand B of the
// MFMAs) in registers for the whole kernel.  Weights travel HBM -> LDS directly
// (global_load_lds_dwordx4, 256 contiguous bytes per row piece) into a per-wave ring of four 4 KiB
// chunk buffers, refilled as soon as its reads have returned, so up to four chunks are in flight; the 16-byte
// pieces of a row are stored xor-swizzled by the row number so that the MFMA-layout reads
// (one row per lane) hit sixteen different bank groups.  Per strip the eight partial 16 x 16
// results meet in LDS (double buffered, one barrier), four wavefronts add them in a fixed order and
// keep a running (largest logit, lowest row) per thread; nothing but 16 candidates per workgroup
// ever goes back to HBM unless the caller asks for the logits.
#include <algorithm>
#include <atomic>

#include "sd2_device.h"
#include "sd2_internal.h"

namespace sd2 {

constexpr int kLmWaves = 8;                     // wavefronts per workgroup = ways the contraction is split
constexpr int kLmChunkCols = 128;               // columns of one staged chunk (16 rows x 128 x bf16 = 4 KiB)
constexpr int kLmRing = 4;                      // chunk buffers per wavefront
constexpr int kLmChunkDw = 16 * kLmChunkCols / 2;
constexpr int kLmRedDw = kLmWaves * 256;        // one set of partial strips
constexpr int kLmMiscDw = kLmWaves * 16 + 512;  // sums of squares per wave and token; final candidates
constexpr int kLmLdsDw = kLmWaves * kLmRing * kLmChunkDw + 2 * kLmRedDw + kLmMiscDw;

struct LmCand {
    float v;
    int32_t i;
};

// (a, ia) <- the better of the two: larger value, on equal values the lower index
__device__ __forceinline__ void lm_better(float& a, int32_t& ia, float b, int32_t ib) {
    if (b > a || (b == a && ib < ia)) {
        a = b;
        ia = ib;
    }
}

// HEAD = true: the LM head (fp32 residual in `h`, final norm, greedy choice, logits optional).
// HEAD = false: the same stream as a plain dense linear, y = x W^T with bf16 activations `x` and every result
// written to `logits` ([k_tok][vocab] with vocab = n_out): the dense baseline of the sparse linears.  There TG = 2
// takes up to 32 tokens in one pass (two sets of B operands in registers, two accumulators per strip; the partial
// strips then share one LDS buffer and need a second barrier per strip).
template <int CPW, bool HEAD, int TG = 1>
__global__ __launch_bounds__(64 * kLmWaves) void lm_head_kernel(const uint16_t* __restrict__ w,
                                                                const float* __restrict__ h,
                                                                const uint16_t* __restrict__ x_all, int vocab, int hidden,
                                                                int k_tok_all, int n_strips, LmCand* __restrict__ part,
                                                                float* __restrict__ logits_all) {
    extern __shared__ __attribute__((aligned(16))) uint32_t lm_smem[];
    // As a plain linear with more tokens than one pass takes, the grid's second dimension numbers the passes of 16 TG
    // tokens (the matrix is streamed once per pass); the head itself is launched with one pass.
    const int pass = HEAD ? 0 : (int)blockIdx.y;
    const uint16_t* __restrict__ x = HEAD ? x_all : x_all + (size_t)pass * (16 * TG) * hidden;
    float* __restrict__ logits = (HEAD || !logits_all) ? logits_all : logits_all + (size_t)pass * (16 * TG) * vocab;
    const int k_tok = HEAD ? k_tok_all : min(16 * TG, k_tok_all - pass * (16 * TG));
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    uint32_t* ring = lm_smem + wave * (kLmRing * kLmChunkDw);
    float* red = reinterpret_cast<float*>(lm_smem + kLmWaves * kLmRing * kLmChunkDw);
    float* misc = red + 2 * kLmRedDw;

    const int n_colchunks = hidden / kLmChunkCols;
    const int my_strips = (n_strips - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int n_chunks = my_strips * CPW;

    static_assert(kLmRing == 4, "the waits below count four loads per chunk and three chunks behind the current one");
    // Chunk ci of this wavefront: strip blockIdx.x + (ci / CPW) * gridDim.x, column chunk wave + 8 * (ci % CPW).
    // Instruction i of a chunk fills LDS rows 4i..4i+3 (16 lanes per row); lane l brings the 16-byte piece
    // (l & 15) ^ row of its row, so piece j of row r sits at LDS piece position j ^ r.
    auto issue_chunk = [&](int ci) {
        if (ci >= n_chunks) return;
        uint32_t* dst = ring + (ci & (kLmRing - 1)) * kLmChunkDw;
        const int strip = (int)blockIdx.x + (ci / CPW) * (int)gridDim.x;
        const int colchunk = min(wave + kLmWaves * (ci % CPW), n_colchunks - 1);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = 4 * i + g;
            // rows past the end of a ragged last strip read the row 16 above instead (results unused): valid, and
            // distinct from every other address this wavefront has in flight
            int row = strip * 16 + r;
            if (row >= vocab) row = max(row - 16, 0);
            const uint16_t* src = w + (size_t)row * hidden + colchunk * kLmChunkCols + ((n ^ r) * 8);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(dst + i * 256), 16, 0, 0);
        }
    };
    // Chunk ci has landed once at most the loads of the chunks issued after it are outstanding (loads return in
    // order): up to three chunks of four loads each, fewer at the end of the wavefront's work.
    auto wait_chunk = [&](int ci) {
        const int later = min(n_chunks - 1 - ci, kLmRing - 1);
        if (later >= 3)
            __builtin_amdgcn_s_waitcnt(0x0F70 | 12);
        else if (later == 2)
            __builtin_amdgcn_s_waitcnt(0x0F70 | 8);
        else if (later == 1)
            __builtin_amdgcn_s_waitcnt(0x0F70 | 4);
        else
            __builtin_amdgcn_s_waitcnt(0x0F70);
        asm volatile("" ::: "memory");
    };
#pragma unroll
    for (int c = 0; c < kLmRing; ++c) issue_chunk(c);

    static_assert(TG == 1 || !HEAD, "the head takes one token group per pass");
    const int tok = min(n, k_tok - 1);  // lanes past the last token repeat it; their results are never used
    Frag b[TG][CPW][4];
    if (HEAD) {
        // ---- final norm of the residual stream, straight into operand B: a = bf16(h / sqrt(mean(h^2) + eps))
        for (int t = 0; t < k_tok; ++t) {
            float s = 0.f;
            for (int c = tid * 4; c < hidden; c += 64 * kLmWaves * 4) {
                const f32x4 v = *reinterpret_cast<const f32x4*>(h + (size_t)t * hidden + c);
                s += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
            if (lane == 0) misc[wave * 16 + t] = s;
        }
        __syncthreads();
        float tot = 0.f;
#pragma unroll
        for (int ww = 0; ww < kLmWaves; ++ww) tot += misc[ww * 16 + tok];
        const float inv = 1.0f / sqrtf(tot / (float)hidden + 1e-5f);
#pragma unroll
        for (int cc = 0; cc < CPW; ++cc) {
            const int colchunk = wave + kLmWaves * cc;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (colchunk < n_colchunks) {
                    const float* src = h + (size_t)tok * hidden + colchunk * kLmChunkCols + (q * 4 + g) * 8;
                    const f32x4 lo = *reinterpret_cast<const f32x4*>(src);
                    const f32x4 hi = *reinterpret_cast<const f32x4*>(src + 4);
                    b[0][cc][q].u[0] = pack_bf16(lo[0] * inv, lo[1] * inv);
                    b[0][cc][q].u[1] = pack_bf16(lo[2] * inv, lo[3] * inv);
                    b[0][cc][q].u[2] = pack_bf16(hi[0] * inv, hi[1] * inv);
                    b[0][cc][q].u[3] = pack_bf16(hi[2] * inv, hi[3] * inv);
                } else {
                    b[0][cc][q].q = u32x4{0u, 0u, 0u, 0u};  // column chunk past the matrix: contributes nothing
                }
            }
        }
    } else {
#pragma unroll
        for (int tg = 0; tg < TG; ++tg) {
            const int tk = min(n + 16 * tg, k_tok - 1);
#pragma unroll
            for (int cc = 0; cc < CPW; ++cc) {
                const int colchunk = wave + kLmWaves * cc;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    b[tg][cc][q].q = colchunk < n_colchunks
                                         ? *reinterpret_cast<const u32x4*>(x + (size_t)tk * hidden + colchunk * kLmChunkCols + (q * 4 + g) * 8)
                                         : u32x4{0u, 0u, 0u, 0u};
            }
        }
    }

    // ---- strips
    // Reducing thread (wave rho < 4, lane l) owns result element l of source lane group rho: token l >> 2,
    // row 4 rho + (l & 3) of each strip, so its running best needs no cross-lane work until the very end.
    float best = -INFINITY;
    int32_t best_i = 0x7fffffff;
    const int red_tok = lane >> 2, red_row = 4 * wave + (lane & 3);
    int ci = 0;
#pragma unroll 1
    for (int si = 0; si < my_strips; ++si) {
        f32x4 acc[TG];
#pragma unroll
        for (int tg = 0; tg < TG; ++tg) acc[tg] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cc = 0; cc < CPW; ++cc) {
            wait_chunk(ci);
            const uint32_t* buf = ring + (ci & (kLmRing - 1)) * kLmChunkDw;
            Frag a[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) a[q].q = *reinterpret_cast<const u32x4*>(buf + (n * 16 + ((q * 4 + g) ^ n)) * 4);
            // the buffer is refilled only after its reads have returned
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
            asm volatile("" ::: "memory");
            issue_chunk(ci + kLmRing);
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int tg = 0; tg < TG; ++tg) acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[q].v, b[tg][cc][q].v, acc[tg], 0, 0, 0);
            ++ci;
        }
        // one token group: the partial strips alternate between two buffers (one barrier per strip); two groups fill
        // both buffers at once and a second barrier frees them
        float* mine = red + (TG == 1 ? (si & 1) * kLmRedDw : 0);
#pragma unroll
        for (int tg = 0; tg < TG; ++tg) *reinterpret_cast<f32x4*>(mine + tg * kLmRedDw + wave * 256 + lane * 4) = acc[tg];
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the partial strip is in LDS; loads stay in flight
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (wave < 4) {
#pragma unroll
            for (int tg = 0; tg < TG; ++tg) {
                float v = 0.f;
#pragma unroll
                for (int ww = 0; ww < kLmWaves; ++ww) v += mine[tg * kLmRedDw + ww * 256 + wave * 64 + lane];
                const int row = ((int)blockIdx.x + si * (int)gridDim.x) * 16 + red_row;
                const int rt = red_tok + 16 * tg;
                if (row < vocab && rt < k_tok) {
                    if (HEAD && v > best) {  // rows come in increasing order: '>' keeps the lowest index among equals
                        best = v;
                        best_i = row;
                    }
                    if (!HEAD || logits) logits[(size_t)rt * vocab + row] = v;
                }
            }
        }
        if (TG > 1) {
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
    }
    if (!HEAD) return;
    // ---- 16 threads per token hold candidates: pick one per token and workgroup
    LmCand* cand = reinterpret_cast<LmCand*>(misc + kLmWaves * 16);
    if (wave < 4) cand[wave * 64 + lane] = LmCand{best, best_i};
    __syncthreads();
    if (tid < 16) {
        float bv = -INFINITY;
        int32_t bi = 0x7fffffff;
        for (int rho = 0; rho < 4; ++rho)
            for (int j = 0; j < 4; ++j) {
                const LmCand c = cand[rho * 64 + tid * 4 + j];
                lm_better(bv, bi, c.v, c.i);
            }
        part[(size_t)blockIdx.x * 16 + tid] = LmCand{bv, bi};
    }
}

// One wavefront per token folds the candidates of all workgroups.
__global__ __launch_bounds__(1024) void lm_head_pick_kernel(const LmCand* __restrict__ part, int n_wg, int k_tok,
                                                            int32_t* __restrict__ token_ids,
                                                            float* __restrict__ max_logit) {
    const int lane = threadIdx.x & 63, t = threadIdx.x >> 6;
    if (t >= k_tok) return;
    float bv = -INFINITY;
    int32_t bi = 0x7fffffff;
    for (int j = lane; j < n_wg; j += 64) {
        const LmCand c = part[(size_t)j * 16 + t];
        lm_better(bv, bi, c.v, c.i);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o);
        const int32_t oi = __shfl_xor(bi, o);
        lm_better(bv, bi, ov, oi);
    }
    if (lane == 0) {
        token_ids[t] = bi == 0x7fffffff ? 0 : bi;  // every logit NaN: no candidate ever won
        if (max_logit) max_logit[t] = bv;
    }
}

static int lm_cu_count() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
        return n;
    return 256;
}

template <int CPW, bool HEAD, int TG = 1>
static hipError_t launch_lm_t(const uint16_t* w, const float* h, const uint16_t* x, int vocab, int hidden, int k_tok,
                              int n_strips, int n_wg, LmCand* part, float* logits, hipStream_t s, int passes = 1) {
    static std::atomic<bool> attr_set{false};  // more than the default 64 KiB of dynamic LDS needs opting in, once per kernel
    const size_t lds = (size_t)kLmLdsDw * 4;
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&lm_head_kernel<CPW, HEAD, TG>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((lm_head_kernel<CPW, HEAD, TG>), dim3((unsigned)n_wg, (unsigned)passes), dim3(64 * kLmWaves), lds, s, w, h, x, vocab, hidden,
                       k_tok, n_strips, part, logits);
    return hipGetLastError();
}

template <bool HEAD>
static hipError_t launch_lm_cpw(const uint16_t* w, const float* h, const uint16_t* x, int vocab, int hidden, int k_tok,
                                int n_strips, int n_wg, LmCand* part, float* logits, hipStream_t s, int passes = 1) {
    const int cpw = (hidden / kLmChunkCols + kLmWaves - 1) / kLmWaves;
    switch (cpw) {
        case 1: return launch_lm_t<1, HEAD>(w, h, x, vocab, hidden, k_tok, n_strips, n_wg, part, logits, s, passes);
        case 2: return launch_lm_t<2, HEAD>(w, h, x, vocab, hidden, k_tok, n_strips, n_wg, part, logits, s, passes);
        case 3: return launch_lm_t<3, HEAD>(w, h, x, vocab, hidden, k_tok, n_strips, n_wg, part, logits, s, passes);
        case 4: return launch_lm_t<4, HEAD>(w, h, x, vocab, hidden, k_tok, n_strips, n_wg, part, logits, s, passes);
        case 5: case 6: return launch_lm_t<6, HEAD>(w, h, x, vocab, hidden, k_tok, n_strips, n_wg, part, logits, s, passes);
        case 7: case 8: return launch_lm_t<8, HEAD>(w, h, x, vocab, hidden, k_tok, n_strips, n_wg, part, logits, s, passes);
        case 9: return launch_lm_t<9, HEAD>(w, h, x, vocab, hidden, k_tok, n_strips, n_wg, part, logits, s, passes);
        default: return hipErrorInvalidValue;
    }
}

// tokens [0, k_tok) with k_tok <= 16; `part` holds kLmMaxWorkgroups * 16 candidates
hipError_t launch_lm_head(const uint16_t* w, const float* h, int vocab, int hidden, int k_tok, void* part_ws,
                          int32_t* token_ids, float* max_logit, float* logits, hipStream_t s) {
    const int n_strips = (vocab + 15) / 16;
    const int n_wg = std::min(std::min(n_strips, lm_cu_count()), kLmMaxWorkgroups);
    LmCand* part = static_cast<LmCand*>(part_ws);
    const hipError_t e = launch_lm_cpw<true>(w, h, nullptr, vocab, hidden, k_tok, n_strips, n_wg, part, logits, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(lm_head_pick_kernel, dim3(1), dim3(1024), 0, s, part, n_wg, k_tok, token_ids, max_logit);
    return hipGetLastError();
}

// y[t][n] = sum_c W[n][c] x[t][c] for a dense row-major bf16 matrix and tokens [0, k_tok); every entry of y written
// (final values: the contraction is added up inside the workgroup).  k_in a multiple of 128, <= 9216.  A pass takes 16
// tokens, or 32 where dense_stream_pair_ok(k_in) (two token groups' activations then fit the registers next to each
// other); more tokens are further passes of the same launch (the grid's second dimension).
hipError_t launch_dense_stream_linear(const uint16_t* w, const uint16_t* x, int n_out, int k_in, int k_tok, float* y,
                                      hipStream_t s) {
    const int n_strips = (n_out + 15) / 16;
    const int n_wg = std::min(n_strips, lm_cu_count());
    if (k_tok < 1 || k_tok > 64) return hipErrorInvalidValue;
    if (k_tok > 16 && dense_stream_pair_ok(k_in)) {
        const int passes = (k_tok + 31) / 32;
        switch ((k_in / kLmChunkCols + kLmWaves - 1) / kLmWaves) {
            case 1: return launch_lm_t<1, false, 2>(w, nullptr, x, n_out, k_in, k_tok, n_strips, n_wg, nullptr, y, s, passes);
            case 2: return launch_lm_t<2, false, 2>(w, nullptr, x, n_out, k_in, k_tok, n_strips, n_wg, nullptr, y, s, passes);
            case 3: return launch_lm_t<3, false, 2>(w, nullptr, x, n_out, k_in, k_tok, n_strips, n_wg, nullptr, y, s, passes);
            case 4: return launch_lm_t<4, false, 2>(w, nullptr, x, n_out, k_in, k_tok, n_strips, n_wg, nullptr, y, s, passes);
            default: return hipErrorInvalidValue;
        }
    }
    return launch_lm_cpw<false>(w, nullptr, x, n_out, k_in, k_tok, n_strips, n_wg, nullptr, y, s, (k_tok + 15) / 16);
}

}  // namespace sd2
