// Whole-forward persistent kernel for the sparse drafter stack on gfx950.
//
// One workgroup of 16 wavefronts per CU lives for the entire forward.  Every wavefront walks its
// own static list of 16x256 weight tiles through all 4 x layers linears; the compacted stream of
// its next tile is always in flight (also across the end of a linear, because weights never
// depend on activations), so HBM keeps streaming while the grid synchronises.  Between dependent
// linears the grid meets at a barrier built from agent-scope atomics only; all activations that
// cross CUs move with agent-scope atomic loads / stores / float adds, which bypass the per-XCD L2,
// so the barrier needs no cache write-back or invalidate.  After each barrier a workgroup rebuilds,
// in LDS, exactly the bf16 activation columns its own tiles need: RMS-normed residual, causal
// attention over the in-flight tokens, or the SiLU-gated product.  Tile results are accumulated
// with float atomic adds (split-K over the 256-column slabs); the wavefront that delivers the last
// slab of a 16-row strip of the residual stream adds that strip's squares to the next norm's sum.
#include "sd2_device.h"
#include "sd2_internal.h"

namespace sd2 {

constexpr int kMegaWaves = 16;
constexpr int kMegaThreads = 64 * kMegaWaves;
constexpr int kMegaCh = 5;                                   // 1 KiB pieces of a staged tile
constexpr int kTileDw = kMegaCh * 256;                       // dwords per wavefront tile buffer
constexpr int kXldsDw = 2 * kMegaMaxTok * 256 / 2;           // bf16 [2 slabs][8 tokens][256]
constexpr int kAttHeads = 4;                                 // query / kv heads one CU may need
constexpr int kScrFloats = 3 * kMegaMaxTok * kAttHeads * 128 + kAttHeads * 64;
constexpr size_t kMegaLds = (size_t)(kMegaWaves * kTileDw + kXldsDw + kScrFloats) * 4;
constexpr int kBarWords = 32 + 8 * 32 + 8 * 32;              // top counter, 8 group counters, 8 group flags

#define SD2_AGENT __HIP_MEMORY_SCOPE_AGENT

__device__ __forceinline__ float aload(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, SD2_AGENT); }
__device__ __forceinline__ void astore(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, SD2_AGENT); }
__device__ __forceinline__ void aadd(float* p, float v) { (void)__hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, SD2_AGENT); }

struct TileRef {
    int p;  // phase = 4 * layer + kind; == n_phases when there is no tile
    int t;  // tile index inside that matrix
};

__device__ __forceinline__ void cu_range(const MegaGeo& g, int cu, int ncu, int& lo, int& hi) {
    lo = (int)((long long)g.n_tiles * cu / ncu);
    hi = (int)((long long)g.n_tiles * (cu + 1) / ncu);
}

__device__ __forceinline__ TileRef first_tile_from(const MegaArgs& a, int p, int n_phases, int cu, int ncu, int wave) {
    for (; p < n_phases; ++p) {
        int lo, hi;
        cu_range(a.geo[p & 3], cu, ncu, lo, hi);
        if (lo + wave < hi) return TileRef{p, lo + wave};
    }
    return TileRef{n_phases, 0};
}

__device__ __forceinline__ TileRef next_tile(const MegaArgs& a, TileRef r, int n_phases, int cu, int ncu, int wave) {
    if (r.p >= n_phases) return r;
    int lo, hi;
    cu_range(a.geo[r.p & 3], cu, ncu, lo, hi);
    if (r.t + kMegaWaves < hi) return TileRef{r.p, r.t + kMegaWaves};
    return first_tile_from(a, r.p + 1, n_phases, cu, ncu, wave);
}

// The 12 dwords of a directory entry, one per lane (lanes 0..11); converted to scalars a tile later.
__device__ __forceinline__ uint32_t load_dir_raw(const MegaArgs& a, TileRef r, int n_phases, int lane) {
    if (r.p >= n_phases) return 0u;
    const uint32_t* d = reinterpret_cast<const uint32_t*>(a.blob[r.p] + 128) + (size_t)r.t * 12;
    return d[lane < 12 ? lane : 11];
}

__device__ __forceinline__ DirEnt dir_from_raw(uint32_t raw) {
    DirEnt e;
    e.val_start = (uint32_t)__builtin_amdgcn_readlane((int)raw, 0);
    e.nnz = (uint32_t)__builtin_amdgcn_readlane((int)raw, 1);
#pragma unroll
    for (int i = 0; i < 8; ++i) e.base[i] = (uint32_t)__builtin_amdgcn_readlane((int)raw, 2 + i);
    e.zero[0] = e.zero[1] = 0;
    return e;
}

// Grid barrier: 8 groups of workgroups (by id mod 8) count arrivals, the last of each group
// arrives at the top counter, the very last releases the 8 group flags.  Counters only grow;
// `gen` is the number of barriers passed.  Waits are bounded: on overrun *err is set and the
// kernel keeps going (results are then invalid, but every wave still terminates).
__device__ __forceinline__ void grid_barrier(unsigned* bar, unsigned* err, unsigned ncu, unsigned& gen, int spin_limit) {
    __builtin_amdgcn_s_waitcnt(0);  // this wave's stores and atomics have been acknowledged
    __syncthreads();
    gen += 1;
    if (threadIdx.x == 0) {
        unsigned* top = bar;
        unsigned* gcount = bar + 32;
        unsigned* gflag = bar + 32 + 8 * 32;
        const unsigned grp = blockIdx.x & 7u;
        const unsigned ngrp = ncu < 8u ? ncu : 8u;
        const unsigned gsize = (ncu - grp + 7u) / 8u;
        bool wait = true;
        const unsigned prev = __hip_atomic_fetch_add(&gcount[grp * 32], 1u, __ATOMIC_RELAXED, SD2_AGENT);
        if (prev + 1 == gen * gsize) {
            const unsigned p2 = __hip_atomic_fetch_add(top, 1u, __ATOMIC_RELAXED, SD2_AGENT);
            if (p2 + 1 == gen * ngrp) {
                wait = false;
                for (unsigned g = 0; g < ngrp; ++g) __hip_atomic_store(&gflag[g * 32], gen, __ATOMIC_RELAXED, SD2_AGENT);
            }
        }
        if (wait) {
            int spins = 0;
            while (__hip_atomic_load(&gflag[grp * 32], __ATOMIC_RELAXED, SD2_AGENT) < gen) {
                __builtin_amdgcn_s_sleep(2);
                if (++spins > spin_limit) {
                    __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, SD2_AGENT);
                    break;
                }
            }
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(kMegaThreads) void mega_forward_kernel(const MegaArgs a) {
    extern __shared__ uint32_t mega_lds[];
    __shared__ uint2 lut[16];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cu = blockIdx.x, ncu = gridDim.x;
    const int n = lane & 15, g = lane >> 4;
    const int n_phases = 4 * a.layers;
    const int k_tok = a.k_tok;

    uint32_t* buf = mega_lds + wave * kTileDw;
    uint16_t* xlds = reinterpret_cast<uint16_t*>(mega_lds + kMegaWaves * kTileDw);
    float* scr = reinterpret_cast<float*>(mega_lds + kMegaWaves * kTileDw + kXldsDw);
    if (tid < 16) lut[tid] = make_expand_selector((uint32_t)tid);

    // this wave's first three tiles; the first one's stream is requested right away
    TileRef cur = first_tile_from(a, 0, n_phases, cu, ncu, wave);
    TileRef nxt = next_tile(a, cur, n_phases, cu, ncu, wave);
    TileRef nn = next_tile(a, nxt, n_phases, cu, ncu, wave);
    DirEnt de_cur = dir_from_raw(load_dir_raw(a, cur, n_phases, lane));
    DirEnt de_nxt = dir_from_raw(load_dir_raw(a, nxt, n_phases, lane));
    uint32_t de_raw = load_dir_raw(a, nn, n_phases, lane);
    u32x4 st[kMegaCh];
    uint2 mk_next = make_uint2(0, 0);
#pragma unroll
    for (int c = 0; c < kMegaCh; ++c) st[c] = u32x4{0, 0, 0, 0};
    if (cur.p < n_phases) {
        const MegaGeo& ge = a.geo[cur.p & 3];
        issue_tile<kMegaCh>(st, mk_next, reinterpret_cast<const uint16_t*>(a.blob[cur.p] + ge.val_off),
                            reinterpret_cast<const uint2*>(a.blob[cur.p] + ge.mask_off), de_cur.val_start, de_cur.nnz,
                            cur.t, lane);
    }
    unsigned gen = 0;

    for (int p = 0; p < n_phases; ++p) {
        const int layer = p >> 2, kind = p & 3;
        const MegaGeo& ge = a.geo[kind];
        if (p > 0) grid_barrier(a.bar, a.err, (unsigned)ncu, gen, a.spin_limit);

        // ---------------- prologue: the activation columns this CU's tiles need, as bf16 in LDS
        int lo, hi;
        cu_range(ge, cu, ncu, lo, hi);
        const int s_lo = lo / ge.n_strips;
        const int s_hi = hi > lo ? (hi - 1) / ge.n_strips : s_lo;
        const int n_sl = hi > lo ? s_hi - s_lo + 1 : 0;  // 0, 1 or 2
        const int nqkv = a.q_out + 2 * a.kv_out;
        float* yq = a.yqkv + (size_t)(layer & 1) * k_tok * nqkv;
        float* yg = a.ygu + (size_t)(layer & 1) * k_tok * 2 * a.inter;
        if (kind == 0 || kind == 2) {
            const float* ss = a.sumsq + (size_t)(2 * layer + (kind == 2 ? 1 : 0)) * 16;
            for (int idx = tid; idx < n_sl * kMegaMaxTok * 256; idx += kMegaThreads) {
                const int c = idx & 255, t = (idx >> 8) & (kMegaMaxTok - 1), sl = idx >> 11;
                const int col = (s_lo + sl) * 256 + c;
                uint16_t v = 0;
                if (t < k_tok && col < ge.k_in) {
                    const float inv = 1.0f / sqrtf(aload(ss + t) / (float)a.hidden + 1e-5f);
                    const float hv = aload(a.h + (size_t)t * a.hidden + col);
                    v = f32_to_bf16(hv * inv);
                    if (a.trace_x) {
                        a.trace_x[((size_t)p * k_tok + t) * a.trace_kmax + col] = v;
                        a.trace_src[((size_t)p * k_tok + t) * a.trace_smax + col] = hv;
                    }
                }
                xlds[idx] = v;
            }
            // recycle an accumulator that is idle now: it will be added into two layers from here
            float* z = kind == 2 ? yq : a.ygu + (size_t)((layer + 1) & 1) * k_tok * 2 * a.inter;
            const int zn = kind == 2 ? k_tok * nqkv : k_tok * 2 * a.inter;
            if (kind == 2 || layer > 0) {
                const int z0 = (int)((long long)zn * cu / ncu), z1 = (int)((long long)zn * (cu + 1) / ncu);
                for (int i = z0 + tid; i < z1; i += kMegaThreads) astore(z + i, 0.f);
            }
        } else if (kind == 3) {
            for (int idx = tid; idx < n_sl * kMegaMaxTok * 256; idx += kMegaThreads) {
                const int c = idx & 255, t = (idx >> 8) & (kMegaMaxTok - 1), sl = idx >> 11;
                const int col = (s_lo + sl) * 256 + c;
                uint16_t v = 0;
                if (t < k_tok && col < ge.k_in) {
                    const float gv = aload(yg + (size_t)t * 2 * a.inter + col);
                    const float uv = aload(yg + (size_t)t * 2 * a.inter + a.inter + col);
                    v = f32_to_bf16(gv / (1.0f + expf(-gv)) * uv);
                    if (a.trace_x) {
                        a.trace_x[((size_t)p * k_tok + t) * a.trace_kmax + col] = v;
                        float* ts = a.trace_src + ((size_t)p * k_tok + t) * a.trace_smax;
                        ts[col] = gv;
                        ts[a.inter + col] = uv;
                    }
                }
                xlds[idx] = v;
            }
        } else {  // kind == 1: causal attention among the in-flight tokens for the heads of these slabs
            const int D = a.head_dim;  // 128
            for (int idx = tid; idx < n_sl * kMegaMaxTok * 256; idx += kMegaThreads) xlds[idx] = 0;
            if (n_sl > 0) {
                const int col_lo = s_lo * 256, col_hi = min((s_hi + 1) * 256, ge.k_in);
                const int h_lo = col_lo / D, h_hi = (col_hi - 1) / D, nh = h_hi - h_lo + 1;
                const int rep = a.n_heads / a.n_kv;
                const int g_lo = h_lo / rep, ng = h_hi / rep - g_lo + 1;
                float* sq = scr;
                float* sk = sq + kMegaMaxTok * kAttHeads * 128;
                float* sv = sk + kMegaMaxTok * kAttHeads * 128;
                float* sp = sv + kMegaMaxTok * kAttHeads * 128;  // [head][i][j], 8 x 8 per head
                for (int idx = tid; idx < k_tok * nh * D; idx += kMegaThreads) {
                    const int d = idx % D, hh = (idx / D) % nh, t = idx / (D * nh);
                    const float qv = aload(yq + (size_t)t * nqkv + (h_lo + hh) * D + d);
                    sq[(t * kAttHeads + hh) * 128 + d] = qv;
                    if (a.trace_x) a.trace_src[((size_t)p * k_tok + t) * a.trace_smax + (h_lo + hh) * D + d] = qv;
                }
                for (int idx = tid; idx < k_tok * ng * D; idx += kMegaThreads) {
                    const int d = idx % D, gg = (idx / D) % ng, t = idx / (D * ng);
                    const float* row = yq + (size_t)t * nqkv + a.q_out + (g_lo + gg) * D + d;
                    const float kv = aload(row), vv = aload(row + a.kv_out);
                    sk[(t * kAttHeads + gg) * 128 + d] = kv;
                    sv[(t * kAttHeads + gg) * 128 + d] = vv;
                    if (a.trace_x) {
                        float* ts = a.trace_src + ((size_t)p * k_tok + t) * a.trace_smax + a.q_out + (g_lo + gg) * D + d;
                        ts[0] = kv;
                        ts[a.kv_out] = vv;
                    }
                }
                __syncthreads();
                const float scale = 1.0f / sqrtf((float)D);
                for (int idx = tid; idx < nh * k_tok * k_tok; idx += kMegaThreads) {
                    const int j = idx % k_tok, i = (idx / k_tok) % k_tok, hh = idx / (k_tok * k_tok);
                    if (j <= i) {
                        const int gg = (h_lo + hh) / rep - g_lo;
                        const float* qa = sq + (i * kAttHeads + hh) * 128;
                        const float* kb = sk + (j * kAttHeads + gg) * 128;
                        float dot = 0.f;
                        for (int d = 0; d < D; ++d) dot += qa[d] * kb[d];
                        sp[(hh * 8 + i) * 8 + j] = dot * scale;
                    }
                }
                __syncthreads();
                for (int idx = tid; idx < nh * k_tok; idx += kMegaThreads) {
                    const int i = idx % k_tok, hh = idx / k_tok;
                    float* row = sp + (hh * 8 + i) * 8;
                    float mx = row[0];
                    for (int j = 1; j <= i; ++j) mx = fmaxf(mx, row[j]);
                    float sum = 0.f;
                    for (int j = 0; j <= i; ++j) {
                        const float e = expf(row[j] - mx);
                        row[j] = e;
                        sum += e;
                    }
                    const float inv = 1.0f / sum;
                    for (int j = 0; j <= i; ++j) row[j] *= inv;
                }
                __syncthreads();
                for (int idx = tid; idx < k_tok * nh * D; idx += kMegaThreads) {
                    const int d = idx % D, hh = (idx / D) % nh, t = idx / (D * nh);
                    const int col = (h_lo + hh) * D + d;
                    if (col >= col_lo && col < col_hi) {
                        const int gg = (h_lo + hh) / rep - g_lo;
                        const float* row = sp + (hh * 8 + t) * 8;
                        float o = 0.f;
                        for (int j = 0; j <= t; ++j) o += row[j] * sv[(j * kAttHeads + gg) * 128 + d];
                        const uint16_t cv = f32_to_bf16(o);
                        xlds[(((col >> 8) - s_lo) * kMegaMaxTok + t) * 256 + (col & 255)] = cv;
                        if (a.trace_x) a.trace_x[((size_t)p * k_tok + t) * a.trace_kmax + col] = cv;
                    }
                }
            }
        }
        __syncthreads();

        // ---------------- this wave's tiles of the phase
        int cur_slab = -1;
        Frag b[4][2];
#pragma unroll
        for (int q = 0; q < 4; ++q) b[q][0].q = b[q][1].q = u32x4{0, 0, 0, 0};
        while (cur.p == p) {
#pragma unroll
            for (int c = 0; c < kMegaCh; ++c) reinterpret_cast<u32x4*>(buf)[c * 64 + lane] = st[c];
            const uint2 mk = mk_next;
            const int strip = cur.t % ge.n_strips, slab = cur.t / ge.n_strips;
            if (slab != cur_slab) {
                cur_slab = slab;
                if (n < kMegaMaxTok) {
                    const u32x4* xr = reinterpret_cast<const u32x4*>(xlds + ((slab - s_lo) * kMegaMaxTok + n) * 256 + 16 * g);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        b[q][0].q = xr[8 * q];
                        b[q][1].q = xr[8 * q + 1];
                    }
                }
            }
            const DirEnt de = de_cur;
            de_cur = de_nxt;
            de_nxt = dir_from_raw(de_raw);
            if (nxt.p < n_phases) {
                const MegaGeo& gn = a.geo[nxt.p & 3];
                issue_tile<kMegaCh>(st, mk_next, reinterpret_cast<const uint16_t*>(a.blob[nxt.p] + gn.val_off),
                                    reinterpret_cast<const uint2*>(a.blob[nxt.p] + gn.mask_off), de_cur.val_start,
                                    de_cur.nnz, nxt.t, lane);
            }
            const TileRef n3 = next_tile(a, nn, n_phases, cu, ncu, wave);
            de_raw = load_dir_raw(a, n3, n_phases, lane);

            const uint8_t* bufb = reinterpret_cast<const uint8_t*>(buf);
            const uint32_t m16[4] = {mk.x & 0xffffu, mk.x >> 16, mk.y & 0xffffu, mk.y >> 16};
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t bits = m16[q];
                uint32_t nib[4];
#pragma unroll
                for (int h = 0; h < 4; ++h) nib[h] = (bits >> (4 * h)) & 15u;
                const uint32_t packed = (uint32_t)__builtin_popcount(nib[0]) | ((uint32_t)__builtin_popcount(nib[1]) << 8) |
                                        ((uint32_t)__builtin_popcount(nib[2]) << 16) |
                                        ((uint32_t)__builtin_popcount(nib[3]) << 24);
                const uint32_t ex = wave_excl_scan(packed);
                Frag f[2];
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    const uint32_t run_base = (de.base[(4 * q + h) >> 1] >> (16 * (h & 1))) & 0xffffu;
                    const uint32_t off = (run_base + ((ex >> (8 * h)) & 0xffu)) * 2u;
                    const Tri32 tr = *reinterpret_cast<const Tri32*>(bufb + (off & ~3u));
                    const uint32_t w0 = __builtin_amdgcn_alignbyte(tr.b, tr.a, off);
                    const uint32_t w1 = __builtin_amdgcn_alignbyte(tr.c, tr.b, off);
                    const uint2 sel = lut[nib[h]];
                    f[h >> 1].u[2 * (h & 1) + 0] = __builtin_amdgcn_perm(w1, w0, sel.x);
                    f[h >> 1].u[2 * (h & 1) + 1] = __builtin_amdgcn_perm(w1, w0, sel.y);
                }
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[0].v, b[q][0].v, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[1].v, b[q][1].v, acc, 0, 0, 0);
            }

            // ---- split-K accumulation: lane (n, g) owns rows 4g..4g+3 of token n
            const int row = strip * 16 + 4 * g;
            float* ybase = kind == 0 ? yq : (kind == 2 ? yg : a.h);
            float* dst = ybase + (size_t)n * ge.n_out + row;
            if (n < k_tok) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (row + v < ge.n_out) aadd(dst + v, acc[v]);
            }
            if (kind == 1 || kind == 3) {
                // last slab of this strip of h -> its squares go into the next norm's sum
                __builtin_amdgcn_s_waitcnt(0);
                unsigned old = 0;
                unsigned* cnt = a.strip_cnt + (size_t)(2 * layer + (kind == 3 ? 1 : 0)) * a.geo[1].n_strips + strip;
                if (lane == 0) old = __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, SD2_AGENT);
                old = (unsigned)__builtin_amdgcn_readfirstlane((int)old);
                if (old + 1 == (unsigned)ge.n_slabs) {
                    float s = 0.f;
                    if (n < k_tok) {
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (row + v < ge.n_out) {
                                const float hv = aload(dst + v);
                                s += hv * hv;
                            }
                    }
                    s += __shfl_xor(s, 16);
                    s += __shfl_xor(s, 32);
                    if (lane < 16 && n < k_tok) aadd(a.sumsq + (size_t)(2 * layer + (kind == 3 ? 2 : 1)) * 16 + n, s);
                }
            }
            cur = nxt;
            nxt = nn;
            nn = n3;
        }
    }
}

// ---------------------------------------------------------------- set-up kernels and launch

__global__ __launch_bounds__(256) void mega_zero_kernel(uint32_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

__global__ __launch_bounds__(256) void mega_h_init_kernel(float* __restrict__ h, const uint16_t* __restrict__ h_in, float* __restrict__ sumsq0,
                                                         int hidden) {
    __shared__ float red[256];
    const int t = blockIdx.x;
    float ss = 0.f;
    for (int i = threadIdx.x; i < hidden; i += 256) {
        const float v = bf16_to_f32(h_in[(size_t)t * hidden + i]);
        h[(size_t)t * hidden + i] = v;
        ss += v * v;
    }
    red[threadIdx.x] = ss;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) sumsq0[t] = red[0];
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

MegaLayout mega_layout(int layers, int hidden, int q_out, int kv_out, int inter, int k_tok) {
    MegaLayout L;
    size_t off = 0;
    L.bar_off = off;
    off += align256((size_t)kBarWords * 4);
    L.err_off = off;
    off += 256;
    L.sumsq_off = off;
    off += align256((size_t)(2 * layers + 1) * 16 * 4);
    L.cnt_off = off;
    off += align256((size_t)2 * layers * ((hidden + 15) / 16) * 4);
    L.yqkv_off = off;
    off += align256((size_t)2 * k_tok * (q_out + 2 * kv_out) * 4);
    L.ygu_off = off;
    off += align256((size_t)2 * k_tok * 2 * inter * 4);
    L.total = off;
    return L;
}

static int mega_grid() {
    static int cus = -1;
    if (cus < 0) {
        int dev = 0, n = 0, coop = 0;
        cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) == hipSuccess && coop &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0 &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(mega_forward_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMegaLds) == hipSuccess) {
            int per_cu = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, mega_forward_kernel, kMegaThreads, kMegaLds) == hipSuccess &&
                per_cu >= 1)
                cus = n;
        }
    }
    return cus;
}

bool mega_supported(const MegaGeo (&geo)[4], int layers, int head_dim, int k_tok, int max_tile_nnz) {
    if (layers < 1 || layers > kMegaMaxLayers || head_dim != 128 || k_tok < 1 || k_tok > kMegaMaxTok) return false;
    if (max_tile_nnz * 2 + 8 > kMegaCh * 1024) return false;
    const int ncu = mega_grid();
    if (ncu < 1) return false;
    for (int k = 0; k < 4; ++k) {
        // a CU's share of a matrix must stay within two 256-column slabs
        if ((geo[k].n_tiles + ncu - 1) / ncu > geo[k].n_strips) return false;
    }
    return true;
}

hipError_t launch_mega_forward(const MegaArgs& a, const uint16_t* h_in, void* zero_base, size_t zero_bytes, hipStream_t s) {
    const int ncu = mega_grid();
    if (ncu < 1) return hipErrorNotSupported;
    hipLaunchKernelGGL(mega_zero_kernel, dim3(256), dim3(256), 0, s, static_cast<uint32_t*>(zero_base), zero_bytes / 4);
    hipLaunchKernelGGL(mega_h_init_kernel, dim3((unsigned)a.k_tok), dim3(256), 0, s, a.h, h_in, a.sumsq, a.hidden);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    MegaArgs args = a;
    void* params[] = {&args};
    return hipLaunchCooperativeKernel(reinterpret_cast<const void*>(mega_forward_kernel), dim3((unsigned)ncu),
                                      dim3(kMegaThreads), params, kMegaLds, s);
}

}  // namespace sd2
