// Whole-forward persistent kernel for the sparse drafter stack on gfx950.
//
// One workgroup of 12 wavefronts per CU lives for the entire forward.  For every linear a
// workgroup owns a block of s strips x b slabs of 16x256 weight tiles; its wavefronts walk those
// tiles, and each wavefront keeps the compacted stream of its next tile in flight -- also across
// the end of a linear, because weights never depend on activations -- so HBM keeps streaming
// while the grid synchronises.  Tile results are summed per strip in LDS and leave the CU once
// per linear as float atomic adds (split-K only across the few slab blocks).  Between dependent
// linears the grid meets at a barrier built from agent-scope atomics.  Everything a CU hands to
// other CUs is written with agent-scope atomic stores / float adds, which go through to memory,
// so no cache write-back is needed before arriving; after the barrier one wavefront per workgroup
// invalidates the caches and the prologue reads with ordinary cached loads.  After each barrier a workgroup
// rebuilds in LDS exactly the bf16 activation columns its tiles need: the RMS-normed residual
// (every workgroup sums the squares of the whole residual itself), causal attention over the
// in-flight tokens for the heads of its slabs, or the SiLU-gated product.
#include "sd2_device.h"
#include "sd2_internal.h"

namespace sd2 {

constexpr int kMegaWaves = 12;
constexpr int kMegaThreads = 64 * kMegaWaves;
constexpr int kMegaCh = 5;                          // 1 KiB pieces of a staged tile
constexpr int kTileDw = kMegaCh * 256;              // dwords per wavefront tile buffer
constexpr int kMaxB = 8;                            // slabs per workgroup block (activation columns kept in LDS)
constexpr int kMaxBAtt = 3;                         // ... for the linear that follows attention
constexpr int kMaxS = 16;                           // strips per workgroup block (LDS accumulators)
constexpr int kXldsDw = kMaxB * kMegaMaxTok * 256 / 2;  // bf16 [slab][token][256]
constexpr int kRedDw = kMaxS * kMegaMaxTok * 16;        // fp32 [strip][token][row]
constexpr int kMiscDw = 512;                            // attention probabilities, per-token scalars
constexpr int kAttHeads = 6;                            // heads (and kv heads) one workgroup may need
constexpr int kScrDw = 3 * kMegaMaxTok * kAttHeads * 128;  // prologue scratch; the tile buffers live in the same area
constexpr int kAreaDw = kScrDw > kMegaWaves * kTileDw ? kScrDw : kMegaWaves * kTileDw;
constexpr size_t kMegaLds = (size_t)(kAreaDw + kXldsDw + kRedDw + kMiscDw) * 4;
constexpr int kBarWords = 32 + 8 * 32 + 8 * 32;     // top counter, 8 group counters, 8 group flags
static_assert(kMaxB * kMegaMaxTok * 256 <= kAreaDw, "column stash must fit the scratch area");
static_assert(kAttHeads * 128 == kMegaThreads, "one thread per (head slot, dimension)");
static_assert(4 * kMegaThreads >= kMegaMaxHidden && 3 * kMegaThreads >= kMaxB * 256, "prologue chunking");

#define SD2_AGENT __HIP_MEMORY_SCOPE_AGENT

// Activations written by other CUs: read with ordinary loads after the barrier's cache invalidate.
__device__ __forceinline__ float aload(const float* p) { return *p; }
__device__ __forceinline__ void astore(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, SD2_AGENT); }
__device__ __forceinline__ void aadd(float* p, float v) { (void)__hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, SD2_AGENT); }

// sum over the 64 lanes (cross-lane adds on the DPP path, no LDS traffic); result in every lane
__device__ __forceinline__ float wave_sum(float v) {
#define SD2_DPP_ADD(ctrl, rmask) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, rmask, 0xf, true))
    SD2_DPP_ADD(0x111, 0xf);  // row_shr:1
    SD2_DPP_ADD(0x112, 0xf);  // row_shr:2
    SD2_DPP_ADD(0x114, 0xf);  // row_shr:4
    SD2_DPP_ADD(0x118, 0xf);  // row_shr:8
    SD2_DPP_ADD(0x142, 0xa);  // row_bcast:15
    SD2_DPP_ADD(0x143, 0xc);  // row_bcast:31
#undef SD2_DPP_ADD
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// The argument block as it sits in the kernarg segment: indexing it with a run-time (wave-uniform) index
// gives scalar loads, where indexing the by-value parameter would make the compiler copy it to scratch.
typedef const __attribute__((address_space(4))) MegaArgs* KArgs;

struct TileRef {
    int p;   // phase = 4 * layer + kind; == n_phases when there is no tile
    int ss;  // strip inside the workgroup's block
    int sl;  // slab inside the workgroup's block
    int t;   // tile index inside the matrix
};

// Where this workgroup's block of each matrix kind starts (computed once).
struct KindPlan {
    int s_blk, b_blk, strip0, slab0, n_strips, n_slabs, active;
};

// The plan of one kind is rebuilt from the kernarg segment whenever it is needed (scalar loads and a
// scalar division): keeping the four plans in a local aggregate chosen at run time would put them in
// scratch memory and turn every tile index into a per-lane value.
__device__ __forceinline__ KindPlan pick_plan(KArgs ka, int kind, int cu) {
    KindPlan k;
    const int n_sblk = ka->geo[kind].n_sblk, n_bblk = ka->geo[kind].n_bblk;
    k.s_blk = ka->geo[kind].s_blk;
    k.b_blk = ka->geo[kind].b_blk;
    const int q = cu / n_sblk;
    k.strip0 = (cu - q * n_sblk) * k.s_blk;
    k.slab0 = q * k.b_blk;
    k.n_strips = ka->geo[kind].n_strips;
    k.n_slabs = ka->geo[kind].n_slabs;
    k.active = cu < n_sblk * n_bblk;
    return k;
}

// First tile of this wavefront at or after local position (ss, sl) of phase p; tiles of a block are numbered
// strip-first and dealt to the 16 wavefronts round-robin, so a wavefront advances by 16 strips at a time.
__device__ __forceinline__ TileRef find_tile(KArgs ka, int cu, int p, int ss, int sl, int n_phases, int wave) {
    for (; p < n_phases; ++p) {
        const KindPlan k = pick_plan(ka, p & 3, cu);
        if (k.active) {
            for (;;) {
                while (ss >= k.s_blk) {
                    ss -= k.s_blk;
                    ++sl;
                }
                if (sl >= k.b_blk) break;
                const int strip = k.strip0 + ss, slab = k.slab0 + sl;
                if (strip < k.n_strips && slab < k.n_slabs) return TileRef{p, ss, sl, slab * k.n_strips + strip};
                ss += kMegaWaves;
            }
        }
        ss = wave;
        sl = 0;
    }
    return TileRef{n_phases, 0, 0, 0};
}

__device__ __forceinline__ TileRef next_tile(KArgs ka, int cu, TileRef r, int n_phases, int wave) {
    if (r.p >= n_phases) return r;
    return find_tile(ka, cu, r.p, r.ss + kMegaWaves, r.sl, n_phases, wave);
}

// The 12 dwords of a directory entry, one per lane (lanes 0..11); converted to scalars a tile later.
__device__ __forceinline__ uint32_t load_dir_raw(KArgs ka, TileRef r, int n_phases, int lane) {
    if (r.p >= n_phases) return 0u;
    const uint32_t* d = reinterpret_cast<const uint32_t*>(ka->blob[r.p] + 128) + (size_t)r.t * 12;
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
    // One wavefront drops this CU's (and its XCD's) cached copies, so that the ordinary cached loads
    // of the prologue see what the other XCDs wrote through to memory with their atomics.
    if (threadIdx.x < 64) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    __syncthreads();
}

template <bool TRACE>
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
    KArgs ka = (KArgs)__builtin_amdgcn_kernarg_segment_ptr();

    uint32_t* buf = mega_lds + wave * kTileDw;                  // this wave's tile buffer
    float* scr = reinterpret_cast<float*>(mega_lds);            // prologue scratch (aliases all tile buffers)
    uint16_t* xlds = reinterpret_cast<uint16_t*>(mega_lds + kAreaDw);
    float* red = reinterpret_cast<float*>(mega_lds + kAreaDw + kXldsDw);
    float* misc = red + kRedDw;                                 // [0,384) probabilities, [384,400) per-token scalars
    if (tid < 16) lut[tid] = make_expand_selector((uint32_t)tid);
    for (int i = tid; i < kRedDw; i += kMegaThreads) red[i] = 0.f;

    // this wave's first three tiles; the first one's stream is requested right away
    TileRef cur = find_tile(ka, cu, 0, wave, 0, n_phases, wave);
    TileRef nxt = next_tile(ka, cu, cur, n_phases, wave);
    TileRef nn = next_tile(ka, cu, nxt, n_phases, wave);
    DirEnt de_cur = dir_from_raw(load_dir_raw(ka, cur, n_phases, lane));
    DirEnt de_nxt = dir_from_raw(load_dir_raw(ka, nxt, n_phases, lane));
    uint32_t de_raw = load_dir_raw(ka, nn, n_phases, lane);
    u32x4 st[kMegaCh];
    uint2 mk_next = make_uint2(0, 0);
#pragma unroll
    for (int c = 0; c < kMegaCh; ++c) st[c] = u32x4{0, 0, 0, 0};
    if (cur.p < n_phases) {
        const unsigned char* bl = ka->blob[cur.p];
        issue_tile<kMegaCh>(st, mk_next, reinterpret_cast<const uint16_t*>(bl + ka->geo[cur.p & 3].val_off),
                            reinterpret_cast<const uint2*>(bl + ka->geo[cur.p & 3].mask_off), de_cur.val_start, de_cur.nnz,
                            cur.t, lane);
    }
    unsigned gen = 0;

    for (int p = 0; p < n_phases; ++p) {
        const int layer = p >> 2, kind = p & 3;
        MegaGeo ge;  // this kind's geometry, fetched with scalar loads
        ge.n_out = ka->geo[kind].n_out;
        ge.k_in = ka->geo[kind].k_in;
        ge.n_strips = ka->geo[kind].n_strips;
        ge.n_slabs = ka->geo[kind].n_slabs;
        ge.s_blk = ka->geo[kind].s_blk;
        ge.b_blk = ka->geo[kind].b_blk;
        unsigned long long* tt = a.trace_time ? a.trace_time + ((size_t)cu * n_phases + p) * 4 : nullptr;
        if (tt && tid == 0) tt[0] = __builtin_amdgcn_s_memrealtime();
        if (p > 0) grid_barrier(a.bar, a.err, (unsigned)ncu, gen, a.spin_limit);
        if (tt && tid == 0) tt[1] = __builtin_amdgcn_s_memrealtime();

        // ---------------- prologue: the activation columns of this workgroup's slabs, as bf16 in LDS
        const KindPlan kpl = pick_plan(ka, kind, cu);
        const bool active = kpl.active;
        const int col_lo = kpl.slab0 * 256;                                       // first column of the block
        const int n_col = active ? max(0, min(ge.b_blk * 256, ge.k_in - col_lo)) : 0;  // columns that exist
        const int nqkv = a.q_out + 2 * a.kv_out;
        float* yq = a.yqkv + (size_t)(layer & 1) * k_tok * nqkv;
        float* yg = a.ygu + (size_t)(layer & 1) * k_tok * 2 * a.inter;
        const size_t tr_x = ((size_t)p * k_tok) * a.trace_kmax, tr_s = ((size_t)p * k_tok) * a.trace_smax;

        if (kind == 0 || kind == 2) {
            // (1) the whole residual: squares for the norm, and a stash of the columns this block needs;
            // four tokens x four column chunks of loads are in flight at a time
            if (tid < 16) misc[384 + tid] = 0.f;
            __syncthreads();
            for (int t0 = 0; t0 < k_tok; t0 += 4) {
                float hv[4][4];
#pragma unroll
                for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int col = tid + e * kMegaThreads;
                        hv[tt][e] = (t0 + tt < k_tok && col < a.hidden) ? aload(a.h + (size_t)(t0 + tt) * a.hidden + col) : 0.f;
                    }
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) {
                    const int t = t0 + tt;
                    if (t < k_tok) {
                        float ss = 0.f;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            ss += hv[tt][e] * hv[tt][e];
                            const int c = tid + e * kMegaThreads - col_lo;
                            if (c >= 0 && c < n_col) {
                                scr[t * (kMaxB * 256) + c] = hv[tt][e];
                                if (TRACE) a.trace_src[tr_s + (size_t)t * a.trace_smax + col_lo + c] = hv[tt][e];
                            }
                        }
                        ss = wave_sum(ss);
                        if (lane == 0) atomicAdd(&misc[384 + t], ss);
                    }
                }
            }
            __syncthreads();
            if (tid < k_tok) misc[400 + tid] = 1.0f / sqrtf(misc[384 + tid] / (float)a.hidden + 1e-5f);
            __syncthreads();
            // (2) normalise and round
            for (int idx = tid; idx < ge.b_blk * kMegaMaxTok * 256; idx += kMegaThreads) {
                const int c = idx & 255, t = (idx >> 8) & (kMegaMaxTok - 1), sl = idx >> 11;
                const int cc = sl * 256 + c;
                uint16_t v = 0;
                if (t < k_tok && cc < n_col) {
                    v = f32_to_bf16(scr[t * (kMaxB * 256) + cc] * misc[400 + t]);
                    if (TRACE) a.trace_x[tr_x + (size_t)t * a.trace_kmax + col_lo + cc] = v;
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
            // rows of unused token slots are zero; then four tokens x three column chunks per round of loads
            for (int idx = tid; idx < ge.b_blk * kMegaMaxTok * 256; idx += kMegaThreads)
                if (((idx >> 8) & (kMegaMaxTok - 1)) >= k_tok) xlds[idx] = 0;
            for (int t0 = 0; t0 < k_tok; t0 += 4) {
                float gv[4][3], uv[4][3];
#pragma unroll
                for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                    for (int e = 0; e < 3; ++e) {
                        const int cc = tid + e * kMegaThreads;
                        const bool ok = t0 + tt < k_tok && cc < n_col;
                        const float* row = yg + (size_t)(t0 + tt) * 2 * a.inter + col_lo + cc;
                        gv[tt][e] = ok ? aload(row) : 0.f;
                        uv[tt][e] = ok ? aload(row + a.inter) : 0.f;
                    }
#pragma unroll
                for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                    for (int e = 0; e < 3; ++e) {
                        const int t = t0 + tt, cc = tid + e * kMegaThreads;
                        if (t < k_tok && cc < ge.b_blk * 256) {
                            uint16_t v = 0;
                            if (cc < n_col) {
                                v = f32_to_bf16(gv[tt][e] / (1.0f + expf(-gv[tt][e])) * uv[tt][e]);
                                if (TRACE) {
                                    a.trace_x[tr_x + (size_t)t * a.trace_kmax + col_lo + cc] = v;
                                    a.trace_src[tr_s + (size_t)t * a.trace_smax + col_lo + cc] = gv[tt][e];
                                    a.trace_src[tr_s + (size_t)t * a.trace_smax + a.inter + col_lo + cc] = uv[tt][e];
                                }
                            }
                            xlds[((cc >> 8) * kMegaMaxTok + t) * 256 + (cc & 255)] = v;
                        }
                    }
            }
        } else {  // kind == 1: causal attention among the in-flight tokens for the heads of these slabs
            const int D = 128;
            for (int idx = tid; idx < ge.b_blk * kMegaMaxTok * 256; idx += kMegaThreads) xlds[idx] = 0;
            float* sq = scr;
            float* sk = sq + kMegaMaxTok * kAttHeads * 128;
            float* sv = sk + kMegaMaxTok * kAttHeads * 128;
            float* sp = misc;  // [head][i][j], 8 x 8 per head
            int h_lo = 0, nh = 0, g_lo = 0, ng = 0;
            const int rep = a.n_heads / a.n_kv;
            if (n_col > 0) {
                h_lo = col_lo / D;
                nh = (col_lo + n_col - 1) / D - h_lo + 1;
                g_lo = h_lo / rep;
                ng = (h_lo + nh - 1) / rep - g_lo + 1;
            }
            {
                // thread (head slot hh = tid / 128, dimension d): q of the block's heads, k and v of their kv heads,
                // four tokens per round of loads
                const int hh = tid >> 7, d = tid & 127;
                for (int t0 = 0; t0 < k_tok; t0 += 4) {
                    float qv[4], kv[4], vv[4];
#pragma unroll
                    for (int tt = 0; tt < 4; ++tt) {
                        const int t = t0 + tt;
                        const bool okq = t < k_tok && hh < nh, okk = t < k_tok && hh < ng;
                        const float* rq = yq + (size_t)t * nqkv + (h_lo + hh) * D + d;
                        const float* rk = yq + (size_t)t * nqkv + a.q_out + (g_lo + hh) * D + d;
                        qv[tt] = okq ? aload(rq) : 0.f;
                        kv[tt] = okk ? aload(rk) : 0.f;
                        vv[tt] = okk ? aload(rk + a.kv_out) : 0.f;
                    }
#pragma unroll
                    for (int tt = 0; tt < 4; ++tt) {
                        const int t = t0 + tt;
                        if (t < k_tok && hh < kAttHeads) {
                            const int el = (t * kAttHeads + hh) * 128 + d;
                            sq[el] = qv[tt];
                            sk[el] = kv[tt];
                            sv[el] = vv[tt];
                            if (TRACE) {
                                float* ts = a.trace_src + tr_s + (size_t)t * a.trace_smax;
                                if (hh < nh) ts[(h_lo + hh) * D + d] = qv[tt];
                                if (hh < ng) {
                                    ts[a.q_out + (g_lo + hh) * D + d] = kv[tt];
                                    ts[a.q_out + a.kv_out + (g_lo + hh) * D + d] = vv[tt];
                                }
                            }
                        }
                    }
                }
            }
            __syncthreads();
            // scores: one wavefront per (head, i, j <= i), two dimensions per lane
            const float scale = 1.0f / sqrtf((float)D);
            {
                int item = 0;
                for (int hh = 0; hh < nh; ++hh) {
                    const int gg = (h_lo + hh) / rep - g_lo;
                    for (int i = 0; i < k_tok; ++i)
                        for (int j = 0; j <= i; ++j, ++item) {
                            if (item % kMegaWaves != wave) continue;
                            const float* qa = sq + (i * kAttHeads + hh) * 128;
                            const float* kb = sk + (j * kAttHeads + gg) * 128;
                            const float dot = wave_sum(qa[lane] * kb[lane] + qa[lane + 64] * kb[lane + 64]);
                            if (lane == 0) sp[(hh * 8 + i) * 8 + j] = dot * scale;
                        }
                }
            }
            __syncthreads();
            if (tid < kAttHeads * 8) {
                const int i = tid & 7, hh = tid >> 3;
                if (hh < nh && i < k_tok) {
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
            }
            __syncthreads();
            {
                const int hh = tid >> 7, d = tid & 127;
                const int cc = (h_lo + hh) * D + d - col_lo;
                if (hh < nh && cc >= 0 && cc < n_col) {
                    const int gg = (h_lo + hh) / rep - g_lo;
                    for (int t = 0; t < k_tok; ++t) {
                        const float* row = sp + (hh * 8 + t) * 8;
                        float o = 0.f;
                        for (int j = 0; j <= t; ++j) o += row[j] * sv[(j * kAttHeads + gg) * 128 + d];
                        const uint16_t cv = f32_to_bf16(o);
                        xlds[((cc >> 8) * kMegaMaxTok + t) * 256 + (cc & 255)] = cv;
                        if (TRACE) a.trace_x[tr_x + (size_t)t * a.trace_kmax + col_lo + cc] = cv;
                    }
                }
            }
        }
        __syncthreads();
        if (tt && tid == 0) tt[2] = __builtin_amdgcn_s_memrealtime();

        // ---------------- this wave's tiles of the phase
        int cur_slab = -1;
        Frag b[4][2];
#pragma unroll
        for (int q = 0; q < 4; ++q) b[q][0].q = b[q][1].q = u32x4{0, 0, 0, 0};
        while (cur.p == p) {
#pragma unroll
            for (int c = 0; c < kMegaCh; ++c) reinterpret_cast<u32x4*>(buf)[c * 64 + lane] = st[c];
            const uint2 mk = mk_next;
            const int sl_strip = cur.ss, sl_slab = cur.sl;
            if (sl_slab != cur_slab) {
                cur_slab = sl_slab;
                if (n < kMegaMaxTok) {
                    const u32x4* xr = reinterpret_cast<const u32x4*>(xlds + (sl_slab * kMegaMaxTok + n) * 256 + 16 * g);
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
                const unsigned char* bl = ka->blob[nxt.p];
                issue_tile<kMegaCh>(st, mk_next, reinterpret_cast<const uint16_t*>(bl + ka->geo[nxt.p & 3].val_off),
                                    reinterpret_cast<const uint2*>(bl + ka->geo[nxt.p & 3].mask_off), de_cur.val_start,
                                    de_cur.nnz, nxt.t, lane);
            }
            const TileRef n3 = next_tile(ka, cu, nn, n_phases, wave);
            de_raw = load_dir_raw(ka, n3, n_phases, lane);

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
            // ---- add to this strip's accumulator in LDS: lane (n, g) owns rows 4g..4g+3 of token n
            if (n < kMegaMaxTok) {
                float* r = red + (sl_strip * kMegaMaxTok + n) * 16 + 4 * g;
#pragma unroll
                for (int v = 0; v < 4; ++v) atomicAdd(r + v, acc[v]);
            }
            cur = nxt;
            nxt = nn;
            nn = n3;
        }
        __syncthreads();
        if (tt && tid == 0) tt[3] = __builtin_amdgcn_s_memrealtime();

        // ---------------- the block's results leave the CU: split-K across the slab blocks by float atomics
        if (active) {
            float* ybase = kind == 0 ? yq : (kind == 2 ? yg : a.h);
            for (int idx = tid; idx < ge.s_blk * kMegaMaxTok * 16; idx += kMegaThreads) {
                const int r = idx & 15, t = (idx >> 4) & (kMegaMaxTok - 1), sl = idx >> 7;
                const float v = red[idx];
                red[idx] = 0.f;
                const int strip = kpl.strip0 + sl, row = strip * 16 + r;
                if (t < k_tok && strip < ge.n_strips && row < ge.n_out) aadd(ybase + (size_t)t * ge.n_out + row, v);
            }
        }
    }
}

// ---------------------------------------------------------------- set-up kernels and launch

__global__ __launch_bounds__(256) void mega_zero_kernel(uint32_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

__global__ __launch_bounds__(256) void mega_h_init_kernel(float* __restrict__ h, const uint16_t* __restrict__ h_in, size_t n) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) h[i] = bf16_to_f32(h_in[i]);
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

MegaLayout mega_layout(int layers, int hidden, int q_out, int kv_out, int inter, int k_tok) {
    (void)layers;
    (void)hidden;
    MegaLayout L;
    size_t off = 0;
    L.bar_off = off;
    off += align256((size_t)kBarWords * 4);
    L.err_off = off;
    off += 256;
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
            hipFuncSetAttribute(reinterpret_cast<const void*>(mega_forward_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMegaLds) == hipSuccess &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(mega_forward_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMegaLds) == hipSuccess) {
            int per_cu = 0, per_cu_t = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, mega_forward_kernel<false>, kMegaThreads, kMegaLds) == hipSuccess &&
                hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_t, mega_forward_kernel<true>, kMegaThreads, kMegaLds) == hipSuccess &&
                per_cu >= 1 && per_cu_t >= 1)
                cus = n;
        }
    }
    return cus;
}

int mega_grid_size() { return mega_grid(); }

// Block of s strips x b slabs per workgroup: fewest tiles per workgroup, then the widest block
// (fewer slab blocks mean fewer float atomics leaving the CU).
static bool plan_kind(MegaGeo& g, int ncu, int max_b) {
    long best_cost = -1;
    for (int b = 1; b <= max_b && b <= g.n_slabs; ++b) {
        const int n_bblk = (g.n_slabs + b - 1) / b;
        const int max_sblk = ncu / n_bblk;
        if (max_sblk < 1) continue;
        const int s = (g.n_strips + max_sblk - 1) / max_sblk;
        if (s > kMaxS) continue;
        const long cost = (long)s * b;
        if (best_cost < 0 || cost < best_cost || (cost == best_cost && b > g.b_blk)) {
            best_cost = cost;
            g.s_blk = s;
            g.b_blk = b;
            g.n_sblk = (g.n_strips + s - 1) / s;
            g.n_bblk = n_bblk;
        }
    }
    return best_cost > 0;
}

bool mega_plan(MegaGeo (&geo)[4], int layers, int hidden, int head_dim, int k_tok, int max_tile_nnz) {
    if (layers < 1 || layers > kMegaMaxLayers || head_dim != 128 || k_tok < 1 || k_tok > kMegaMaxTok) return false;
    if (hidden > kMegaMaxHidden || max_tile_nnz * 2 + 8 > kMegaCh * 1024) return false;
    const int ncu = mega_grid();
    if (ncu < 1) return false;
    for (int k = 0; k < 4; ++k)
        if (!plan_kind(geo[k], ncu, k == 1 ? kMaxBAtt : kMaxB)) return false;
    return true;
}

hipError_t launch_mega_forward(const MegaArgs& a, const uint16_t* h_in, void* zero_base, size_t zero_bytes, hipStream_t s) {
    const int ncu = mega_grid();
    if (ncu < 1) return hipErrorNotSupported;
    hipLaunchKernelGGL(mega_zero_kernel, dim3(256), dim3(256), 0, s, static_cast<uint32_t*>(zero_base), zero_bytes / 4);
    const size_t nh = (size_t)a.k_tok * a.hidden;
    hipLaunchKernelGGL(mega_h_init_kernel, dim3((unsigned)((nh + 255) / 256)), dim3(256), 0, s, a.h, h_in, nh);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    MegaArgs args = a;
    void* params[] = {&args};
    const void* fn = a.trace_x ? reinterpret_cast<const void*>(mega_forward_kernel<true>)
                               : reinterpret_cast<const void*>(mega_forward_kernel<false>);
    return hipLaunchCooperativeKernel(fn, dim3((unsigned)ncu), dim3(kMegaThreads), params, kMegaLds, s);
}

}  // namespace sd2
