// Whole-forward persistent kernel for the sparse drafter stack on gfx950.
//
// One workgroup of 12 wavefronts per CU lives for the entire forward.  For every linear a
// workgroup owns a block of s strips x b slabs of 16x256 weight tiles; its wavefronts walk those
// tiles, and each wavefront keeps the compacted stream of its next tile in flight -- also across
// the end of a linear, because weights never depend on activations -- so HBM keeps streaming
// while the grid synchronises.  Tile results are summed per strip in LDS and leave the CU once
// per linear as integer atomic adds of fixed-point numbers (split-K only across the few slab blocks):
// integer sums are exact, so their order does not matter and the forward is bit-reproducible.  Between
// dependent linears the grid meets at a barrier built from agent-scope atomics.  Everything a CU hands to
// other CUs is written with agent-scope atomic stores / integer adds, which go through to memory,
// so no cache write-back is needed before arriving; nothing is invalidated after the barrier either:
// every activation buffer exists once per layer, so what the prologue reads (with ordinary cached loads)
// lies at addresses no compute unit has touched before in this launch.  After each barrier a workgroup
// rebuilds in LDS exactly the bf16 activation columns its tiles need: the RMS-normed residual
// (every workgroup sums the squares of the whole residual itself), causal attention over the
// in-flight tokens for the heads of its slabs, or the SiLU-gated product.
#include <algorithm>
#include <atomic>
#include <type_traits>

#include "sd2_device.h"
#include "sd2_internal.h"

#ifndef SD2_MEGA_STEPS
#define SD2_MEGA_STEPS 2  // super-steps per batch of LDS reads in the tile expansion
#endif

namespace sd2 {

constexpr int kMegaWaves = 12;
constexpr int kMegaThreads = 64 * kMegaWaves;
constexpr int kMegaCh = 5;                          // 1 KiB pieces of a staged tile
constexpr int kTileDw = kMegaCh * 256;              // dwords per wavefront tile buffer
constexpr int kMaxB = 6;                            // slabs per workgroup block (activation columns kept in LDS)
constexpr int kMaxBAtt = 3;                         // ... for the linear that follows attention
constexpr int kMaxS = 16;                           // strips per workgroup block (LDS accumulators)
// A token's 256 activation columns of a slab take a row of 264 bf16: with 528-byte rows the eight tokens that read
// the same 16 columns for the MFMA B operand (one 16-byte read per lane) fall into eight different bank groups.
constexpr int kXRow = 264;
constexpr int kXldsDw = kMaxB * kMegaMaxTok * kXRow / 2;  // bf16 [slab][token][kXRow]
constexpr int kMaxUnits = 24;                           // (strip, slab group) units of a block: one result slot each
constexpr int kRedDw = kMaxUnits * kMegaMaxTok * 16;    // fp32 [strip][group][token][row]
constexpr int kPlanDw = 16;                             // per-kind plan: s_eff b_eff strip0 slab0 | n_strips 1/grp_slabs active tiles/wave | mask_off(2) val_off(2) | grp_slabs n_grp 1/n_grp -
constexpr int kMiscDw = 544;                            // attention probabilities, per-token scalars
constexpr int kAttHeads = 6;                            // heads (and kv heads) one workgroup may need
constexpr int kAreaDw = 2 * kMegaWaves * kTileDw;       // two tile buffers per wavefront: one being expanded, one being filled
constexpr size_t kMegaLds = (size_t)(kAreaDw + kXldsDw + kRedDw + kMiscDw + 4 * kPlanDw) * 4;
constexpr int kBarWords = 8 * 32;                   // 8 group counters, one per 128-byte line
static_assert(kAttHeads * 128 == kMegaThreads, "one thread per (head slot, dimension)");
static_assert(4 * kMegaThreads >= kMegaMaxHidden && 2 * kMegaThreads >= kMaxB * 256, "columns per thread in the prologues");
static_assert(kMaxBAtt * 256 <= kAttHeads * 128, "attention block fits the head slots");

#define SD2_AGENT __HIP_MEMORY_SCOPE_AGENT

// Activations cross compute units through memory: written by agent-scope stores and integer atomics, read (after a
// grid barrier, at addresses no compute unit has read before in this launch) with ordinary loads.
__device__ __forceinline__ void astore(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, SD2_AGENT); }
__device__ __forceinline__ void astore_i(int* p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, SD2_AGENT); }
__device__ __forceinline__ void aadd_i(int* p, int v) { (void)__hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, SD2_AGENT); }

// What crosses compute units as a sum of several workgroups' contributions (the results of a linear whose contraction
// is split over slab blocks, and the residual stream they are added to) is kept in 32-bit fixed point: a workgroup
// adds up its tiles in fp32, rounds its contribution once to a multiple of 2^-F and adds it with an integer atomic.
// Integer adds are exact, so the sum does not depend on the order in which the workgroups arrive -- the forward is
// bit-reproducible -- and a consumer reads four bytes per value, as it would for fp32.  F = 17 by default: resolution
// 7.6e-6 (the fp32 spacing at magnitude 64; activations are rounded to bf16, spacing 2^-8 relative, before their next
// use), range +-16384.  No sum can wrap unnoticed: a contribution must stay below 2^30 / (slab blocks of its linear)
// in fixed point, and a token's residual below 2^30 in norm (checked where the norm is computed anyway); whatever
// breaks that raises bit 1 of the error word, which the status calls report as SD2_ERR_RANGE.
__device__ __forceinline__ float from_fixed(int w, float inv) { return (float)w * inv; }
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));

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

// The same for N values at once, stage by stage: the N cross-lane adds of a stage are independent, so they issue back to
// back and fill the wait states that a chain of dependent cross-lane operations would spend idle.  Result in lane 63.
template <int N>
__device__ __forceinline__ void wave_sums_lane63(float (&v)[N]) {
#define SD2_DPP_STAGE(ctrl, rmask) \
    _Pragma("unroll") for (int i = 0; i < N; ++i) \
        v[i] += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v[i]), ctrl, rmask, 0xf, true))
    SD2_DPP_STAGE(0x111, 0xf);  // row_shr:1
    SD2_DPP_STAGE(0x112, 0xf);  // row_shr:2
    SD2_DPP_STAGE(0x114, 0xf);  // row_shr:4
    SD2_DPP_STAGE(0x118, 0xf);  // row_shr:8
    SD2_DPP_STAGE(0x142, 0xa);  // row_bcast:15
    SD2_DPP_STAGE(0x143, 0xc);  // row_bcast:31
#undef SD2_DPP_STAGE
}

// The argument block as it sits in the kernarg segment: indexing it with a run-time (wave-uniform) index
// gives scalar loads, where indexing the by-value parameter would make the compiler copy it to scratch.
typedef const __attribute__((address_space(4))) MegaArgs* KArgs;

// Per-kind plan in LDS, written once by threads 0..3: the part of the matrix this workgroup owns (clipped to
// the matrix, so every position of the s_eff x b_eff block is a real tile) and the blob offsets common to all
// layers of the kind.
constexpr int kMaxTilesPerWave = 8;  // per phase: ceil(kMaxS * kMaxB / waves)
constexpr int kFlushIters = (kMaxS * kMegaMaxTok * 16 + kMegaThreads - 1) / kMegaThreads;  // results per thread leaving the CU


__device__ __forceinline__ int uni(uint32_t v) { return __builtin_amdgcn_readfirstlane((int)v); }

// This wavefront's tiles of one phase, described in lanes.  A block's work is cut into units: the slabs of a
// strip form n_grp groups of grp_slabs consecutive slabs, unit u = strip * n_grp + group.  Units are dealt to the
// wavefronts in runs (unit order), and a wavefront walks the tiles of a unit one after the other, so that the sums
// of a unit stay in the MFMA accumulator and reach LDS once, with a plain store into the unit's own slot.
// Tile j of the wavefront is position i = wave * per_wave + j of that walk.  Lane L holds what belongs to tile
// L / 8: its index in the matrix, a key (place in the block and flags), and (lanes 8j + d) the dwords of its
// directory entry.  One pass of vector arithmetic and two loads per phase replace per-tile index juggling; a
// tile's numbers are then picked with v_readlane at lane 8j.  A position whose slab lies past the matrix (ragged
// last block) is an empty tile: nothing is loaded for it and its masks are zero.
struct PhaseTiles {
    uint32_t t;    // tile index in the matrix
    uint32_t key;  // strip in block | slab in block << 8 | unit << 16 | first of unit << 24 | last << 25 | empty << 26
    uint32_t ra;   // lane 8j + d: directory dword d       (val_start, nnz, run bases 0..11)
    uint32_t rb;   // lane 8j + d: directory dword 8 + d   (run bases 12..15 in d = 0, 1)
    int n;         // number of tiles (wave-uniform)
    const unsigned char* masks;  // mask section of the phase's blob
    const unsigned char* vals;   // value section
};

constexpr uint32_t kKeyFirst = 1u << 24, kKeyLast = 1u << 25, kKeyEmpty = 1u << 26;

template <bool NM24>
__device__ __forceinline__ void plan_phase(PhaseTiles& pt, KArgs ka, const uint32_t* plans, int p, int n_phases, int wave,
                                           int lane) {
    pt.t = pt.key = pt.ra = pt.rb = 0u;
    pt.n = 0;
    pt.masks = pt.vals = nullptr;
    if (p >= n_phases) return;
    const u32x4* e = reinterpret_cast<const u32x4*>(plans + (p & 3) * kPlanDw);
    const u32x4 a = e[0], b = e[1], c = e[2], d4 = e[3];  // same address in every lane: broadcast reads, values stay in VGPRs
    const int s_eff = (int)a[0], b_eff = (int)a[1], per_wave = (int)b[3];
    const int grp_slabs = (int)d4[0], n_grp = (int)d4[1];
    const int j = lane >> 3;
    const int i = wave * per_wave + j;
    // exact for these small integers: i / grp_slabs, u / n_grp
    const int u = (int)(((float)i + 0.5f) * __uint_as_float(b[1]));
    const int r = i - u * grp_slabs;
    const int ss = (int)(((float)u + 0.5f) * __uint_as_float(d4[2]));
    const int grp = u - ss * n_grp;
    const int sl = grp * grp_slabs + r;
    const bool exists = j < per_wave && ss < s_eff;
    const bool empty = sl >= b_eff;
    const uint32_t t = (a[3] + (uint32_t)sl) * b[0] + a[2] + (uint32_t)ss;
    const unsigned char* blob = ka->blob[p];
    pt.masks = blob + ((unsigned long long)(uint32_t)uni(c[0]) | ((unsigned long long)(uint32_t)uni(c[1]) << 32));
    pt.vals = blob + ((unsigned long long)(uint32_t)uni(c[2]) | ((unsigned long long)(uint32_t)uni(c[3]) << 32));
    pt.n = __builtin_popcountll(__ballot(exists && (lane & 7) == 0));
    if (exists) {
        pt.key = (uint32_t)ss | ((uint32_t)sl << 8) | ((uint32_t)u << 16) | (r == 0 ? kKeyFirst : 0u) |
                 (r == grp_slabs - 1 ? kKeyLast : 0u) | (empty ? kKeyEmpty : 0u);
        if (!empty) {
            pt.t = t;
            if (!NM24) {  // the 2:4 format has no directory: tiles have one size
                const uint32_t* d = reinterpret_cast<const uint32_t*>(blob + 128) + (size_t)t * 12;
                pt.ra = d[lane & 7];
                pt.rb = d[8 + (lane & 3)];
            }
        }
    }
}

__device__ __forceinline__ uint32_t lane_word(uint32_t v, int l) { return (uint32_t)__builtin_amdgcn_readlane((int)v, l); }

// Requests the value stream (straight into LDS) and the masks of tile j of a phase.  A 2:4 tile is 4608 bytes in
// the layout of the structured-sparse matrix instruction: four KiB of values, then 512 bytes of column indices.
//
// Invariant for every direct-to-LDS request of this kernel: the buffer it fills is one whose previous contents are
// dead -- the request before it into that buffer was drained by a full wait (vmcnt(0): nothing here is decided by
// counting outstanding loads, so no assumption about their completion order is made), and the expansion that read
// those contents has ended, i.e. its LDS reads have returned (their results were consumed before this point in
// program order).  A wavefront never has two requests for one buffer in flight.  Lanes past a tile's last 16-byte
// piece repeat that piece's source address, each into a destination of its own that no window reads.
template <bool NM24>
__device__ __forceinline__ void issue_phase_tile(const PhaseTiles& pt, int j, uint32_t* lds_buf, uint2& mk, int lane) {
    if (lane_word(pt.key, 8 * j) & kKeyEmpty) {  // nothing stored for it: all-zero masks expand to zeros
        mk = make_uint2(0u, 0u);
        return;
    }
    if (NM24) {
        const u32x4* src = reinterpret_cast<const u32x4*>(pt.vals + (size_t)lane_word(pt.t, 8 * j) * 4608);
#pragma unroll
        for (int c = 0; c < 4; ++c)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + c * 64 + lane),
                                             (__attribute__((address_space(3))) void*)(lds_buf + c * 256), 16, 0, 0);
        if (lane < 32)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + 256 + lane),
                                             (__attribute__((address_space(3))) void*)(lds_buf + 1024), 16, 0, 0);
        mk = make_uint2(0u, 0u);
        return;
    }
    const uint32_t val_start = lane_word(pt.ra, 8 * j), nnz = lane_word(pt.ra, 8 * j + 1), t = lane_word(pt.t, 8 * j);
    issue_tile_lds<kMegaCh>(lds_buf, mk, reinterpret_cast<const uint16_t*>(pt.vals),
                            reinterpret_cast<const uint2*>(pt.masks + (size_t)t * 512), val_start, nnz, lane);
}

// The sixteen run bases of tile j as the eight directory words that hold them.
__device__ __forceinline__ void tile_bases(const PhaseTiles& pt, int j, int lane, uint32_t (&base)[8]) {
    // bring the tile's lanes down to lanes 0..7 (one cross-lane move each), then pick with constant lane numbers
    const int src = ((lane + 8 * j) & 63) * 4;
    const uint32_t ra = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)pt.ra);
    const uint32_t rb = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)pt.rb);
#pragma unroll
    for (int i = 0; i < 6; ++i) base[i] = lane_word(ra, 2 + i);
    base[6] = lane_word(rb, 0);
    base[7] = lane_word(rb, 1);
}

// Workgroup barrier that orders LDS traffic only: the wavefront's own LDS operations have completed, loads and stores
// to memory stay in flight (a __syncthreads would also wait for every store acknowledgement: about a microsecond).
__device__ __forceinline__ void lds_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Grid barrier: the workgroups form 8 groups (by id mod 8), each with an arrival counter of its own in a separate
// cache line.  Counters only grow; `gen` is the number of barriers passed, so after barrier number gen counter g
// holds gen * (size of group g).  Arriving is one atomic add whose result nobody waits for; waiting is eight lanes
// of one wavefront polling the eight counters side by side, so a barrier costs about one trip to memory and back
// after the last arrival.  Waits are bounded: on overrun *err is set and the kernel keeps going (results are then
// invalid, but every wave still terminates).
//
// The barrier comes in two halves so that a wavefront can expand its next weight tile (which needs no
// activations) between announcing its arrival and waiting for the release.
//
// Arrive: every wavefront has its stores and atomics acknowledged; thread 0 then counts the workgroup in.
__device__ __forceinline__ void barrier_arrive(unsigned* bar, unsigned& gen) {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    gen += 1;
    if (threadIdx.x == 0) (void)__hip_atomic_fetch_add(&bar[(blockIdx.x & 7u) * 32], 1u, __ATOMIC_RELAXED, SD2_AGENT);
}

// Wait: lanes 0..7 of the first wavefront poll the group counters (bounded), then the workgroup goes on together.
__device__ __forceinline__ void barrier_wait(unsigned* bar, unsigned* err, unsigned ncu, unsigned gen, int& spin_limit) {
    if (threadIdx.x < 64) {
        const unsigned g = threadIdx.x;
        const unsigned ngrp = ncu < 8u ? ncu : 8u;
        const unsigned want = g < ngrp ? gen * ((ncu - g + 7u) / 8u) : 0u;
        int spins = 0;
        for (;;) {
            const unsigned have = g < ngrp ? __hip_atomic_load(&bar[g * 32], __ATOMIC_RELAXED, SD2_AGENT) : 0u;
            if (__all(have >= want)) break;  // wave-uniform exit
            __builtin_amdgcn_s_sleep(1);
            if (++spins > spin_limit) {
                if (g == 0) __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, SD2_AGENT);
                spin_limit = 0;  // the forward is lost: later barriers of this wavefront give up at once
                break;
            }
        }
    }
    // No cache invalidation: what is read after a barrier lies at addresses no CU has read before in this launch.
    // The workgroup goes on together; weight streams already requested for the coming tiles stay in flight.
    lds_barrier();
}

// A 2:4 tile in registers: the sparse operands of its four matrix instructions and their column indices.
struct Tile24 {
    u32x4 v[4];
    uint2 idx;
};
typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 bf16x16;
union Frag16 {
    u32x4 q[2];
    bf16x16 v;
};

__device__ __forceinline__ void read_tile24(Tile24& t, const uint8_t* bufb, int lane) {
#pragma unroll
    for (int q = 0; q < 4; ++q) t.v[q] = *reinterpret_cast<const u32x4*>(bufb + (64 * q + lane) * 16);
    t.idx = *reinterpret_cast<const uint2*>(bufb + 4096 + 8 * lane);
}

// ---- attention over the key/value cache, one stretch of positions per workgroup
//
// Work item (key/value head g, token t, chunk c): the group's query heads of token t against the cache positions of
// chunk c (the history is cut into att_chunks equal stretches; the last chunk also takes the call's own tokens
// 0 .. t, whose keys and values come from this layer's q|k|v result: rotated, rounded to bf16 as the cache holds
// them; the item of token t stores that token's row in the cache for later calls).  A cache row is read by 16
// consecutive lanes (16 bytes each), a wavefront reads four consecutive rows, the workgroup 48 per pass, four passes
// in flight.  Scores stay in registers; the running maximum is agreed across the workgroup per 192 rows (online
// softmax), sums and weighted values meet in LDS at the end.  Result per head: maximum, sum of exponentials and the
// unnormalised weighted values, which the workgroups of the next linear combine over the chunks.
constexpr int kAttSo = 0, kAttMax = kMegaWaves * 4 * 128, kAttSum = kAttMax + kMegaWaves * 8;
static_assert(kAttSum + kMegaWaves * 8 <= kXldsDw, "attention scratch fits the activation area");

__device__ __forceinline__ void bf16x8_unpack(const u32x4 w, float (&f)[8]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = __uint_as_float(w[e] << 16);
        f[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
}

// four consecutive results of the q|k|v linear (fixed point) as fp32
__device__ __forceinline__ f32x4 load_fixed4(const int* __restrict__ p, float inv) {
    const i32x4 w = *reinterpret_cast<const i32x4*>(p);
    return f32x4{from_fixed(w[0], inv), from_fixed(w[1], inv), from_fixed(w[2], inv), from_fixed(w[3], inv)};
}

// dimensions 8 piece .. 8 piece + 7 of a head (128 fixed-point values at `head`) after the rotation of token u
__device__ __forceinline__ void rotated_piece(const int* __restrict__ head, float inv, const float2* __restrict__ rope, int u, int piece,
                                              float (&out)[8]) {
    const int d0 = 8 * piece, i0 = d0 & 63;
    const f32x4 a0 = load_fixed4(head + d0, inv), a1 = load_fixed4(head + d0 + 4, inv);
    const f32x4 b0 = load_fixed4(head + (d0 ^ 64), inv), b1 = load_fixed4(head + (d0 ^ 64) + 4, inv);
    const f32x4* cs = reinterpret_cast<const f32x4*>(rope + (size_t)u * 64 + i0);  // (cos, sin) pairs, two per load
    const float sgn = d0 < 64 ? -1.f : 1.f;  // lower half: x cos - y sin; upper half: x cos + y sin
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const f32x4 c2 = cs[e >> 1];
        const float co = c2[2 * (e & 1)], si = c2[2 * (e & 1) + 1];
        const float x = e < 4 ? a0[e & 3] : a1[e & 3], y = e < 4 ? b0[e & 3] : b1[e & 3];
        out[e] = x * co + sgn * (y * si);
    }
}

__device__ __forceinline__ u32x4 pack_bf16x8(const float (&f)[8]) {
    return u32x4{pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3]), pack_bf16(f[4], f[5]), pack_bf16(f[6], f[7])};
}

constexpr int kAttUnr = 2;                 // passes of a workgroup's cache loads in flight
constexpr int kAttRpi = kMegaWaves * 4;    // cache rows per pass: four per wavefront

struct AttItem {
    int c, t, g;     // chunk, token, key/value head
    int j_lo, j_hi;  // positions [j_lo, j_hi): cache rows below pos0, the call's own tokens from pos0 on
};

__device__ __forceinline__ AttItem att_geometry(KArgs ka, int item) {
    const int k_tok = ka->k_tok, C = ka->att_chunks, pos0 = ka->pos0;
    AttItem it;
    it.c = item % C;
    it.t = (item / C) % k_tok;
    it.g = item / (C * k_tok);
    const int per = (pos0 + C - 1) / C;
    it.j_lo = min(it.c * per, pos0);
    it.j_hi = it.c == C - 1 ? pos0 + it.t + 1 : min(pos0, it.j_lo + per);
    return it;
}

// The cache rows of one pass group starting at `base` (this lane's 16 bytes of each): nothing of them depends on the
// current layer, so the first group is requested before the barrier that completes q|k|v.
__device__ __forceinline__ void attention_loads(KArgs ka, int layer, const AttItem& it, int base, int tid, u32x4 (&kw)[kAttUnr],
                                                u32x4 (&vw)[kAttUnr]) {
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int piece = lane & 15, slot = wave * 4 + (lane >> 4);
    const size_t head = ((size_t)layer * ka->n_kv + it.g) * ka->max_pos * 128;
    const u32x4* kg = reinterpret_cast<const u32x4*>(ka->k_cache + head) + piece;
    const u32x4* vg = reinterpret_cast<const u32x4*>(ka->v_cache + head) + piece;
    const int lim = min(it.j_hi, ka->pos0);
#pragma unroll
    for (int u = 0; u < kAttUnr; ++u) {
        const int j = base + u * kAttRpi + slot;
        kw[u] = j < lim ? kg[(size_t)j * 16] : u32x4{0u, 0u, 0u, 0u};
        vw[u] = j < lim ? vg[(size_t)j * 16] : u32x4{0u, 0u, 0u, 0u};
    }
}

template <int REP>
__device__ __forceinline__ void attention_item(KArgs ka, int layer, const AttItem& it, float* scratch, int tid,
                                               u32x4 (&kw)[kAttUnr], u32x4 (&vw)[kAttUnr]) {
    constexpr int D = 128, RPI = kAttRpi, UNR = kAttUnr;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int piece = lane & 15, slot = wave * 4 + (lane >> 4);
    const int k_tok = ka->k_tok, C = ka->att_chunks, n_kv = ka->n_kv, n_heads = ka->n_heads;
    const int rep = n_heads / n_kv;
    const int c = it.c, t = it.t, g = it.g, j_lo = it.j_lo, j_hi = it.j_hi;
    const int pos0 = ka->pos0, max_pos = ka->max_pos, q_out = ka->q_out, kv_out = ka->kv_out;
    const int nqkv = q_out + 2 * kv_out;
    const int* yq = ka->yqkv + (size_t)layer * ka->yqkv_stride;
    const float2* rope = ka->rope;
    float* so = scratch + kAttSo;
    float* smax = scratch + kAttMax;
    float* ssum = scratch + kAttSum;
    const float scale = 0.08838834764831845f;  // 1 / sqrt(128)

    // One rotation per row slot, all requested at once: slots below REP take the group's queries of token t (scaled,
    // kept in LDS as [REP][128] floats and read back piece by piece in the loop: registers go to the running sums);
    // in the last chunk the next t + 1 slots take the call's own tokens 0 .. t: key rotated, key and value rounded to
    // bf16 as the cache holds them, kept in LDS for the loop; token t's row also goes to the cache, for later calls.
    u32x4* own_k = reinterpret_cast<u32x4*>(scratch);  // [kMegaMaxTok][16 pieces]
    u32x4* own_v = own_k + kMegaMaxTok * 16;
    f32x4* sq = reinterpret_cast<f32x4*>(scratch + 2 * kMegaMaxTok * 64);
    const int n_own = c == C - 1 ? t + 1 : 0;
    if (slot < REP + n_own) {
        const bool is_q = slot < REP;
        const int tok = is_q ? t : slot - REP;
        const int* head = yq + (size_t)tok * nqkv + (is_q ? (size_t)(g * rep + min(slot, rep - 1)) * D : q_out + (size_t)g * D);
        const float fix_inv = ka->fix_inv;
        float f[8];
        rotated_piece(head, fix_inv, rope, tok, piece, f);
        if (is_q) {
            sq[slot * 32 + 2 * piece] = f32x4{f[0] * scale, f[1] * scale, f[2] * scale, f[3] * scale};
            sq[slot * 32 + 2 * piece + 1] = f32x4{f[4] * scale, f[5] * scale, f[6] * scale, f[7] * scale};
        } else {
            const int* src = head + kv_out + 8 * piece;  // the value head sits kv_out values after the key head
            const f32x4 v0 = load_fixed4(src, fix_inv), v1 = load_fixed4(src + 4, fix_inv);
            const u32x4 pk = pack_bf16x8(f);
            const u32x4 pv = u32x4{pack_bf16(v0[0], v0[1]), pack_bf16(v0[2], v0[3]), pack_bf16(v1[0], v1[1]), pack_bf16(v1[2], v1[3])};
            own_k[tok * 16 + piece] = pk;
            own_v[tok * 16 + piece] = pv;
            if (tok == t) {
                const size_t at = (((size_t)layer * n_kv + g) * max_pos + (size_t)(pos0 + t)) * D + 8 * piece;
                *reinterpret_cast<u32x4*>(ka->k_cache + at) = pk;
                *reinterpret_cast<u32x4*>(ka->v_cache + at) = pv;
            }
        }
    }
    lds_barrier();

    float M[REP], L[REP], acc[REP][8];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        M[r] = -3.0e38f;
        L[r] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
    }
    for (int base = j_lo; base < j_hi; base += RPI * UNR) {
        if (base != j_lo) attention_loads(ka, layer, it, base, tid, kw, vw);  // the first group is already on its way
        float sdot[REP][UNR], mx[REP];
#pragma unroll
        for (int r = 0; r < REP; ++r) mx[r] = -3.0e38f;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int j = base + u * RPI + slot;
            float kf[8];
            bf16x8_unpack((j >= pos0 && j < j_hi) ? own_k[(j - pos0) * 16 + piece] : kw[u], kf);
#pragma unroll
            for (int r = 0; r < REP; ++r) {
                const f32x4 q0 = sq[r * 32 + 2 * piece], q1 = sq[r * 32 + 2 * piece + 1];
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) dot += kf[e] * q0[e] + kf[4 + e] * q1[e];
                dot += __shfl_xor(dot, 1);
                dot += __shfl_xor(dot, 2);
                dot += __shfl_xor(dot, 4);
                dot += __shfl_xor(dot, 8);
                sdot[r][u] = j < j_hi ? dot : -3.0e38f;
                mx[r] = fmaxf(mx[r], sdot[r][u]);
            }
        }
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            float m = fmaxf(mx[r], __shfl_xor(mx[r], 16));
            m = fmaxf(m, __shfl_xor(m, 32));
            if (lane == 0) smax[wave * 8 + r] = m;
        }
        lds_barrier();
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            float m = M[r];
#pragma unroll 4
            for (int ww = 0; ww < kMegaWaves; ++ww) m = fmaxf(m, smax[ww * 8 + r]);
            const float f = __expf(M[r] - m);
            M[r] = m;
            L[r] *= f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] *= f;
        }
        lds_barrier();
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int j = base + u * RPI + slot;
            float vf[8];
            bf16x8_unpack((j >= pos0 && j < j_hi) ? own_v[(j - pos0) * 16 + piece] : vw[u], vf);
#pragma unroll
            for (int r = 0; r < REP; ++r) {
                const float pr = j < j_hi ? __expf(sdot[r][u] - M[r]) : 0.f;
                L[r] += pr;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[r][e] += pr * vf[e];
            }
        }
    }
    lds_barrier();  // the rows of the call's own tokens and the queries share LDS with the sums below
    // the sixteen lanes of a row all counted its weight: a wavefront's total is the sum over its lanes / 16
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        const float l = wave_sum(L[r]) * 0.0625f;
        if (lane == 0) {
            ssum[wave * 8 + r] = l;
            if (wave == 0) smax[r] = M[r];  // the same in every thread
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[r][e];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (lane < 16) so[(wave * 4 + r) * D + 8 * piece + e] = v;
        }
    }
    lds_barrier();
    for (int idx = tid; idx < rep * D; idx += kMegaThreads) {
        const int r = idx >> 7, d = idx & 127;
        float o = 0.f;
#pragma unroll 4
        for (int ww = 0; ww < kMegaWaves; ++ww) o += so[(ww * 4 + r) * D + d];
        float* dst = ka->att_part + ((((size_t)layer * k_tok + t) * n_heads + (size_t)g * rep + r) * C + c) * kMegaAttPartDw;
        astore(dst + 4 + d, o);
        if (d == 0) {
            float l = 0.f;
#pragma unroll 4
            for (int ww = 0; ww < kMegaWaves; ++ww) l += ssum[ww * 8 + r];
            astore(dst, smax[r]);
            astore(dst + 1, l);
        }
    }
    lds_barrier();
}

template <bool TRACE, bool PROBE, bool NM24, int KV = 0>
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
    // Results leave the CU as (strip, token, row) triples dealt to the threads: entry q = idx / 16 is strip q / k_tok, token
    // q % k_tok; for q < 128 and k_tok <= 8 the quotient is (q * ceil(1024 / k_tok)) >> 10.
    const uint32_t tok_mul = (1024u + (uint32_t)k_tok - 1u) / (uint32_t)k_tok;
    static_assert(kMaxS * kMegaMaxTok <= 128 && kMegaMaxTok <= 8, "range in which the multiply-shift division is exact");
    KArgs ka = (KArgs)__builtin_amdgcn_kernarg_segment_ptr();

    uint32_t* bufs = mega_lds + wave * (2 * kTileDw);           // this wave's two tile buffers
    int cb = 0;                                                 // the one the current tile's stream is in (or on its way to)
    uint16_t* xlds = reinterpret_cast<uint16_t*>(mega_lds + kAreaDw);
    float* red = reinterpret_cast<float*>(mega_lds + kAreaDw + kXldsDw);
    float* misc = red + kRedDw;                                 // [0,432) attention scores / probabilities
    float* part_sums = misc + 448;                              // [token][wave] sums of squares of a wavefront's columns
    static_assert(448 + kMegaMaxTok * kMegaWaves <= kMiscDw && (kAreaDw + kXldsDw + kRedDw + 448) % 4 == 0, "partial sums fit, 16-byte aligned");
    if (tid < 16) lut[tid] = make_expand_selector((uint32_t)tid);
    for (int i = tid; i < kRedDw + kMiscDw; i += kMegaThreads) red[i] = 0.f;  // accumulators, scores, sums
    for (int i = tid; i < kXldsDw; i += kMegaThreads) (mega_lds + kAreaDw)[i] = 0u;  // rows of unused token slots stay zero

    // per-kind plans -> LDS
    uint32_t* plans = reinterpret_cast<uint32_t*>(misc + kMiscDw);
    if (tid < 4) {
        const int n_sblk = ka->geo[tid].n_sblk, n_bblk = ka->geo[tid].n_bblk;
        const int s_blk = ka->geo[tid].s_blk, b_blk = ka->geo[tid].b_blk;
        const int qb = cu / n_sblk;
        const int strip0 = (cu - qb * n_sblk) * s_blk, slab0 = qb * b_blk;
        const bool act = cu < n_sblk * n_bblk;
        const int s_eff = act ? max(0, min(s_blk, ka->geo[tid].n_strips - strip0)) : 0;
        const int b_eff = act ? max(0, min(b_blk, ka->geo[tid].n_slabs - slab0)) : 0;
        const int n_grp = max(ka->geo[tid].n_grp, 1), grp_slabs = max(ka->geo[tid].grp_slabs, 1);
        const int units_per_wave = (s_blk * n_grp + kMegaWaves - 1) / kMegaWaves;
        uint32_t* e = plans + tid * kPlanDw;
        e[0] = (uint32_t)(b_eff > 0 ? s_eff : 0);
        e[1] = (uint32_t)b_eff;
        e[2] = (uint32_t)strip0;
        e[3] = (uint32_t)slab0;
        e[4] = (uint32_t)ka->geo[tid].n_strips;
        e[5] = __float_as_uint(1.0f / (float)grp_slabs);
        e[6] = act ? 1u : 0u;
        e[7] = (uint32_t)(units_per_wave * grp_slabs);  // tiles per wavefront
        e[8] = (uint32_t)ka->geo[tid].mask_off;
        e[9] = (uint32_t)(ka->geo[tid].mask_off >> 32);
        e[10] = (uint32_t)ka->geo[tid].val_off;
        e[11] = (uint32_t)(ka->geo[tid].val_off >> 32);
        e[12] = (uint32_t)grp_slabs;
        e[13] = (uint32_t)n_grp;
        e[14] = __float_as_uint(1.0f / (float)n_grp);
        e[15] = 0u;
    }
    __syncthreads();
    // this wave's tiles of the first phase; the first one's stream is requested right away
    // Plans run two phases ahead of the tiles (ct: this phase, nt: the next, nnt: the one after), so that the loads of a
    // plan's directory entries have a whole phase to arrive and nobody waits for them between a barrier and the work.
    PhaseTiles ct, nt, nnt;
    plan_phase<NM24>(ct, ka, plans, 0, n_phases, wave, lane);
    uint2 mk_next = make_uint2(0, 0);
    if (ct.n > 0) issue_phase_tile<NM24>(ct, 0, bufs, mk_next, lane);
    plan_phase<NM24>(nt, ka, plans, 1, n_phases, wave, lane);
    unsigned gen = 0;
    int spin_limit = a.spin_limit;

    for (int p = 0; p < n_phases; ++p) {
        const int layer = p >> 2, kind = p & 3;
        MegaGeo ge;  // this kind's geometry, fetched with scalar loads
        ge.n_out = ka->geo[kind].n_out;
        ge.k_in = ka->geo[kind].k_in;
        ge.n_strips = ka->geo[kind].n_strips;
        ge.n_slabs = ka->geo[kind].n_slabs;
        ge.s_blk = ka->geo[kind].s_blk;
        ge.b_blk = ka->geo[kind].b_blk;
        const int n_grp = max(ka->geo[kind].n_grp, 1);
        unsigned long long* tt = a.trace_time ? a.trace_time + ((size_t)cu * n_phases + p) * 8 : nullptr;
        if (tt && tid == 0) tt[0] = __builtin_amdgcn_s_memrealtime();
        if (p > 0) barrier_arrive(a.bar, gen);

        if (KV && kind == 1) {
            // The attention step over the cache, then a barrier of its own; the first tile of the linear is expanded
            // while that one settles.  The item's first cache rows are requested before q, k and v are complete.
            const bool has_item = cu < a.n_kv * k_tok * a.att_chunks;
            const AttItem it = att_geometry(ka, has_item ? cu : 0);
            u32x4 kw[kAttUnr], vw[kAttUnr];
#pragma unroll
            for (int u = 0; u < kAttUnr; ++u) kw[u] = vw[u] = u32x4{0u, 0u, 0u, 0u};
            if (has_item) attention_loads(ka, layer, it, it.j_lo, tid, kw, vw);
            barrier_wait(a.bar, a.err, (unsigned)ncu, gen, spin_limit);
            if (has_item) {
                attention_item<(KV > 0 ? KV : 1)>(ka, layer, it, reinterpret_cast<float*>(xlds), tid, kw, vw);
                // the scratch was the activation area, whose rows of unused token slots must read as zero
                for (int i = tid; i < kXldsDw; i += kMegaThreads) (mega_lds + kAreaDw)[i] = 0u;
            }
            barrier_arrive(a.bar, gen);
        }

        // Waits for tile j's stream, requests the stream of the tile after it (the next one of this phase, else the
        // first one of the next phase: weights do not depend on activations) and returns what the expansion needs.
        auto stage_tile = [&](int j, uint2& mk, uint32_t (&base)[8], uint32_t& key) -> const uint8_t* {
            wait_vector_memory();  // the tile's stream is in LDS, its masks in registers
            mk = mk_next;
            const uint8_t* bufb = reinterpret_cast<const uint8_t*>(bufs + cb * kTileDw);
            cb ^= 1;
            if (j + 1 < ct.n)
                issue_phase_tile<NM24>(ct, j + 1, bufs + cb * kTileDw, mk_next, lane);
            else if (nt.n > 0)
                issue_phase_tile<NM24>(nt, 0, bufs + cb * kTileDw, mk_next, lane);
            if (!NM24) tile_bases(ct, j, lane, base);
            key = lane_word(ct.key, 8 * j);
            return bufb;
        };

        // While the barrier settles, this wave's first tile of the phase is expanded into its eight MFMA operands.
        Frag fpre[4][2];
        Tile24 tpre;
        const bool have_pre = ct.n > 0;
        uint32_t pre_key = 0;
        if (have_pre) {
            uint2 mk;
            uint32_t base[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            const uint8_t* bufb = stage_tile(0, mk, base, pre_key);
            if (NM24) {
                if (pre_key & kKeyEmpty) {
                    tpre.v[0] = tpre.v[1] = tpre.v[2] = tpre.v[3] = u32x4{0, 0, 0, 0};
                    tpre.idx = make_uint2(0x44444444u, 0x44444444u);
                } else {
                    read_tile24(tpre, bufb, lane);
                }
            } else {
                expand_tile<SD2_MEGA_STEPS>(bufb, lut, base, mk, [&](int q, const Frag& f0, const Frag& f1) {
                    fpre[q][0].q = f0.q;
                    fpre[q][1].q = f1.q;
                });
            }
        }
        if (NM24 || !have_pre) {
#pragma unroll
            for (int q = 0; q < 4; ++q) fpre[q][0].q = fpre[q][1].q = u32x4{0, 0, 0, 0};  // defined in every path
        }
        if (!NM24 || !have_pre) {
            tpre.v[0] = tpre.v[1] = tpre.v[2] = tpre.v[3] = u32x4{0, 0, 0, 0};
            tpre.idx = make_uint2(0u, 0u);
        }
        // The next version of the residual stream starts from zero and receives every slab block's contribution by
        // integer adds; the workgroups of the first slab block add the current version along with theirs.  Their
        // entries of it are requested here, between arrival and release (final since the barrier before last).
        const int slab_block = cu / ka->geo[kind].n_sblk;
        const uint32_t* kpl_s = plans + kind * kPlanDw;
        const int strip_lo_s = uni(kpl_s[2]);
        const bool adds_residual = (kind & 1) && uni(kpl_s[6]) != 0 && slab_block == 0;
        const int* h_seed_src = a.hv + (size_t)(2 * layer + (kind >= 2 ? 1 : 0)) * a.h_stride;
        int hseed[kFlushIters];
#pragma unroll
        for (int j = 0; j < kFlushIters; ++j) {
            hseed[j] = 0;
            const int idx = tid + j * kMegaThreads;
            const int r = idx & 15, sl = (int)(((uint32_t)(idx >> 4) * tok_mul) >> 10), t = (idx >> 4) - sl * k_tok;
            const int strip = strip_lo_s + sl, row = strip * 16 + r;
            if (adds_residual && sl < ge.s_blk && strip < ge.n_strips && row < ge.n_out) hseed[j] = h_seed_src[(size_t)t * ge.n_out + row];
        }

        if (PROBE && tt && tid == 0) tt[4] = __builtin_amdgcn_s_memrealtime();
        plan_phase<NM24>(nnt, ka, plans, p + 2, n_phases, wave, lane);  // its loads travel during the barrier and the prologue
        if (p > 0) barrier_wait(a.bar, a.err, (unsigned)ncu, gen, spin_limit);
        if (tt && tid == 0) tt[1] = __builtin_amdgcn_s_memrealtime();

        // ---------------- prologue: the activation columns of this workgroup's slabs, as bf16 in LDS
        const uint32_t* kpl = plans + kind * kPlanDw;
        const bool active = uni(kpl[6]) != 0;
        const int strip_lo = uni(kpl[2]);
        const int col_lo = uni(kpl[3]) * 256;                                     // first column of the block
        const int n_col = active ? max(0, min(ge.b_blk * 256, ge.k_in - col_lo)) : 0;  // columns that exist
        const int nqkv = a.q_out + 2 * a.kv_out;
        int* yq = a.yqkv + (size_t)layer * a.yqkv_stride;
        int* yg = a.ygu + (size_t)layer * a.ygu_stride;
        const float fix_inv = a.fix_inv;
        // residual versions: 2 layer before the attention output is added, 2 layer + 1 after it, 2 layer + 2 after the MLP
        const int hv_in = 2 * layer + (kind >= 2 ? 1 : 0);  // what this phase's norm reads / what its output is added to
        const int* h_cur = a.hv + (size_t)hv_in * a.h_stride;
        int* h_nxt = a.hv + (size_t)(hv_in + 1) * a.h_stride;
        const size_t tr_x = ((size_t)p * k_tok) * a.trace_kmax, tr_s = ((size_t)p * k_tok) * a.trace_smax;

        // columns past the end of a ragged last slab must read as zero
        if (n_col < ge.b_blk * 256)
            for (int idx = tid; idx < ge.b_blk * kMegaMaxTok * 256; idx += kMegaThreads)
                if ((idx >> 11) * 256 + (idx & 255) >= n_col) xlds[(idx >> 8) * kXRow + (idx & 255)] = 0;

        if (kind == 0 || kind == 2) {
            // Thread i owns columns 4i..4i+3 of every token: all loads of the residual are in flight at once,
            // the squares meet in LDS, and each thread then normalises and rounds the columns it holds.
            const int c4 = 4 * tid;
            i32x4 hraw[kMegaMaxTok];
#pragma unroll
            for (int t = 0; t < kMegaMaxTok; ++t)
                hraw[t] = (t < k_tok && c4 < a.hidden) ? *reinterpret_cast<const i32x4*>(h_cur + (size_t)t * a.hidden + c4) : i32x4{0, 0, 0, 0};
            if (PROBE) {
                    __builtin_amdgcn_s_waitcnt(0);
                    if (tt && tid == 0) tt[5] = __builtin_amdgcn_s_memrealtime();
            }
            {
                // Sums of squares of all token slots at once (unused slots hold zeros), on the fixed-point numbers as they
                // are: the scale is a power of two, so it can be applied to the totals without changing a bit.  Lane 63
                // ends up with the wavefront's totals.
                auto sums_of = [&](auto n_tag) {
                    constexpr int N = decltype(n_tag)::value;
                    float ss[N];
#pragma unroll
                    for (int t = 0; t < N; ++t) {
                        const float f0 = (float)hraw[t][0], f1 = (float)hraw[t][1], f2 = (float)hraw[t][2], f3 = (float)hraw[t][3];
                        ss[t] = f0 * f0 + f1 * f1 + f2 * f2 + f3 * f3;
                    }
                    wave_sums_lane63(ss);
                    if (lane == 63) {
#pragma unroll
                        for (int t = 0; t < N; ++t) part_sums[t * kMegaWaves + wave] = ss[t];  // plain stores: LDS float atomics are slow
                    }
                };
                // the usual draft lengths skip the work of the unused slots (their partial sums stay zero)
                if (k_tok <= 5)
                    sums_of(std::integral_constant<int, 5>{});
                else
                    sums_of(std::integral_constant<int, kMegaMaxTok>{});
            }
            lds_barrier();
            // Every wavefront adds the twelve partial sums itself (lane t: token t, always in the same order), so the
            // scale factors reach its lanes through scalar registers: no second trip through LDS, no second barrier.
            float inv_t[kMegaMaxTok];
            {
                float tot = 0.f;
                if (lane < kMegaMaxTok) {
                    const f32x4* ps = reinterpret_cast<const f32x4*>(part_sums + lane * kMegaWaves);
                    static_assert(kMegaWaves == 12, "three 16-byte reads hold a token's partial sums");
                    const f32x4 p0 = ps[0], p1 = ps[1], p2 = ps[2];
                    tot = ((((((((((p0[0] + p0[1]) + p0[2]) + p0[3]) + p1[0]) + p1[1]) + p1[2]) + p1[3]) + p2[0]) + p2[1]) + p2[2]) + p2[3];
                }
                tot *= fix_inv * fix_inv;
                const float r = 1.0f / sqrtf(tot / (float)a.hidden + 1e-5f);
                // a residual whose norm stays below the limit has every entry below it: the adds into it cannot wrap
                if (wave == 0 && lane < k_tok && !(tot < a.h_limit_sq)) __hip_atomic_fetch_or(a.err, 2u, __ATOMIC_RELAXED, SD2_AGENT);
                const float scaled = r * fix_inv;
#pragma unroll
                for (int t = 0; t < kMegaMaxTok; ++t) inv_t[t] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(scaled), t));
            }
            const int c = c4 - col_lo;
            if (c >= 0 && c < n_col) {
#pragma unroll
                for (int t = 0; t < kMegaMaxTok; ++t)
                    if (t < k_tok) {
                        const float inv = inv_t[t];
                        const uint32_t lo = pack_bf16((float)hraw[t][0] * inv, (float)hraw[t][1] * inv);
                        const uint32_t hi = pack_bf16((float)hraw[t][2] * inv, (float)hraw[t][3] * inv);
                        *reinterpret_cast<uint2*>(xlds + ((c >> 8) * kMegaMaxTok + t) * kXRow + (c & 255)) = make_uint2(lo, hi);
                        if (TRACE) {
                            *reinterpret_cast<f32x4*>(a.trace_src + tr_s + (size_t)t * a.trace_smax + c4) =
                                f32x4{from_fixed(hraw[t][0], fix_inv), from_fixed(hraw[t][1], fix_inv), from_fixed(hraw[t][2], fix_inv),
                                      from_fixed(hraw[t][3], fix_inv)};
                            *reinterpret_cast<uint2*>(a.trace_x + tr_x + (size_t)t * a.trace_kmax + c4) = make_uint2(lo, hi);
                        }
                    }
            }
        } else if (kind == 3) {
            // thread i owns columns 2i, 2i+1 of the block; gate and up of every token are in flight at once
            const int c = 2 * tid;
            if (c < n_col) {
                // loads of every token first, conversions afterwards: a use inside a token's own block would wait there,
                // with the loads of the tokens after it not yet issued
                i32x2 gr[kMegaMaxTok], ur[kMegaMaxTok];
#pragma unroll
                for (int t = 0; t < kMegaMaxTok; ++t) {
                    gr[t] = ur[t] = i32x2{0, 0};  // defined in every path: nothing is carried from the phase before
                    if (t < k_tok) {
                        const int* row = yg + (size_t)t * 2 * a.inter + col_lo + c;
                        gr[t] = *reinterpret_cast<const i32x2*>(row);
                        ur[t] = *reinterpret_cast<const i32x2*>(row + a.inter);
                    }
                }
                f32x2 gv[kMegaMaxTok], uv[kMegaMaxTok];
#pragma unroll
                for (int t = 0; t < kMegaMaxTok; ++t) {
                    gv[t] = f32x2{from_fixed(gr[t][0], fix_inv), from_fixed(gr[t][1], fix_inv)};
                    uv[t] = f32x2{from_fixed(ur[t][0], fix_inv), from_fixed(ur[t][1], fix_inv)};
                }
#pragma unroll
                for (int t = 0; t < kMegaMaxTok; ++t)
                    if (t < k_tok) {
                        // hardware exp2 and reciprocal: about 1e-6 relative, far inside the bf16 rounding that follows
                        const uint32_t pk = pack_bf16(gv[t][0] * __builtin_amdgcn_rcpf(1.0f + __expf(-gv[t][0])) * uv[t][0],
                                                      gv[t][1] * __builtin_amdgcn_rcpf(1.0f + __expf(-gv[t][1])) * uv[t][1]);
                        *reinterpret_cast<uint32_t*>(xlds + ((c >> 8) * kMegaMaxTok + t) * kXRow + (c & 255)) = pk;
                        if (TRACE) {
                            float* ts = a.trace_src + tr_s + (size_t)t * a.trace_smax + col_lo + c;
                            *reinterpret_cast<f32x2*>(ts) = gv[t];
                            *reinterpret_cast<f32x2*>(ts + a.inter) = uv[t];
                            *reinterpret_cast<uint32_t*>(a.trace_x + tr_x + (size_t)t * a.trace_kmax + col_lo + c) = pk;
                        }
                    }
            }
        } else if (KV) {
            // kind == 1 with a cache: the attention step left, per head, token and chunk, a maximum, a sum and 128
            // weighted values; thread (head slot hh, dimension d) combines the chunks of its head
            const int D = 128;
            const int hh = wave >> 1, d = (wave & 1) * 64 + lane;
            const int head = col_lo / D + hh;
            if (hh * D < n_col) {
                const int cc = hh * D + d, C = a.att_chunks;
#pragma unroll
                for (int t = 0; t < kMegaMaxTok; ++t)
                    if (t < k_tok) {
                        const float* pp = a.att_part + (((size_t)layer * k_tok + t) * a.n_heads + head) * C * kMegaAttPartDw;
                        // eight chunks at a time: their loads are in flight together, the running maximum rescales
                        float mx = -3.0e38f, num = 0.f, den = 0.f;
                        for (int c0 = 0; c0 < C; c0 += 8) {
                            float pm[8], pl[8], po[8];
#pragma unroll
                            for (int i = 0; i < 8; ++i) {
                                const float* q = pp + min(c0 + i, C - 1) * kMegaAttPartDw;
                                pm[i] = q[0];
                                pl[i] = q[1];
                                po[i] = q[4 + d];
                            }
                            float gm = mx;
#pragma unroll
                            for (int i = 0; i < 8; ++i)
                                if (c0 + i < C) gm = fmaxf(gm, pm[i]);
                            const float f = __expf(mx - gm);
                            num *= f;
                            den *= f;
                            mx = gm;
#pragma unroll
                            for (int i = 0; i < 8; ++i) {
                                const float wgt = c0 + i < C ? __expf(pm[i] - mx) : 0.f;
                                num += wgt * po[i];
                                den += wgt * pl[i];
                            }
                        }
                        xlds[((cc >> 8) * kMegaMaxTok + t) * kXRow + (cc & 255)] = f32_to_bf16(num * __builtin_amdgcn_rcpf(den));
                    }
            }
        } else {
            // kind == 1: causal attention among the in-flight tokens.  Thread (head slot hh, dimension d) keeps q of
            // its head and k, v of that head's kv group for every token in registers; a score is summed over the
            // 128 dimensions = two wavefronts (cross-lane adds, then one LDS add per wavefront).
            const int D = 128;
            const int hh = wave >> 1, d = (wave & 1) * 64 + lane;  // head slot is wave-uniform: scalar addressing
            const int rep = a.n_heads / a.n_kv;
            const int head = col_lo / D + hh;                 // blocks start on head boundaries (256 | col_lo)
            const int kvh = head / rep;
            const bool live = hh * D < n_col;
            int qr[kMegaMaxTok], kr[kMegaMaxTok], vr[kMegaMaxTok];
#pragma unroll
            for (int t = 0; t < kMegaMaxTok; ++t) {
                qr[t] = kr[t] = vr[t] = 0;
                if (live && t < k_tok) {
                    const int* row = yq + (size_t)t * nqkv;
                    qr[t] = row[head * D + d];
                    kr[t] = row[a.q_out + kvh * D + d];
                    vr[t] = row[a.q_out + a.kv_out + kvh * D + d];
                }
            }
            // the compiler would otherwise move each conversion into its token's block above, where it waits for that
            // token's loads before the next token's are issued: eight trips to memory in a row
#pragma unroll
            for (int t = 0; t < kMegaMaxTok; ++t) asm volatile("" : "+v"(qr[t]), "+v"(kr[t]), "+v"(vr[t]));
            float qv[kMegaMaxTok], kv[kMegaMaxTok], vv[kMegaMaxTok];
#pragma unroll
            for (int t = 0; t < kMegaMaxTok; ++t) {  // after all the loads (see the gated product above)
                qv[t] = from_fixed(qr[t], fix_inv);
                kv[t] = from_fixed(kr[t], fix_inv);
                vv[t] = from_fixed(vr[t], fix_inv);
            }
            // scores of a head: lower triangle [i][j <= i] at i (i + 1) / 2 + j, 36 entries; two shares, one per wavefront
            float* sp = misc + hh * 36;
            float* sp_hi = misc + 216 + hh * 36;
            if (live) {
                // The triangle in batches whose sums cross the lanes together: rows 0..2 (six products), then a row at a
                // time (four to eight products): wide enough to fill the hazard slots, without the unused half of a square.
                float* share = (wave & 1) ? sp_hi : sp;
                {
                    float part[6] = {qv[0] * kv[0], qv[1] * kv[0], qv[1] * kv[1], qv[2] * kv[0], qv[2] * kv[1], qv[2] * kv[2]};
                    wave_sums_lane63(part);  // (rows of unused token slots are zeros: nothing reads them)
                    if (lane == 63) {
#pragma unroll
                        for (int e = 0; e < 6; ++e) share[e] = part[e];  // plain stores, summed below
                    }
                }
#define SD2_SCORE_ROW(I) \
    if (I < k_tok) { \
        float part[I + 1]; \
        _Pragma("unroll") for (int j = 0; j <= I; ++j) part[j] = qv[I] * kv[j]; \
        wave_sums_lane63(part); \
        if (lane == 63) { \
            _Pragma("unroll") for (int j = 0; j <= I; ++j) share[I * (I + 1) / 2 + j] = part[j]; \
        } \
    }
                SD2_SCORE_ROW(3)
                SD2_SCORE_ROW(4)
                SD2_SCORE_ROW(5)
                SD2_SCORE_ROW(6)
                SD2_SCORE_ROW(7)
#undef SD2_SCORE_ROW
                static_assert(kMegaMaxTok == 8, "one row of scores per token slot");
            }
            lds_barrier();
            // softmax: wavefront = head, lane = (row i, column j); a row's maximum and sum go round its eight lanes
            if (wave < kAttHeads && wave * D < n_col) {
                const int i = lane >> 3, j = lane & 7;
                const bool on = i < k_tok && j <= i;
                float* row = misc + wave * 36 + i * (i + 1) / 2;
                const float scale = 1.0f / sqrtf((float)D);
                const float sc = on ? (row[j] + row[216 + j]) * scale : -3.0e38f;
                float mx = sc;
                mx = fmaxf(mx, __shfl_xor(mx, 1));
                mx = fmaxf(mx, __shfl_xor(mx, 2));
                mx = fmaxf(mx, __shfl_xor(mx, 4));
                const float e = on ? __expf(sc - mx) : 0.f;
                float sum = e;
                sum += __shfl_xor(sum, 1);
                sum += __shfl_xor(sum, 2);
                sum += __shfl_xor(sum, 4);
                if (on) row[j] = e * __builtin_amdgcn_rcpf(sum);
            }
            lds_barrier();
            if (live) {
                const int cc = hh * D + d;
#pragma unroll
                for (int t = 0; t < kMegaMaxTok; ++t)
                    if (t < k_tok) {
                        float o = 0.f;
#pragma unroll
                        for (int j = 0; j <= t; ++j) o += sp[t * (t + 1) / 2 + j] * vv[j];
                        const uint16_t cv = f32_to_bf16(o);
                        xlds[((cc >> 8) * kMegaMaxTok + t) * kXRow + (cc & 255)] = cv;
                        if (TRACE) {
                            a.trace_x[tr_x + (size_t)t * a.trace_kmax + col_lo + cc] = cv;
                            float* ts = a.trace_src + tr_s + (size_t)t * a.trace_smax;
                            ts[head * D + d] = qv[t];
                            // heads of one kv group all record the same k and v
                            ts[a.q_out + kvh * D + d] = kv[t];
                            ts[a.q_out + a.kv_out + kvh * D + d] = vv[t];
                        }
                    }
            }
        }
        lds_barrier();
        if (tt && tid == 0) tt[2] = __builtin_amdgcn_s_memrealtime();

        // ---------------- this wave's tiles of the phase
        int cur_slab = -1;
        Frag b[4][2];
#pragma unroll
        for (int q = 0; q < 4; ++q) b[q][0].q = b[q][1].q = u32x4{0, 0, 0, 0};
        auto load_b = [&](int sl) {  // the slab's activation columns as MFMA B operands: lane (n, g) = token n, columns 16g..
            if (sl != cur_slab) {
                cur_slab = sl;
                if (n < kMegaMaxTok) {
                    const u32x4* xr = reinterpret_cast<const u32x4*>(xlds + (sl * kMegaMaxTok + n) * kXRow + 16 * g);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        b[q][0].q = xr[8 * q];
                        b[q][1].q = xr[8 * q + 1];
                    }
                }
            }
        };
        // The sums of a unit (a strip's group of slabs) stay in the accumulators from its first tile to its last;
        // then lane (n, g) stores rows 4g..4g+3 of token n into the unit's own slot: no other wavefront writes there.
        f32x4 acc0 = f32x4{0.f, 0.f, 0.f, 0.f}, acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
        auto unit_done = [&](uint32_t key) {
            if (n < kMegaMaxTok) {
                const int unit = (int)((key >> 16) & 255u);
                *reinterpret_cast<f32x4*>(red + (unit * kMegaMaxTok + n) * 16 + 4 * g) = acc0 + acc1;
            }
        };
        // 2:4: one matrix instruction per 64-column step; the dense operand of a step is the pair (b[q][0], b[q][1])
        auto multiply24 = [&](const Tile24& t) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                Frag16 bq;
                bq.q[0] = b[q][0].q;
                bq.q[1] = b[q][1].q;
                const int ix = (int)(q < 2 ? t.idx.x : t.idx.y);
                if (q & 1)
                    acc1 = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8, t.v[q]), bq.v, acc1, ix, 0, 1);
                else
                    acc0 = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8, t.v[q]), bq.v, acc0, ix, 0, 0);
            }
        };
        if (have_pre) {
            load_b((int)((pre_key >> 8) & 255u));
            if (NM24) {
                multiply24(tpre);
            } else {
                // two accumulators: consecutive MFMAs do not wait for each other's result
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fpre[q][0].v, b[q][0].v, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fpre[q][1].v, b[q][1].v, acc1, 0, 0, 0);
                }
            }
            if (pre_key & kKeyLast) unit_done(pre_key);
        }
        if (PROBE && tt && tid == 0) tt[6] = __builtin_amdgcn_s_memrealtime();
        for (int j = 1; j < ct.n; ++j) {
            uint32_t key;
            uint2 mk;
            uint32_t base[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            const uint8_t* bufb = stage_tile(j, mk, base, key);
            load_b((int)((key >> 8) & 255u));
            if (key & kKeyFirst) acc0 = acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
            if (NM24) {
                if (!(key & kKeyEmpty)) {  // an empty tile adds nothing
                    Tile24 t;
                    read_tile24(t, bufb, lane);
                    multiply24(t);
                }
            } else {
                expand_tile<SD2_MEGA_STEPS>(bufb, lut, base, mk, [&](int q, const Frag& f0, const Frag& f1) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0.v, b[q][0].v, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f1.v, b[q][1].v, acc1, 0, 0, 0);
                });
            }
            if (key & kKeyLast) unit_done(key);
        }
        // a wavefront without tiles in this phase starts the stream of its first tile of the next one here
        if (ct.n == 0 && nt.n > 0) issue_phase_tile<NM24>(nt, 0, bufs + cb * kTileDw, mk_next, lane);
        ct = nt;
        nt = nnt;
        if (PROBE && tt && tid == 0) tt[7] = __builtin_amdgcn_s_memrealtime();
        lds_barrier();
        if (tt && tid == 0) tt[3] = __builtin_amdgcn_s_memrealtime();

        // ---------------- the block's results leave the CU: split-K across the slab blocks by exact fixed-point adds
        if (active) {
            int* ybase = kind == 0 ? yq : (kind == 2 ? yg : h_nxt);
            const float scale = a.fix_scale, lim = ka->fix_limit[kind];
            bool bad = false;
#pragma unroll
            for (int j = 0; j < kFlushIters; ++j) {
                const int idx = tid + j * kMegaThreads;
                if (idx >= ge.s_blk * k_tok * 16) break;
                const int r = idx & 15, sl = (int)(((uint32_t)(idx >> 4) * tok_mul) >> 10), t = (idx >> 4) - sl * k_tok;
                float v = 0.f;
                for (int gq = 0; gq < n_grp; ++gq) {  // the strip's slab groups, each summed by one wavefront
                    float* slot = red + (((sl * n_grp + gq) * kMegaMaxTok + t) << 4) + r;
                    v += *slot;
                    *slot = 0.f;
                }
                const int strip = strip_lo + sl, row = strip * 16 + r;
                if (strip < ge.n_strips && row < ge.n_out) {
                    const float sv = v * scale;
                    bad |= !(fabsf(sv) < lim);  // also true for NaN
                    aadd_i(ybase + (size_t)t * ge.n_out + row, (int)__builtin_rintf(fminf(fmaxf(sv, -lim), lim)) + hseed[j]);
                }
            }
            if (bad) __hip_atomic_fetch_or(a.err, 2u, __ATOMIC_RELAXED, SD2_AGENT);  // the call's results are invalid
        }
    }
    // ---------------- the last version of the residual stream as fp32
    if (n_phases > 0) {
        barrier_arrive(a.bar, gen);
        barrier_wait(a.bar, a.err, (unsigned)ncu, gen, spin_limit);
    }
    {
        const int* h_last = a.hv + (size_t)(2 * a.layers) * a.h_stride;
        const int n_h = k_tok * a.hidden;
        const float fix_inv = a.fix_inv;
        for (int idx = cu * kMegaThreads + tid; idx < n_h; idx += ncu * kMegaThreads) a.h_out[idx] = from_fixed(h_last[idx], fix_inv);
    }
}

// ---------------------------------------------------------------- set-up kernels and launch

// One set-up launch: the barrier words, the accumulators and every residual version but the first start from zero;
// the first version is the bf16 input in fixed point.
__global__ __launch_bounds__(256) void mega_setup_kernel(uint32_t* __restrict__ zero, size_t n_zero, int* __restrict__ h,
                                                        const uint16_t* __restrict__ h_in, size_t n_h, size_t n_h_rest, float scale) {
    const size_t i0 = (size_t)blockIdx.x * 256 + threadIdx.x, step = (size_t)gridDim.x * 256;
    for (size_t i = i0; i < n_zero; i += step) zero[i] = 0u;
    // out-of-range inputs saturate here; the first norm's range check then reports them
    for (size_t i = i0; i < n_h; i += step) h[i] = (int)__builtin_rintf(fminf(fmaxf(bf16_to_f32(h_in[i]) * scale, -1073741824.f), 1073741824.f));
    for (size_t i = n_h + i0; i < n_h + n_h_rest; i += step) h[i] = 0;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

MegaLayout mega_layout(int layers, int hidden, int q_out, int kv_out, int inter, int k_tok) {
    MegaLayout L;
    const size_t nl = (size_t)(layers > 0 ? layers : 1);
    L.h_stride = align256((size_t)k_tok * hidden * 4) / 4;
    L.yqkv_stride = align256((size_t)k_tok * (q_out + 2 * kv_out) * 4) / 4;
    L.ygu_stride = align256((size_t)k_tok * 2 * inter * 4) / 4;
    size_t off = 0;
    L.bar_off = off;
    off += align256((size_t)kBarWords * 4);
    L.err_off = off;
    off += 256;
    L.yqkv_off = off;
    off += nl * L.yqkv_stride * 4;
    L.ygu_off = off;
    off += nl * L.ygu_stride * 4;
    L.hv_off = off;
    off += (2 * nl + 1) * L.h_stride * 4;
    L.total = off;
    return L;
}

// The kernel with the attention step over a cache, compiled per number of query heads per key/value head (its
// register arrays have that size, and one variant per kernel keeps the code within the instruction cache).
static const void* mega_kv_kernel(bool nm24, int rep) {
#define SD2_KV_CASE(R) \
    case R: \
        return nm24 ? reinterpret_cast<const void*>(mega_forward_kernel<false, false, true, R>) \
                    : reinterpret_cast<const void*>(mega_forward_kernel<false, false, false, R>)
    switch (rep) {
        SD2_KV_CASE(1);
        SD2_KV_CASE(2);
        SD2_KV_CASE(3);
        SD2_KV_CASE(4);
    }
#undef SD2_KV_CASE
    return nullptr;
}

// Prepares one kernel for launches with the full LDS and checks that a workgroup of it fits a compute unit.
static bool mega_kernel_fits(const void* fn) {
    int per_cu = 0;
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMegaLds) == hipSuccess &&
           hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kMegaThreads, kMegaLds) == hipSuccess && per_cu >= 1;
}

static int mega_probe_device() {
    int dev = 0, n = 0, coop = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
        return 0;
    const void* plain[] = {reinterpret_cast<const void*>(mega_forward_kernel<false, false, false>),
                           reinterpret_cast<const void*>(mega_forward_kernel<true, false, false>),
                           reinterpret_cast<const void*>(mega_forward_kernel<false, true, false>),
                           reinterpret_cast<const void*>(mega_forward_kernel<false, false, true>),
                           reinterpret_cast<const void*>(mega_forward_kernel<true, false, true>)};
    for (const void* fn : plain)
        if (!mega_kernel_fits(fn)) return 0;
    for (int nm24 = 0; nm24 < 2; ++nm24)
        for (int rep = 1; rep <= 4; ++rep)
            if (!mega_kernel_fits(mega_kv_kernel(nm24 != 0, rep))) return 0;
    return n;
}

// Workgroups of the persistent kernel (one per compute unit), 0 when it cannot run on this device.  Probed once;
// threads that race here compute the same value.
static int mega_grid() {
    static std::atomic<int> cached{-1};
    int cus = cached.load(std::memory_order_acquire);
    if (cus < 0) {
        cus = mega_probe_device();
        cached.store(cus, std::memory_order_release);
    }
    return cus;
}

int mega_grid_size() { return mega_grid(); }

// Block of s strips x b slabs per workgroup, the b slabs of a strip cut into groups of grp_slabs (a group is summed
// in registers by one wavefront): fewest tiles for the busiest wavefront, then fewest tiles per workgroup, then the
// widest block (fewer slab blocks mean fewer float atomics leaving the CU), then the fewest groups.
static bool plan_kind(MegaGeo& g, int ncu, int max_b) {
    long best_wave = -1, best_cost = -1;
    for (int b = 1; b <= max_b && b <= g.n_slabs; ++b) {
        const int n_bblk = (g.n_slabs + b - 1) / b;
        const int max_sblk = ncu / n_bblk;
        if (max_sblk < 1) continue;
        const int s = (g.n_strips + max_sblk - 1) / max_sblk;
        if (s > kMaxS) continue;
        for (int grp_slabs = b; grp_slabs >= 1; --grp_slabs) {
            const int n_grp = (b + grp_slabs - 1) / grp_slabs;
            if (s * n_grp > kMaxUnits) continue;
            const long wave_tiles = (long)((s * n_grp + kMegaWaves - 1) / kMegaWaves) * grp_slabs;
            if (wave_tiles > kMaxTilesPerWave) continue;
            const long cost = (long)s * b;
            const bool better = best_wave < 0 || wave_tiles < best_wave || (wave_tiles == best_wave && cost < best_cost) ||
                                (wave_tiles == best_wave && cost == best_cost && b > g.b_blk);
            if (better) {
                best_wave = wave_tiles;
                best_cost = cost;
                g.s_blk = s;
                g.b_blk = b;
                g.n_sblk = (g.n_strips + s - 1) / s;
                g.n_bblk = n_bblk;
                g.n_grp = n_grp;
                g.grp_slabs = grp_slabs;
            }
        }
    }
    return best_wave > 0;
}

bool mega_plan(MegaGeo (&geo)[4], int layers, int hidden, int head_dim, int k_tok, int max_tile_nnz, bool nm24) {
    if (layers < 1 || layers > kMegaMaxLayers || head_dim != 128 || k_tok < 1 || k_tok > kMegaMaxTok) return false;
    // a tile's stream must fit a 5 KiB buffer (a 2:4 tile always takes 4608 bytes)
    if (hidden > kMegaMaxHidden || (!nm24 && max_tile_nnz * 2 + 8 > kMegaCh * 1024)) return false;
    const int ncu = mega_grid();
    if (ncu < 1) return false;
    for (int k = 0; k < 4; ++k)
        if (!plan_kind(geo[k], ncu, k == 1 ? kMaxBAtt : kMaxB)) return false;
    return true;
}

int mega_attention_chunks(int n_heads, int n_kv, int k_tok) {
    const int ncu = mega_grid();
    if (ncu < 1 || n_kv < 1 || k_tok < 1 || n_heads % n_kv || n_heads / n_kv > 4) return 0;
    return std::max(0, std::min(kMegaMaxChunks, ncu / (n_kv * k_tok)));
}

hipError_t launch_mega_forward(const MegaArgs& a, const uint16_t* h_in, void* zero_base, size_t zero_bytes, bool probe,
                               bool nm24, hipStream_t s) {
    const int ncu = mega_grid();
    if (ncu < 1) return hipErrorNotSupported;
    const size_t nh = (size_t)a.k_tok * a.hidden;
    const size_t n_rest = (size_t)(2 * a.layers + 1) * a.h_stride - nh;  // the padding of the first version and all later ones
    hipLaunchKernelGGL(mega_setup_kernel, dim3(512), dim3(256), 0, s, static_cast<uint32_t*>(zero_base), zero_bytes / 4, a.hv,
                       h_in, nh, n_rest, a.fix_scale);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    MegaArgs args = a;
    void* params[] = {&args};
    const void* fn;
    if (a.k_cache) {
        if (a.trace_x || a.trace_time || probe || a.att_chunks < 1 || a.att_chunks > kMegaMaxChunks ||
            a.n_kv * a.k_tok * a.att_chunks > ncu || a.n_heads > 4 * a.n_kv || !a.v_cache || !a.rope || !a.att_part)
            return hipErrorInvalidValue;
        fn = mega_kv_kernel(nm24, a.n_heads / a.n_kv);
        if (!fn) return hipErrorInvalidValue;
    } else if (nm24)
        fn = a.trace_x ? reinterpret_cast<const void*>(mega_forward_kernel<true, false, true>)
                       : reinterpret_cast<const void*>(mega_forward_kernel<false, false, true>);
    else
        fn = a.trace_x ? reinterpret_cast<const void*>(mega_forward_kernel<true, false, false>)
             : probe   ? reinterpret_cast<const void*>(mega_forward_kernel<false, true, false>)
                       : reinterpret_cast<const void*>(mega_forward_kernel<false, false, false>);
    return hipLaunchCooperativeKernel(fn, dim3((unsigned)ncu), dim3(kMegaThreads), params, kMegaLds, s);
}

}  // namespace sd2
