// Launch interface between the C ABI layer and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sd2 {

// One matrix as the kernels see it.  Sparse: dir/masks/vals point into the device blob.
// Dense: w points at the row-major bf16 matrix.  The tile geometry is common to both.
struct MatArgs {
    const void* dir;       // 48-byte directory entries                      (sparse)
    const uint2* masks;    // 4 x uint16 per lane and tile                    (sparse)
    const uint16_t* vals;  // compacted bf16 values                           (sparse)
    const uint16_t* w;     // [n_out][k_in] bf16                              (dense)
    int n_out, k_in;
    int n_strips, n_slabs, n_tiles;
    int max_tile_nnz;
};

// Where a linear reads its activations from and where the partial sums go.
struct LinArgs {
    const uint16_t* x;  // [k_tok][k_in] bf16
    int k_tok;
    float* out;         // n_slabs == 1: y [k_tok][n_out]; else partials [n_slabs][k_tok][n_out]
};

hipError_t launch_sparse_linear(const MatArgs& m, const LinArgs& a, hipStream_t s);
hipError_t launch_dense_linear(const MatArgs& m, const LinArgs& a, hipStream_t s);
// the sparse linear with final results in one launch (no partial sums): a.out is y [k_tok][n_out]
bool sparse_strip_supported(const MatArgs& m, int k_tok);
// the per-slab kernel with the multiply on the vector ALU (up to 8 tokens): a measurement variant
bool sparse_linear_valu_supported(const MatArgs& m, int k_tok);
hipError_t launch_sparse_linear_valu(const MatArgs& m, const LinArgs& a, hipStream_t s);
hipError_t launch_sparse_strip_linear(const MatArgs& m, const LinArgs& a, hipStream_t s);
// the fused [gate; up] product with the gating in its epilogue: m_out [k_tok][n_out / 2] = bf16(silu(gate x) * (up x))
bool sparse_strip_gated_supported(const MatArgs& m, int k_tok);
hipError_t launch_sparse_strip_gated(const MatArgs& m, const uint16_t* x, int k_tok, uint16_t* m_out, hipStream_t s);

// Device address, on the current device, of the library's static scratch array (kStaticScratchBytes bytes, 256-byte
// aligned): looked up once per device, no allocation.  Calls that use it on one GPU share it.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
hipError_t static_scratch(void** ptr_out);

// y[i] = sum_s part[s][i], i < n  (n = k_tok * n_out)
hipError_t launch_reduce_partials(const float* part, int n_splits, size_t n, float* y, hipStream_t s);

// y[i] = sum_s part[s * split_stride + i], i < n
hipError_t launch_reduce_partials_strided(const float* part, int n_splits, size_t split_stride, size_t n, float* y,
                                          hipStream_t s);

// h (fp32 [k_tok][hidden]) is initialised from bf16 h_in (when given) or updated in place with
// h += sum_s part[s]; then a = bf16(h / sqrt(mean(h^2) + 1e-5)) is written when a != nullptr.
// ssq: scratch of k_tok * ceil(hidden / 256) floats (per-block sums of squares).
hipError_t launch_residual_rmsnorm(float* h, const uint16_t* h_in, const float* part, int n_splits,
                                   int k_tok, int hidden, uint16_t* a, float* ssq, hipStream_t s);

// Causal softmax attention among the k_tok <= 64 in-flight tokens (head_dim a multiple of 8, <= 256); qkv partials
// [n_splits][k_tok][q_out+2*kv_out].
hipError_t launch_inflight_attention(const float* part, int n_splits, int k_tok, int q_out, int kv_out,
                                     int n_heads, int n_kv, int head_dim, uint16_t* ctx, hipStream_t s);

// m[t][j] = bf16( silu(g) * u ), g = sum_s part[s][t][j], u = sum_s part[s][t][inter + j]
hipError_t launch_silu_mul(const float* part, int n_splits, int k_tok, int inter, uint16_t* m, hipStream_t s);

hipError_t launch_greedy_verify(const int32_t* draft, const int32_t* target, int batch, int k,
                                int32_t* accepted, int32_t* out_tokens, hipStream_t s);

// decode step with rotary embedding and a key/value cache (bf16 [n_kv][max_pos][head_dim] per layer): the angle table
// [k_tok][head_dim / 2] of the call's positions; q rotated into q_rot (fp32 [k_tok][q_out]), rotated keys and values
// appended at positions pos0 .. pos0 + k_tok - 1; attention of token t over positions 0 .. pos0 + t into ctx (bf16)
hipError_t launch_rope_table(int pos0, int k_tok, int head_dim, double theta, float2* table, hipStream_t s);
hipError_t launch_rope_append(const float* part, int n_splits, int k_tok, int q_out, int kv_out, int n_heads, int n_kv,
                              int head_dim, const float2* table, int pos0, int max_pos, float* q_rot, uint16_t* k_cache,
                              uint16_t* v_cache, hipStream_t s);
bool cached_attention_supported(int n_heads, int n_kv, int head_dim, int max_pos);
hipError_t launch_cached_attention(const float* q_rot, const uint16_t* k_cache, const uint16_t* v_cache, int max_pos, int pos0,
                                   int k_tok, int q_out, int n_heads, int n_kv, int head_dim, uint16_t* ctx, hipStream_t s);

// drafting round helpers: rows of the embedding for the window [*start, drafts[0..n_tok-1)); *acc |= *flag
hipError_t launch_embed_window(const uint16_t* emb, int vocab, int hidden, const int32_t* start, const int32_t* drafts,
                               int n_tok, uint16_t* h_in, hipStream_t s);
hipError_t launch_fold_flag(const unsigned* flag, unsigned* acc, hipStream_t s);

// one-shot magnitude pruning in place (bf16 [n_out][k_in]): rows keeps n_keep per row (k_in a multiple of 256, <= 9216)
hipError_t launch_prune_rows(uint16_t* w, int n_out, int k_in, int n_keep, hipStream_t s);
hipError_t launch_prune_2of4(uint16_t* w, int n_out, int k_in, hipStream_t s);

// g <- g where the blob's mask bit is set, +0 elsewhere; grad is [n_out][k_in] fp32 or bf16 (bitmask format only)
hipError_t launch_mask_gradient(const MatArgs& m, void* grad, bool bf16, hipStream_t s);

// dst[0..bytes) = src[0..bytes), bytes a multiple of 16 (traffic calibration for profiler counters)
hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
// pure read of src[0..bytes): one checksum word per workgroup goes to sink[0..2048)
hipError_t launch_calibration_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s);

}  // namespace sd2

namespace sd2 {

// ---- whole-forward persistent kernel ("mega" path): one cooperative launch per forward.
constexpr int kMegaMaxLayers = 64;
constexpr int kMegaMaxTok = 8;
constexpr int kMegaMaxHidden = 3072;

// One kind of matrix (qkv, o, gate_up, down).  Workgroup c < n_sblk * n_bblk owns the block of
// s_blk strips x b_blk slabs with strip block c % n_sblk and slab block c / n_sblk.
struct MegaGeo {
    int n_out, k_in, n_strips, n_slabs, n_tiles;
    int s_blk, b_blk, n_sblk, n_bblk;
    int n_grp, grp_slabs;  // a strip's b_blk slabs are cut into n_grp groups of grp_slabs; one wavefront sums a group in registers
    int pad;
    unsigned long long mask_off, val_off;  // byte offsets inside a blob (equal for all layers of a kind)
};

struct MegaArgs {
    MegaGeo geo[4];  // qkv, o, gate_up, down
    int layers, hidden, q_out, kv_out, inter, n_heads, n_kv, head_dim, k_tok, spin_limit;
    // Every activation buffer is written (by agent-scope stores and integer atomics, which go through to memory) and
    // afterwards read at addresses no CU has touched before in this launch: one copy per layer, so a barrier needs no
    // cache invalidation.  The buffers hold 32-bit fixed point (17 fraction bits): contributions of several workgroups
    // are added by integer atomics, which are exact, so the sums do not depend on the order of arrival.
    int* hv;              // [2 layers + 1][k_tok][hidden] residual versions (stride h_stride values)
    float* h_out;         // [k_tok][hidden]: the last version as fp32
    int* yqkv;            // [layers][k_tok][q_out + 2 kv_out] accumulators (stride yqkv_stride values)
    int* ygu;             // [layers][k_tok][2 inter] (stride ygu_stride values)
    unsigned long long h_stride, yqkv_stride, ygu_stride;
    float fix_scale, fix_inv;  // 2^F and 2^-F
    float fix_limit[4];        // per kind: what one workgroup's contribution must stay below, 2^30 / slab blocks
    float h_limit_sq;          // (2^30 / 2^F)^2: a token's squared residual norm must stay below it
    unsigned* bar;        // grid barrier state (see mega kernel)
    unsigned* err;        // bit 0: a bounded wait ran out; bit 1: a fixed-point sum left the checked range
    uint16_t* trace_x;    // optional [phase][k_tok][trace_kmax] bf16: the activations each linear consumed
    float* trace_src;     // optional [phase][k_tok][trace_smax] fp32: the values its input glue read
    int trace_kmax, trace_smax;
    unsigned long long* trace_time;  // optional [workgroup][phase][8] 100 MHz clock: start, barrier, prologue, tiles (timestamps);
                                     // wavefront 0's ticks spent waiting for streams, ticks decoding, tiles; spare
    // Decode with a key/value cache (k_cache == nullptr: attention among the call's tokens only).  After the q|k|v
    // linear, att_chunks workgroups per (key/value head, token) each attend to one stretch of the positions and
    // leave a partial softmax result; the linear that follows combines them.
    uint16_t* k_cache;    // [layers][n_kv][max_pos][128] bf16, rotated keys
    uint16_t* v_cache;    // the same shape, values
    const float2* rope;   // [k_tok][64] cos and sin of the call's positions
    float* att_part;      // [layers][k_tok][n_heads][att_chunks][kMegaAttPartDw]: running maximum, sum, 2 spare, 128 sums
    int max_pos, pos0, att_chunks, pad2;
    const unsigned char* blob[4 * kMegaMaxLayers];
};
constexpr int kMegaAttPartDw = 132;
constexpr int kMegaMaxChunks = 32;

struct MegaLayout {
    size_t bar_off, err_off, yqkv_off, ygu_off, hv_off, total;  // [0, hv_off) starts as zero
    size_t h_stride, yqkv_stride, ygu_stride;                    // in values of four bytes
};

MegaLayout mega_layout(int layers, int hidden, int q_out, int kv_out, int inter, int k_tok);
// workgroups of the persistent kernel on the current device (0 when it cannot run here)
int mega_grid_size();
// Chooses the workgroup tiling of each matrix kind; false when the persistent kernel cannot run this model here.
bool mega_plan(MegaGeo (&geo)[4], int layers, int hidden, int head_dim, int k_tok, int max_tile_nnz, bool nm24);
// probe: timestamps only, plus wavefront 0's wait/decode split (needs a.trace_time, a.trace_x == nullptr)
hipError_t launch_mega_forward(const MegaArgs& a, const uint16_t* h_in, void* zero_base, size_t zero_bytes, bool probe, bool nm24,
                               hipStream_t s);
// Workgroups per (key/value head, token) of the cached attention step, 0 when the persistent kernel cannot serve it.
int mega_attention_chunks(int n_heads, int n_kv, int k_tok);

// ---- 2:4 semi-structured linear (blob format 3): final y for tokens [0, k_tok), k_tok <= 16; m.dir = first tile
bool nm24_supported(int n_slabs);
hipError_t launch_nm24_linear(const MatArgs& m, const LinArgs& a, hipStream_t s);

// ---- LM head with greedy choice: tokens [0, k_tok), k_tok <= 16, hidden a multiple of 128 and <= 9216.
// part_ws: kLmMaxWorkgroups * 16 candidates of 8 bytes.  max_logit and logits ([k_tok][vocab]) may be null.
constexpr int kLmMaxWorkgroups = 1024;
constexpr int kLmMaxHidden = 9216;
hipError_t launch_lm_head(const uint16_t* w, const float* h, int vocab, int hidden, int k_tok, void* part_ws,
                          int32_t* token_ids, float* max_logit, float* logits, hipStream_t s);

// the same streaming kernel as a plain dense linear (final y, tokens [0, k_tok), k_tok <= 16; k_in % 128 == 0, <= 9216)
hipError_t launch_dense_stream_linear(const uint16_t* w, const uint16_t* x, int n_out, int k_in, int k_tok, float* y,
                                      hipStream_t s);
inline bool dense_stream_ok(int k_in) { return k_in % 128 == 0 && k_in <= kLmMaxHidden; }
// up to 4096 columns the kernel takes 32 tokens per pass
inline bool dense_stream_pair_ok(int k_in) { return dense_stream_ok(k_in) && k_in <= 4096; }

}  // namespace sd2
