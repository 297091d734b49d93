/*
 * sd2.h -- C ABI of libsd2: the hot path of a pruned ("sparse") draft model for
 * speculative decoding on one AMD MI355X (gfx950).
 *
 * What the calls compute follows the paper's problem statement:
 *   - the draft model M_d is a decoder whose linear layers (q, k, v, o, gate, up,
 *     down) carry a fixed binary weight mask; pruned weights are exactly zero
 *     (Sec. 2.3 "Fine-grained pruning", Sec. 2.4 "Sparse fine-tuning");
 *   - per round M_d proposes k tokens and the target keeps the longest prefix that
 *     equals its own greedy choices, then adds one token of its own
 *     (Sec. 2.1, Eq. 1 and Eq. 2; footnote to Eq. 3);
 *   - the cost of M_d per token is what Eq. 3 calls c; it is set by the bytes the
 *     pruned linears stream, which is what the packed format minimises (Sec. 3.3
 *     asks for "efficient sparse representations and kernels").
 *
 * Conventions
 *   - Every function returns SD2_OK (0) or a negative sd2_status; nothing throws or
 *     aborts.  All argument and blob checks happen on the host before any launch.
 *   - "host" pointers are ordinary CPU memory.  "device" pointers are HIP device
 *     memory owned by the caller (for example torch tensors); the library never
 *     allocates or frees device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Device
 *     calls only enqueue work on that stream and return.
 *   - bf16 values travel as uint16_t bit patterns.  Activations are token-major:
 *     X is [k_tok][k_in], Y is [k_tok][n_out]; weights are row-major [n_out][k_in]
 *     (the layout of nn.Linear.weight).  Outputs are fp32 (fp32 accumulation of
 *     exact bf16 x bf16 products).
 *   - Limits: 1 <= k_tok <= 64; k_in a multiple of 64; device pointers 16-byte aligned.
 */
#ifndef SD2_H
#define SD2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum sd2_status {
    SD2_OK = 0,
    SD2_ERR_NULL = -1,        /* a required pointer is NULL */
    SD2_ERR_SHAPE = -2,       /* a dimension is out of range or inconsistent */
    SD2_ERR_FORMAT = -3,      /* unknown / unsupported format id or geometry */
    SD2_ERR_BUFFER = -4,      /* a caller buffer is too small or misaligned */
    SD2_ERR_BLOB = -5,        /* blob header, directory or checksum is corrupt */
    SD2_ERR_RANGE = -6,       /* a value (token id, k_tok, ...) is outside its range */
    SD2_ERR_HIP = -7,         /* a HIP runtime call or kernel launch failed */
    SD2_ERR_UNSUPPORTED = -8, /* valid request that this build does not implement */
    SD2_ERR_TIMEOUT = -9      /* a bounded wait inside a kernel ran out; the results of that call are invalid */
};

#define SD2_MAX_TOKENS 64
#define SD2_FORMAT_AUTO 0
#define SD2_FORMAT_BITMASK 1
/* Reserved, returns SD2_ERR_UNSUPPORTED: a tile of uint16 column indices costs 4 bytes per stored weight whatever the
 * sparsity, against 2 + 1/(8 density) for the bitmask (2.25 at 50 %, 2.5 at 75 %); at 50 % it moves exactly the bytes
 * of the dense matrix and only wins beyond 93.75 % sparsity, outside the range the paper prunes to (Sec. 3: 50-75 %). */
#define SD2_FORMAT_INDEX16 2
#define SD2_FORMAT_NM24 3    /* 2:4 semi-structured: at most two non-zeros in every aligned group of four columns */

/* Static, never freed. */
const char* sd2_strerror(int status);
int sd2_version(void);

/* Process-wide switches for tests and profiling.  Their start values come from the environment, read once when a
 * call first needs one (SD2_FORWARD=multi, SD2_LINEAR=partials, SD2_MEGA_SPIN_LIMIT=<n>, SD2_MEGA_TIMING=1|2); no
 * device call reads the environment afterwards.
 *   SD2_OPT_FORWARD_MULTI    1: the stack runs as one launch per linear and glue step even where the single-launch
 *                               kernel could serve it
 *   SD2_OPT_LINEAR_PARTIALS  1: sparse linears keep one partial result per slab and add them in a second launch even
 *                               where the kernel that writes final results could serve them; 2: as 1, and for up to 8
 *                               tokens that kernel multiplies on the vector ALU (packed bf16 dot products) instead of
 *                               the matrix cores: a measurement variant, same results within the same bound
 *   SD2_OPT_SPIN_LIMIT       polls a bounded wait of the single-launch kernel may spend; -1: the default (2^20)
 *   SD2_OPT_MEGA_TIMING      1 / 2: the trace variant of the forward records timestamps only (2: also wavefront 0's
 *                               split into waiting and decoding)
 *   SD2_OPT_FIXED_BITS       fraction bits F (8..22, default 17) of the fixed-point sums of the single-launch kernel:
 *                               resolution 2^-F, range +-2^(31-F); see sd2_sparse_drafter_forward
 * SD2_ERR_RANGE for an unknown switch or a value outside its range. */
#define SD2_OPT_FORWARD_MULTI 0
#define SD2_OPT_LINEAR_PARTIALS 1
#define SD2_OPT_SPIN_LIMIT 2
#define SD2_OPT_MEGA_TIMING 3
#define SD2_OPT_FIXED_BITS 4
#define SD2_OPT_COUNT 5
int sd2_set_option(int32_t which, int32_t value);
int sd2_get_option(int32_t which, int32_t* value_out);

/* ------------------------------------------------------------------ packing (host only)
 * The sparse representation: Sec. 1 and Sec. 3.3 require one but do not define it.
 * The byte layout is specified in docs/FORMAT.md (tiles of 16 rows x 256 columns,
 * one 16-bit mask per lane and 64-column step, compacted bf16 values in the order
 * a wavefront consumes them, a per-tile directory with the offsets of its 16 runs).
 * SD2_FORMAT_NM24 is the 2:4 pattern the paper evaluates next to unstructured sparsity
 * (Sec. 3, Sec. 3.3): two bf16 values and two 2-bit column indices per group of four weights,
 * 1.125 bytes per dense weight, laid out as the operands of the structured-sparse matrix
 * instruction.  It must be asked for explicitly (SD2_FORMAT_AUTO never chooses it), and packing
 * a matrix that is not 2:4 returns SD2_ERR_FORMAT. */

typedef struct sd2_blob_info {
    int32_t format, n_out, k_in;
    int32_t n_strips, n_slabs, n_tiles; /* tiles of 16 rows x 256 columns; n_slabs = split-K factor */
    int32_t max_tile_nnz;
    int32_t reserved0;
    uint64_t nnz;          /* non-zero weights */
    uint64_t total_bytes;  /* size of the blob */
    uint64_t useful_bytes; /* bitmask: 2*nnz + n_out*k_in/8 (values plus one mask bit per position); 2:4: 9*n_out*k_in/8 */
    uint64_t mask_off, val_off;
    uint32_t checksum;
    uint32_t reserved;
} sd2_blob_info_t;

/* Bytes needed for the blob of `w_bf16` (host, [n_out][k_in], zeros = pruned; both +0
 * and -0 count as pruned).  format: SD2_FORMAT_AUTO or SD2_FORMAT_BITMASK. */
int sd2_pack_sparse_size(const uint16_t* w_bf16, int32_t n_out, int32_t k_in, int32_t format,
                         size_t* bytes_out);

/* Writes the blob into caller-owned host memory `blob` of `blob_bytes` bytes.
 * SD2_ERR_BUFFER if it does not fit.  Deterministic: equal inputs give equal bytes. */
int sd2_pack_sparse(const uint16_t* w_bf16, int32_t n_out, int32_t k_in, int32_t format, void* blob,
                    size_t blob_bytes, size_t* bytes_written);

/* Inverse of sd2_pack_sparse: fills w_bf16_out (host, [n_out][k_in]) with the stored
 * values and +0 elsewhere.  n_out/k_in must match the blob.  Validates the blob first. */
int sd2_unpack_sparse(const void* blob, size_t blob_bytes, uint16_t* w_bf16_out, int32_t n_out,
                      int32_t k_in);

/* Parses and checks the header (magic, version, geometry, offsets vs blob_bytes). */
int sd2_blob_info(const void* blob, size_t blob_bytes, sd2_blob_info_t* out);

/* Full check of a host blob: header, checksum, directory vs masks, and that no mask bit of a
 * ragged last strip or slab lies outside the matrix. */
int sd2_blob_validate(const void* blob, size_t blob_bytes);

/* ------------------------------------------------------------------ matrices on the device */

#define SD2_KIND_SPARSE 1
#define SD2_KIND_DENSE 2

/* Plain descriptor, owned by the caller, no hidden state.  `data_dev` is the device copy
 * of the blob (sparse) or of the row-major bf16 matrix (dense). */
typedef struct sd2_matrix {
    int32_t kind;
    int32_t reserved;
    const void* data_dev;
    sd2_blob_info_t info; /* dense: only the shape and tile counts are used */
} sd2_matrix_t;

/* Sparse descriptor from the host copy of the blob and the device address the same bytes were
 * uploaded to.  Only the header is parsed and checked here; the kernels trust the directory
 * (offsets and counts of a tile's values drive their reads), so a blob that does not come
 * straight from sd2_pack_sparse should go through sd2_blob_validate first. */
int sd2_matrix_init_sparse(sd2_matrix_t* m, const void* blob_host, size_t blob_bytes,
                           const void* blob_dev);
/* Dense descriptor for the baseline kernel: W is the same masked matrix stored with
 * its zeros, 2 bytes per weight. */
int sd2_matrix_init_dense(sd2_matrix_t* m, const uint16_t* w_bf16_dev, int32_t n_out, int32_t k_in);

/* ------------------------------------------------------------------ linears
 * Y[t][n] = sum_c W[n][c] * X[t][c] over the stored (non-pruned) weights, fp32
 * accumulate -- one pruned decoder linear applied to k_tok in-flight tokens
 * (Sec. 2.1: the drafter runs on the draft tokens; Sec. 2.4: pruned weights are zero).
 * When k_in spans more than one 256-column slab, per-slab partial sums go through
 * `workspace` (device, >= the size reported below, 16-byte aligned) and are added up in
 * a fixed order; otherwise it may be NULL. */
int sd2_linear_workspace_size(const sd2_matrix_t* m, int32_t k_tok, size_t* bytes_out);
int sd2_sparse_linear(const sd2_matrix_t* m, const uint16_t* x_bf16_dev, int32_t k_tok, float* y_dev,
                      void* workspace_dev, size_t workspace_bytes, void* stream);
/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture, serving loops
 * with a fixed memory plan, harnesses that forbid allocation): sd2_sparse_linear with the per-slab partial sums kept
 * in a static device array of the library (sd2_static_scratch_bytes: 8 MiB, held by every GPU the library has run
 * on until the process ends) instead of a caller workspace.  The call allocates and frees nothing.  A product whose
 * partial sums (sd2_linear_workspace_size) exceed the array returns SD2_ERR_BUFFER before anything is enqueued.
 * All calls on one GPU share the array: calls that may overlap in time (different streams) race on it; calls on
 * one stream are ordered and safe.  Nothing in the array has to be cleared between calls: a call overwrites every
 * partial sum it reads.  Results are identical to sd2_sparse_linear's. */
int sd2_static_scratch_bytes(size_t* bytes_out);
int sd2_sparse_linear_static(const sd2_matrix_t* m, const uint16_t* x_bf16_dev, int32_t k_tok, float* y_dev, void* stream);
/* The same product without the final add: writes the n_slabs per-slab partial results
 * [n_slabs][k_tok][n_out] (fp32) to `partials_dev` (>= n_slabs*k_tok*n_out*4 bytes).  This is
 * what the stack's glue kernels consume; with n_slabs == 1 it equals sd2_sparse_linear.  A 2:4
 * matrix (SD2_FORMAT_NM24) has no per-slab results: its kernel adds the slabs up inside the
 * workgroup, and this call then writes one final result [k_tok][n_out]. */
int sd2_sparse_linear_partials(const sd2_matrix_t* m, const uint16_t* x_bf16_dev, int32_t k_tok,
                               float* partials_dev, size_t partials_bytes, void* stream);
/* Hand-written dense bf16 baseline for the same shapes; `m` must be a dense descriptor.  For k_in a multiple of
 * 128 up to 9216 it streams the matrix like the LM head does and needs no workspace. */
int sd2_dense_linear(const sd2_matrix_t* m, const uint16_t* x_bf16_dev, int32_t k_tok, float* y_dev,
                     void* workspace_dev, size_t workspace_bytes, void* stream);

/* Gated MLP block: y = Wd * bf16( silu(Wg x) * (Wu x) ), with [Wg; Wu] packed as one
 * matrix of 2*inter rows (they share their input) and Wd as a second one. */
int sd2_mlp_workspace_size(const sd2_matrix_t* gate_up, const sd2_matrix_t* down, int32_t k_tok,
                           size_t* bytes_out);
int sd2_sparse_mlp_forward(const sd2_matrix_t* gate_up, const sd2_matrix_t* down,
                           const uint16_t* x_bf16_dev, int32_t k_tok, float* y_dev,
                           void* workspace_dev, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ drafter stack
 * The decoder-linear stack of the draft model (Sec. 3: every decoder linear pruned,
 * embedding and LM head excluded), run on k_tok tokens.  Between the linears sits a
 * fixed minimal glue that keeps a block's data dependencies: RMS norm (eps 1e-5, no
 * learned scale), causal softmax attention among the k_tok in-flight tokens only
 * (grouped KV heads, scale 1/sqrt(head_dim), no rotary embedding, no cache), SiLU
 * gating, residual adds; activations are rounded to bf16 where a linear consumes them. */

typedef struct sd2_model_shape {
    int32_t layers, hidden, q_out, kv_out, inter, n_heads, n_kv, head_dim;
} sd2_model_shape_t;

typedef struct sd2_model sd2_model_t; /* host-side metadata only; owned by the library */

/* mats: 4 descriptors per layer in the order [q;k;v] fused (q_out+2*kv_out rows),
 * o, [gate;up] fused (2*inter rows), down.  Descriptors are copied. */
int sd2_model_create(const sd2_model_shape_t* shape, const sd2_matrix_t* mats, int32_t n_mats,
                     sd2_model_t** out);
int sd2_model_destroy(sd2_model_t* model);
int sd2_drafter_workspace_size(const sd2_model_t* model, int32_t k_tok, size_t* bytes_out);
/* h_in: device bf16 [k_tok][hidden]; h_out: device fp32 [k_tok][hidden]. */
int sd2_sparse_drafter_forward(const sd2_model_t* model, const uint16_t* h_in_bf16_dev, int32_t k_tok,
                               float* h_out_dev, void* workspace_dev, size_t workspace_bytes,
                               void* stream);
/* The forward is asynchronous and its single-launch kernel synchronises the GPU's compute units with
 * bounded waits (it needs all of them at once; a wait that runs out sets a flag in the workspace and the
 * kernel still ends).  This call waits for `stream`, reads that flag of the last forward that used
 * `workspace_dev` with this model and k_tok, and returns SD2_OK, SD2_ERR_TIMEOUT or SD2_ERR_RANGE.
 *
 * Arithmetic of the single-launch kernel (k_tok <= 8): every workgroup adds up its share of a linear in fp32 and hands
 * it over as a 32-bit fixed-point number with F = 17 fraction bits (SD2_OPT_FIXED_BITS); the shares and the residual
 * stream are summed by integer atomics, which are exact, so equal inputs give bit-identical outputs whatever the order
 * in which workgroups finish.  Resolution 2^-17 (the fp32 spacing at magnitude 64), range +-16384: a share must stay
 * below 8192 / (its linear's slab blocks) and a token's residual norm below 8192.  A forward that leaves that range
 * still ends, and the status call reports SD2_ERR_RANGE (results invalid) -- nothing wraps silently.  The
 * launch-per-step path (more tokens, dense or mixed models, SD2_OPT_FORWARD_MULTI) accumulates in fp32 throughout, in a
 * fixed order, and has no such range. */
int sd2_drafter_forward_status(const sd2_model_t* model, int32_t k_tok, const void* workspace_dev, void* stream);

/* Debug variant for step-by-step checking: the same forward, which also records, per linear
 * (4 per layer, in execution order), the fp32 values its input glue read -- the residual
 * stream for the normed inputs, the q|k|v results for attention, the gate|up results for the
 * gated product -- and the bf16 activations it handed to the linear.  trace_dev layout:
 * n_lin x [k_tok][kmax] uint16, then (256-byte aligned) n_lin x [k_tok][smax] float, with
 * kmax = max(hidden, q_out, inter) and smax = max(hidden, q_out + 2 kv_out, 2 inter); after that
 * (256-byte aligned, up to the size reported) per-workgroup timestamps of the single-launch kernel. */
int sd2_drafter_trace_size(const sd2_model_t* model, int32_t k_tok, size_t* bytes_out);
int sd2_sparse_drafter_forward_trace(const sd2_model_t* model, const uint16_t* h_in_bf16_dev,
                                     int32_t k_tok, float* h_out_dev, void* workspace_dev,
                                     size_t workspace_bytes, void* trace_dev, size_t trace_bytes,
                                     void* stream);

/* ------------------------------------------------------------------ decode step with a key/value cache
 * The drafter conditions each candidate on the prompt and on the candidates before it (Sec. 2.1, the definition of
 * p_{n+j+1}); for the Llama / Qwen decoders of Sec. 3 that is rotary position embedding and attention over the keys
 * and values of every earlier position.  This call runs the decoder-linear stack on k_tok new tokens at positions
 * pos0 .. pos0 + k_tok - 1 against a cache of the positions before them.  Differences from
 * sd2_sparse_drafter_forward, per layer:
 *   q, k  <- rotary embedding, half-split pairing: within a head, dimensions i and i + head_dim/2 (i < head_dim/2)
 *            rotate by the angle position * rope_theta^(-2 i / head_dim); values are not rotated
 *   cache <- bf16(k rotated), bf16(v) at positions pos0 + t
 *   token t attends to cache positions 0 .. pos0 + t (old and new positions alike are read from the cache)
 * k_cache_dev, v_cache_dev: device bf16 [layers][n_kv][max_pos][head_dim], 16-byte aligned, owned by the caller;
 * positions below pos0 must hold the history, positions from pos0 + k_tok on are neither read nor written.
 * 0 <= pos0, pos0 + k_tok <= max_pos; head_dim a multiple of 8; at most 8 query heads per key/value head;
 * max_pos limited by the attention kernel's LDS (about 12000 positions at 3 query heads per key/value head):
 * SD2_ERR_UNSUPPORTED beyond.  rope_theta > 1.  h_in, h_out, workspace as for sd2_sparse_drafter_forward, with the
 * size reported here.  Asynchronous on `stream`; all checks happen on the host before the first launch.
 * Where the single-launch kernel of sd2_sparse_drafter_forward serves the model (k_tok <= 8, head_dim 128, at most 4
 * query heads per key/value head) it runs here too, with one more step per layer: after the q|k|v linear the
 * workgroups share the attention over the cache (a stretch of positions each), and the linear that follows combines
 * their partial results.  Otherwise: one launch per linear and glue step.  sd2_drafter_decode_status is to this call
 * what sd2_drafter_forward_status is to the forward: it waits for `stream` and reports a bounded wait that ran out. */
int sd2_drafter_decode_workspace_size(const sd2_model_t* model, int32_t k_tok, size_t* bytes_out);
int sd2_drafter_decode_status(const sd2_model_t* model, int32_t k_tok, const void* workspace_dev, void* stream);
int sd2_sparse_drafter_decode(const sd2_model_t* model, const uint16_t* h_in_bf16_dev, int32_t k_tok, int32_t pos0,
                              uint16_t* k_cache_dev, uint16_t* v_cache_dev, int32_t max_pos, double rope_theta,
                              float* h_out_dev, void* workspace_dev, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ LM head with greedy choice
 * The drafter's next-token choice (Eq. 1 with greedy decoding, as in the footnote to Eq. 3): the
 * largest logit of the LM head, the one linear of the drafter that stays dense (Sec. 2.3 prunes
 * the decoder blocks; Sec. 3.2 counts the head's MACs in full).  For each of the k_tok rows of h:
 *   a = bf16(h / sqrt(mean(h^2) + 1e-5))      final RMS norm, no learned scale
 *   logit[v] = sum_c W[v][c] * a[c]            fp32 accumulation of exact bf16 products
 *   token = the lowest v among the largest logits
 * w_lm_bf16_dev: device, row-major [vocab][hidden] bf16 (the layout of nn.Linear.weight), read only.
 * h_dev: device fp32 [k_tok][hidden] (what sd2_sparse_drafter_forward writes).  token_ids_dev: device
 * int32 [k_tok].  max_logit_dev (fp32 [k_tok]) and logits_dev (fp32 [k_tok][vocab], every entry
 * written) are optional: NULL skips them, and without logits_dev nothing of size vocab is written.
 * hidden: a multiple of 128, at most 9216.  vocab >= 1 (need not be a multiple of 16).  k_tok > 16
 * streams the matrix once per 16 tokens.  workspace_dev: >= the reported size, 16-byte aligned,
 * contents irrelevant before and after.  A row whose logits are all NaN yields token 0.
 * Asynchronous on `stream`; all checks happen on the host before the first launch. */
int sd2_lm_head_workspace_size(int32_t vocab, int32_t hidden, int32_t k_tok, size_t* bytes_out);
int sd2_lm_head_argmax(const uint16_t* w_lm_bf16_dev, int32_t vocab, int32_t hidden, const float* h_dev,
                       int32_t k_tok, int32_t* token_ids_dev, float* max_logit_dev, float* logits_dev,
                       void* workspace_dev, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ drafting round
 * One round of drafting (Sec. 2.1, Eq. 1 with greedy decoding): k tokens, each chosen from the window extended by the
 * tokens chosen so far.  Step i embeds the window [start, d_0 .. d_{i-1}] (rows of emb_bf16_dev), runs the decoder-linear
 * stack on its i + 1 tokens (sd2_sparse_drafter_forward; the stack is causal and attends within the call, so recomputing
 * the window equals caching its keys and values), and gives the last position to the LM head (sd2_lm_head_argmax with
 * the tied matrix emb_bf16_dev as the head): d_i = lowest id among the largest logits.  Everything stays on the device
 * and is enqueued on `stream`: 3 k small launches plus k forwards, no host synchronisation, no memset nodes.
 * emb_bf16_dev: device [vocab][hidden] bf16, 16-byte aligned (embedding and LM head: the drafters of the paper tie them).
 * start_token_dev: device int32[1]; ids outside [0, vocab) are clamped.  draft_ids_dev: device int32[k], written in
 * order (entry i is read again by steps i+1..).  1 <= k <= 64.  The result feeds sd2_greedy_verify as `draft`.
 * sd2_draft_round_status waits for `stream` and returns SD2_ERR_TIMEOUT if a bounded wait of any step's forward ran out. */
int sd2_draft_round_workspace_size(const sd2_model_t* model, int32_t vocab, int32_t k, size_t* bytes_out);
int sd2_draft_round(const sd2_model_t* model, const uint16_t* emb_bf16_dev, int32_t vocab,
                    const int32_t* start_token_dev, int32_t k, int32_t* draft_ids_dev, void* workspace_dev,
                    size_t workspace_bytes, void* stream);
int sd2_draft_round_status(const sd2_model_t* model, int32_t vocab, int32_t k, const void* workspace_dev, void* stream);

/* The round against a key/value cache: k single-token steps of sd2_sparse_drafter_decode (the k sequential forwards of
 * Sec. 2.1, each conditioned on the prompt through the cache).  The start token sits at position pos0, the cache holds
 * positions 0 .. pos0 - 1; step i embeds one token (the start token, then d_{i-1}), decodes it at position pos0 + i
 * (appending its key and value) and gives the result to the LM head: d_i.  Afterwards the cache holds positions
 * pos0 .. pos0 + k - 1 (the start token and d_0 .. d_{k-2}).  pos0 + k <= max_pos.  Cache, rope_theta and limits as for
 * sd2_sparse_drafter_decode; everything else as for sd2_draft_round.  2 k small launches plus k decode steps and k heads,
 * no host synchronisation. */
int sd2_draft_round_cached_workspace_size(const sd2_model_t* model, int32_t vocab, int32_t k, size_t* bytes_out);
int sd2_draft_round_cached(const sd2_model_t* model, const uint16_t* emb_bf16_dev, int32_t vocab,
                           const int32_t* start_token_dev, int32_t k, int32_t pos0, uint16_t* k_cache_dev,
                           uint16_t* v_cache_dev, int32_t max_pos, double rope_theta, int32_t* draft_ids_dev,
                           void* workspace_dev, size_t workspace_bytes, void* stream);
int sd2_draft_round_cached_status(const sd2_model_t* model, int32_t vocab, int32_t k, const void* workspace_dev,
                                  void* stream);

/* ------------------------------------------------------------------ verification
 * Strict top-1 verification (Eq. 2): accepted_len[b] = number of leading positions
 * where draft[b][i] == target[b][i]; out_tokens[b] = those drafts, then target[b][n],
 * then -1 up to k+1 entries.  target[b][i] is the target model's greedy token after
 * the prompt and draft[b][0..i).  All arrays int32 on the device.  batch >= 0, k >= 0,
 * vocab > 0.  Ids are compared as opaque integers (they cannot be range-checked
 * without a device sync; use sd2_check_token_ids_host on host copies). */
int sd2_greedy_verify(const int32_t* draft_dev, const int32_t* target_dev, int32_t batch, int32_t k,
                      int32_t vocab, int32_t* accepted_len_dev, int32_t* out_tokens_dev, void* stream);
/* The same rule on host arrays, with the range check the device call cannot make: SD2_ERR_RANGE (and nothing
 * written) if any draft or target id lies outside [0, vocab).  A reference for callers that hold the ids on the
 * host anyway, and for checking a device result. */
int sd2_greedy_verify_host(const int32_t* draft, const int32_t* target, int32_t batch, int32_t k, int32_t vocab,
                           int32_t* accepted_len, int32_t* out_tokens);
/* SD2_ERR_RANGE if any of the n host ids lies outside [0, vocab). */
int sd2_check_token_ids_host(const int32_t* ids, size_t n, int32_t vocab);

/* Expected improvement factor of draft-then-verify over decoding with the target alone (Eq. 3): MAL / (k c + 1), with MAL the
 * mean number of tokens emitted per round (accepted drafts plus the target's one), k the drafts per round and c the cost of a
 * drafter step relative to a target step (a latency ratio in practice, a MAC ratio in theory: Sec. 2.1).  Host arithmetic in
 * double precision.  mean_emitted >= 0, k >= 0, cost_ratio >= 0 and all finite, else SD2_ERR_RANGE. */
int sd2_improvement_factor(double mean_emitted, int32_t k, double cost_ratio, double* factor_out);

/* ------------------------------------------------------------------ one-shot pruning
 * Sec. 2.3: every decoder linear is pruned one-shot to a uniform per-layer sparsity.  The paper's criterion is
 * second-order and needs calibration data; this call prunes by weight magnitude, in place, on the device:
 *   SD2_PRUNE_ROWS: per output row keep the k_in - (sparsity_pct * k_in) div 100 entries of largest |w|
 *                   (k_in a multiple of 256, at most 9216; SD2_ERR_UNSUPPORTED otherwise);
 *   SD2_PRUNE_2OF4: in every aligned group of four columns keep the two of largest |w| (sparsity_pct must be 50).
 * Ties go to the lower column; pruned entries become +0, kept ones keep their bits.  w_bf16_dev: device, row-major
 * [n_out][k_in] bf16, 16-byte aligned.  The result is what sd2_pack_sparse expects (after a copy to the host). */
#define SD2_PRUNE_ROWS 0
#define SD2_PRUNE_2OF4 1
int sd2_prune_magnitude(uint16_t* w_bf16_dev, int32_t n_out, int32_t k_in, int32_t sparsity_pct, int32_t pattern,
                        void* stream);

/* ------------------------------------------------------------------ sparse fine-tuning: masked gradient
 * Sec. 2.4 (and the sparse fine-tuning algorithm it refers to): the mask stays fixed during fine-tuning because
 * the gradients of pruned parameters are set to zero.  grad_dev: device, row-major [n_out][k_in], fp32
 * (grad_is_bf16 = 0) or bf16 (1), 16-byte aligned, updated in place: entries whose weight is pruned become +0
 * (a selection, so a NaN there vanishes), all others keep their bits.  `m`: a sparse descriptor in the bitmask
 * format (SD2_ERR_UNSUPPORTED for the 2:4 format), whose mask section is the mask.  Asynchronous on `stream`. */
int sd2_mask_gradient(const sd2_matrix_t* m, void* grad_dev, int32_t grad_is_bf16, void* stream);

/* ------------------------------------------------------------------ measurement aid
 * Plain device-to-device copy kernel (16 bytes per lane, grid-stride): dst[0..bytes) = src[0..bytes).
 * It moves exactly `bytes` in and `bytes` out, so the HBM counters it produces under a profiler give
 * the scale that turns the same counters of the other kernels into bytes.  bytes must be a multiple
 * of 16, both pointers 16-byte aligned, the ranges disjoint; asynchronous on `stream`. */
int sd2_calibration_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream);
/* Pure read stream of src[0..bytes) (16 bytes per lane, eight loads in flight, folded into checksums): the rate a
 * kernel that only reads reaches on this part, the ceiling the weight-streaming kernels are measured against next to
 * the published peak.  sink_dev: device, 2048 uint32 (one checksum per workgroup, overwritten).  bytes a non-zero
 * multiple of 16; pointers 16-byte aligned; asynchronous on `stream`. */
int sd2_calibration_read(const void* src_dev, size_t bytes, uint32_t* sink_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SD2_H */
