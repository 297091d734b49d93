// C ABI of libsd2 (see include/sd2.h): argument checks on the host, then launches.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <new>
#include <vector>

#include "sd2_format.h"
#include "sd2_internal.h"

using namespace sd2;

struct sd2_model {
    sd2_model_shape_t shape;
    std::vector<sd2_matrix_t> mats;  // 4 per layer: qkv, o, gate_up, down
};

namespace {

// Process-wide switches (sd2_set_option).  The environment is consulted once, when the first call needs a switch;
// after that a call reads an atomic and nothing else.
struct Options {
    std::atomic<int> v[SD2_OPT_COUNT];
    Options() {
        const char* e;
        v[SD2_OPT_FORWARD_MULTI] = ((e = getenv("SD2_FORWARD")) && strcmp(e, "multi") == 0) ? 1 : 0;
        v[SD2_OPT_LINEAR_PARTIALS] = ((e = getenv("SD2_LINEAR")) && strcmp(e, "partials") == 0) ? 1 : 0;
        v[SD2_OPT_SPIN_LIMIT] = (e = getenv("SD2_MEGA_SPIN_LIMIT")) ? std::max(0, atoi(e)) : -1;
        v[SD2_OPT_MEGA_TIMING] = ((e = getenv("SD2_MEGA_TIMING")) && (e[0] == '1' || e[0] == '2')) ? e[0] - '0' : 0;
        v[SD2_OPT_FIXED_BITS] = 17;
    }
};
Options& options() {
    static Options o;
    return o;
}
inline int option(int which) { return options().v[which].load(std::memory_order_relaxed); }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

inline bool is_nm24(const sd2_matrix_t* m) { return m->kind == SD2_KIND_SPARSE && m->info.format == SD2_FORMAT_NM24; }

int check_matrix(const sd2_matrix_t* m, int kind) {
    if (!m) return SD2_ERR_NULL;
    if (m->kind != kind) return SD2_ERR_FORMAT;
    if (!m->data_dev) return SD2_ERR_NULL;
    if (!aligned16(m->data_dev)) return SD2_ERR_BUFFER;
    const sd2_blob_info_t& i = m->info;
    if (i.n_out < 1 || i.k_in < 64 || i.k_in % 64) return SD2_ERR_SHAPE;
    if (i.n_strips != (int32_t)ceil_div((uint32_t)i.n_out, kStripRows) ||
        i.n_slabs != (int32_t)ceil_div((uint32_t)i.k_in, kSlabCols) || (int64_t)i.n_strips * i.n_slabs != i.n_tiles)
        return SD2_ERR_FORMAT;
    if (i.max_tile_nnz < 0 || i.max_tile_nnz > kStripRows * kSlabCols) return SD2_ERR_FORMAT;
    if (kind == SD2_KIND_SPARSE && i.format != SD2_FORMAT_BITMASK && i.format != SD2_FORMAT_NM24) return SD2_ERR_FORMAT;
    if (is_nm24(m) && !nm24_supported(i.n_slabs)) return SD2_ERR_UNSUPPORTED;  // k_in beyond 9216
    return SD2_OK;
}

MatArgs mat_args(const sd2_matrix_t* m) {
    MatArgs a;
    memset(&a, 0, sizeof(a));
    const uint8_t* base = static_cast<const uint8_t*>(m->data_dev);
    if (m->kind == SD2_KIND_SPARSE) {
        a.dir = base + kHeaderBytes;
        a.masks = reinterpret_cast<const uint2*>(base + m->info.mask_off);
        a.vals = reinterpret_cast<const uint16_t*>(base + m->info.val_off);
    } else {
        a.w = reinterpret_cast<const uint16_t*>(base);
    }
    a.n_out = m->info.n_out;
    a.k_in = m->info.k_in;
    a.n_strips = m->info.n_strips;
    a.n_slabs = m->info.n_slabs;
    a.n_tiles = m->info.n_tiles;
    a.max_tile_nnz = m->info.max_tile_nnz;
    return a;
}

// Partial results a linear leaves for the next kernel to add: one per slab, except that the 2:4 kernel adds the
// slabs up inside the workgroup and writes final values, and so does the streaming dense kernel.
inline bool is_dense_stream(const sd2_matrix_t* m) { return m->kind == SD2_KIND_DENSE && dense_stream_ok(m->info.k_in); }
inline int n_partials(const sd2_matrix_t* m) { return (is_nm24(m) || is_dense_stream(m)) ? 1 : m->info.n_slabs; }

size_t partial_bytes(const sd2_matrix_t* m, int k_tok) {
    return (size_t)n_partials(m) * (size_t)k_tok * (size_t)m->info.n_out * sizeof(float);
}

int check_tokens(int32_t k_tok) { return (k_tok < 1 || k_tok > SD2_MAX_TOKENS) ? SD2_ERR_RANGE : SD2_OK; }

// The bitmask format has a kernel that adds the slabs up inside the workgroup, too (up to 16 tokens, up to 32 slabs,
// tiles that fit its buffers); SD2_OPT_LINEAR_PARTIALS keeps the kernel with one partial result per slab (tests cover both).
inline bool sparse_final_ok(const sd2_matrix_t* m, int k_tok) {
    if (m->kind != SD2_KIND_SPARSE || is_nm24(m)) return false;
    if (option(SD2_OPT_LINEAR_PARTIALS)) return false;
    return sparse_strip_supported(mat_args(m), k_tok);
}

// The gate|up linear and the gated product in one launch (the bitmask kernel that adds the slabs up inside the workgroup).
inline bool gated_ok(const sd2_matrix_t* m, int k_tok) {
    return sparse_final_ok(m, k_tok) && sparse_strip_gated_supported(mat_args(m), k_tok);
}

// Partial results run_linear leaves in `out` for this token count (1: final values).  Never more than n_partials(m),
// which sizes the buffers.
inline int n_splits(const sd2_matrix_t* m, int k_tok) { return sparse_final_ok(m, k_tok) ? 1 : n_partials(m); }

hipError_t run_linear(const sd2_matrix_t* m, const uint16_t* x, int k_tok, float* out, hipStream_t s, bool allow_final = true) {
    MatArgs ma = mat_args(m);
    if (allow_final && sparse_final_ok(m, k_tok)) {
        LinArgs la{x, k_tok, out};
        return launch_sparse_strip_linear(ma, la, s);
    }
    if (is_nm24(m)) {
        // the structured-sparse matrix instruction takes 16 tokens; more tokens stream the matrix once per group
        for (int t0 = 0; t0 < k_tok; t0 += 16) {
            LinArgs la{x + (size_t)t0 * ma.k_in, std::min(16, k_tok - t0), out + (size_t)t0 * ma.n_out};
            const hipError_t e = launch_nm24_linear(ma, la, s);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    if (is_dense_stream(m))  // one launch; 32 tokens per pass where two groups' activations fit the registers, else 16
        return launch_dense_stream_linear(ma.w, x, ma.n_out, ma.k_in, k_tok, out, s);
    LinArgs la{x, k_tok, out};
    if (m->kind == SD2_KIND_SPARSE && option(SD2_OPT_LINEAR_PARTIALS) == 2 && sparse_linear_valu_supported(ma, k_tok))
        return launch_sparse_linear_valu(ma, la, s);  // the measurement variant without matrix instructions
    return m->kind == SD2_KIND_SPARSE ? launch_sparse_linear(ma, la, s) : launch_dense_linear(ma, la, s);
}

int linear_entry(const sd2_matrix_t* m, int kind, const uint16_t* x, int32_t k_tok, float* y, void* ws,
                 size_t ws_bytes, void* stream) {
    int rc = check_matrix(m, kind);
    if (rc != SD2_OK) return rc;
    if (!x || !y) return SD2_ERR_NULL;
    if ((rc = check_tokens(k_tok)) != SD2_OK) return rc;
    if (!aligned16(x) || !aligned16(y)) return SD2_ERR_BUFFER;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n_partials(m) > 1) {  // the contract of the workspace does not depend on which kernel runs
        if (!ws) return SD2_ERR_NULL;
        if (!aligned16(ws) || ws_bytes < partial_bytes(m, k_tok)) return SD2_ERR_BUFFER;
    }
    if (n_splits(m, k_tok) == 1) {
        return run_linear(m, x, k_tok, y, s) == hipSuccess ? SD2_OK : SD2_ERR_HIP;
    }
    float* part = static_cast<float*>(ws);
    if (run_linear(m, x, k_tok, part, s) != hipSuccess) return SD2_ERR_HIP;
    if (launch_reduce_partials(part, n_partials(m), (size_t)k_tok * m->info.n_out, y, s) != hipSuccess)
        return SD2_ERR_HIP;
    return SD2_OK;
}

struct StackLayout {
    size_t act_off, act2_off, part_off, ssq_off, total;  // two activation buffers: a fused kernel reads one and writes the other
};

StackLayout stack_layout(const sd2_model* md, int k_tok) {
    const sd2_model_shape_t& sh = md->shape;
    StackLayout L;
    const size_t widest = (size_t)std::max(std::max(sh.hidden, sh.q_out), sh.inter);
    L.act_off = 0;
    size_t part = 0;
    for (const sd2_matrix_t& m : md->mats) part = std::max(part, partial_bytes(&m, k_tok));
    L.act2_off = align256((size_t)k_tok * widest * sizeof(uint16_t));
    L.part_off = 2 * L.act2_off;
    L.ssq_off = L.part_off + align256(part);
    L.total = L.ssq_off + align256((size_t)k_tok * ((sh.hidden + 255) / 256) * sizeof(float));
    return L;
}

MegaGeo mega_geo(const sd2_matrix_t& m) {
    MegaGeo g;
    memset(&g, 0, sizeof(g));
    g.n_out = m.info.n_out;
    g.k_in = m.info.k_in;
    g.n_strips = m.info.n_strips;
    g.n_slabs = m.info.n_slabs;
    g.n_tiles = m.info.n_tiles;
    g.mask_off = m.info.mask_off;
    g.val_off = m.info.val_off;
    return g;
}

// The single-launch persistent kernel serves the decode regime (k_tok <= 8) of an all-sparse model
// whose layers share one geometry; everything else runs as one launch per linear and glue step.
// SD2_OPT_FORWARD_MULTI forces the latter (used by tests to cover both).
bool plan_mega_path(const sd2_model* md, int k_tok, MegaGeo (&geo)[4], bool* nm24_out = nullptr) {
    if (option(SD2_OPT_FORWARD_MULTI)) return false;
    const sd2_model_shape_t& sh = md->shape;
    if (sh.layers < 1) return false;
    int max_nnz = 0;
    for (size_t i = 0; i < md->mats.size(); ++i) {
        const sd2_matrix_t& m = md->mats[i];
        const sd2_matrix_t& ref = md->mats[i % 4];
        if (m.kind != SD2_KIND_SPARSE || m.info.format != md->mats[0].info.format) return false;  // one format throughout
        if (m.info.format != SD2_FORMAT_BITMASK && m.info.format != SD2_FORMAT_NM24) return false;
        if (m.info.mask_off != ref.info.mask_off || m.info.val_off != ref.info.val_off) return false;
        max_nnz = std::max(max_nnz, m.info.max_tile_nnz);
    }
    for (int kd = 0; kd < 4; ++kd) geo[kd] = mega_geo(md->mats[kd]);
    const bool nm24 = md->mats[0].info.format == SD2_FORMAT_NM24;
    if (nm24_out) *nm24_out = nm24;
    return mega_plan(geo, sh.layers, sh.hidden, sh.head_dim, k_tok, max_nnz, nm24);
}

// Workspace layout of the single-launch kernel for a plan made by plan_mega_path.
MegaLayout planned_layout(const sd2_model* md, int k_tok, const MegaGeo (&geo)[4]) {
    const sd2_model_shape_t& sh = md->shape;
    (void)geo;
    return mega_layout(sh.layers, sh.hidden, sh.q_out, sh.kv_out, sh.inter, k_tok);
}

}  // namespace

extern "C" {

const char* sd2_strerror(int status) {
    switch (status) {
        case SD2_OK: return "ok";
        case SD2_ERR_NULL: return "null pointer";
        case SD2_ERR_SHAPE: return "bad shape";
        case SD2_ERR_FORMAT: return "bad format or geometry";
        case SD2_ERR_BUFFER: return "buffer too small or misaligned";
        case SD2_ERR_BLOB: return "corrupt blob";
        case SD2_ERR_RANGE: return "value out of range";
        case SD2_ERR_HIP: return "HIP call failed";
        case SD2_ERR_UNSUPPORTED: return "not implemented in this build";
        case SD2_ERR_TIMEOUT: return "a bounded wait inside a kernel ran out";
        default: return "unknown status";
    }
}

int sd2_version(void) { return 101; }

int sd2_set_option(int32_t which, int32_t value) {
    if (which < 0 || which >= SD2_OPT_COUNT) return SD2_ERR_RANGE;
    if (which == SD2_OPT_FIXED_BITS) {
        if (value < 8 || value > 22) return SD2_ERR_RANGE;
    } else if (which == SD2_OPT_SPIN_LIMIT ? value < -1 : (value < 0 || value > ((which == SD2_OPT_MEGA_TIMING || which == SD2_OPT_LINEAR_PARTIALS) ? 2 : 1))) {
        return SD2_ERR_RANGE;
    }
    options().v[which].store(value, std::memory_order_relaxed);
    return SD2_OK;
}

int sd2_get_option(int32_t which, int32_t* value_out) {
    if (!value_out) return SD2_ERR_NULL;
    if (which < 0 || which >= SD2_OPT_COUNT) return SD2_ERR_RANGE;
    *value_out = option(which);
    return SD2_OK;
}

int sd2_matrix_init_sparse(sd2_matrix_t* m, const void* blob_host, size_t blob_bytes, const void* blob_dev) {
    if (!m || !blob_host || !blob_dev) return SD2_ERR_NULL;
    if (!aligned16(blob_dev)) return SD2_ERR_BUFFER;
    Header h;
    int rc = parse_header(blob_host, blob_bytes, &h);
    if (rc != SD2_OK) return rc;
    memset(m, 0, sizeof(*m));
    m->kind = SD2_KIND_SPARSE;
    m->data_dev = blob_dev;
    info_from_header(h, &m->info);
    return SD2_OK;
}

int sd2_matrix_init_dense(sd2_matrix_t* m, const uint16_t* w_dev, int32_t n_out, int32_t k_in) {
    if (!m || !w_dev) return SD2_ERR_NULL;
    if (!aligned16(w_dev)) return SD2_ERR_BUFFER;
    if (n_out < 1 || k_in < 64 || (k_in % 64) != 0 || (uint64_t)n_out * (uint64_t)k_in > (1ull << 36))
        return SD2_ERR_SHAPE;
    memset(m, 0, sizeof(*m));
    m->kind = SD2_KIND_DENSE;
    m->data_dev = w_dev;
    sd2_blob_info_t& i = m->info;
    i.n_out = n_out;
    i.k_in = k_in;
    i.n_strips = (int32_t)ceil_div((uint32_t)n_out, kStripRows);
    i.n_slabs = (int32_t)ceil_div((uint32_t)k_in, kSlabCols);
    i.n_tiles = i.n_strips * i.n_slabs;
    i.max_tile_nnz = kStripRows * kSlabCols;
    i.nnz = (uint64_t)n_out * k_in;
    i.total_bytes = i.useful_bytes = 2 * i.nnz;
    return SD2_OK;
}

int sd2_linear_workspace_size(const sd2_matrix_t* m, int32_t k_tok, size_t* bytes_out) {
    if (!m || !bytes_out) return SD2_ERR_NULL;
    if (m->kind != SD2_KIND_SPARSE && m->kind != SD2_KIND_DENSE) return SD2_ERR_FORMAT;
    int rc = check_tokens(k_tok);
    if (rc != SD2_OK) return rc;
    *bytes_out = n_partials(m) > 1 ? partial_bytes(m, k_tok) : 0;
    return SD2_OK;
}

int sd2_sparse_linear(const sd2_matrix_t* m, const uint16_t* x, int32_t k_tok, float* y, void* ws, size_t ws_bytes,
                      void* stream) {
    return linear_entry(m, SD2_KIND_SPARSE, x, k_tok, y, ws, ws_bytes, stream);
}

int sd2_sparse_linear_static(const sd2_matrix_t* m, const uint16_t* x, int32_t k_tok, float* y, void* stream) {
    int rc = check_matrix(m, SD2_KIND_SPARSE);
    if (rc != SD2_OK) return rc;
    if ((rc = check_tokens(k_tok)) != SD2_OK) return rc;
    // the size check comes first and touches no device: a request the static array cannot hold is refused as such
    if (n_partials(m) > 1 && partial_bytes(m, k_tok) > kStaticScratchBytes) return SD2_ERR_BUFFER;
    void* ws = nullptr;
    if (n_partials(m) > 1 && static_scratch(&ws) != hipSuccess) return SD2_ERR_HIP;
    return linear_entry(m, SD2_KIND_SPARSE, x, k_tok, y, ws, kStaticScratchBytes, stream);
}

int sd2_static_scratch_bytes(size_t* bytes_out) {
    if (!bytes_out) return SD2_ERR_NULL;
    *bytes_out = kStaticScratchBytes;
    return SD2_OK;
}

int sd2_sparse_linear_partials(const sd2_matrix_t* m, const uint16_t* x, int32_t k_tok, float* part, size_t part_bytes,
                               void* stream) {
    int rc = check_matrix(m, SD2_KIND_SPARSE);
    if (rc != SD2_OK) return rc;
    if (!x || !part) return SD2_ERR_NULL;
    if ((rc = check_tokens(k_tok)) != SD2_OK) return rc;
    if (!aligned16(x) || !aligned16(part) || part_bytes < partial_bytes(m, k_tok)) return SD2_ERR_BUFFER;
    return run_linear(m, x, k_tok, part, static_cast<hipStream_t>(stream), /*allow_final=*/false) == hipSuccess ? SD2_OK : SD2_ERR_HIP;
}

int sd2_dense_linear(const sd2_matrix_t* m, const uint16_t* x, int32_t k_tok, float* y, void* ws, size_t ws_bytes,
                     void* stream) {
    return linear_entry(m, SD2_KIND_DENSE, x, k_tok, y, ws, ws_bytes, stream);
}

static int mlp_check(const sd2_matrix_t* gu, const sd2_matrix_t* dn) {
    if (!gu || !dn) return SD2_ERR_NULL;
    int rc = check_matrix(gu, gu->kind);
    if (rc == SD2_OK) rc = check_matrix(dn, dn->kind);
    if (rc != SD2_OK) return rc;
    if ((gu->kind != SD2_KIND_SPARSE && gu->kind != SD2_KIND_DENSE) || gu->kind != dn->kind) return SD2_ERR_FORMAT;
    if (gu->info.n_out % 2 || gu->info.n_out / 2 != dn->info.k_in) return SD2_ERR_SHAPE;
    return SD2_OK;
}

int sd2_mlp_workspace_size(const sd2_matrix_t* gu, const sd2_matrix_t* dn, int32_t k_tok, size_t* bytes_out) {
    if (!bytes_out) return SD2_ERR_NULL;
    int rc = mlp_check(gu, dn);
    if (rc == SD2_OK) rc = check_tokens(k_tok);
    if (rc != SD2_OK) return rc;
    *bytes_out = align256((size_t)k_tok * dn->info.k_in * sizeof(uint16_t)) +
                 align256(std::max(partial_bytes(gu, k_tok), partial_bytes(dn, k_tok)));
    return SD2_OK;
}

int sd2_sparse_mlp_forward(const sd2_matrix_t* gu, const sd2_matrix_t* dn, const uint16_t* x, int32_t k_tok, float* y,
                           void* ws, size_t ws_bytes, void* stream) {
    size_t need = 0;
    int rc = sd2_mlp_workspace_size(gu, dn, k_tok, &need);
    if (rc != SD2_OK) return rc;
    if (!x || !y || !ws) return SD2_ERR_NULL;
    if (!aligned16(x) || !aligned16(y) || !aligned16(ws) || ws_bytes < need) return SD2_ERR_BUFFER;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int inter = dn->info.k_in;
    uint16_t* act = static_cast<uint16_t*>(ws);
    float* part = reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + align256((size_t)k_tok * inter * sizeof(uint16_t)));
    if (gated_ok(gu, k_tok)) {
        if (launch_sparse_strip_gated(mat_args(gu), x, k_tok, act, s) != hipSuccess) return SD2_ERR_HIP;
    } else {
        if (run_linear(gu, x, k_tok, part, s) != hipSuccess) return SD2_ERR_HIP;
        if (launch_silu_mul(part, n_splits(gu, k_tok), k_tok, inter, act, s) != hipSuccess) return SD2_ERR_HIP;
    }
    if (n_splits(dn, k_tok) == 1) return run_linear(dn, act, k_tok, y, s) == hipSuccess ? SD2_OK : SD2_ERR_HIP;
    if (run_linear(dn, act, k_tok, part, s) != hipSuccess) return SD2_ERR_HIP;
    if (launch_reduce_partials(part, n_splits(dn, k_tok), (size_t)k_tok * dn->info.n_out, y, s) != hipSuccess)
        return SD2_ERR_HIP;
    return SD2_OK;
}

int sd2_model_create(const sd2_model_shape_t* sh, const sd2_matrix_t* mats, int32_t n_mats, sd2_model_t** out) {
    if (!sh || !out) return SD2_ERR_NULL;
    *out = nullptr;
    if (sh->layers < 0 || sh->hidden < 64 || sh->q_out < 64 || sh->kv_out < 64 || sh->inter < 64 || sh->n_heads < 1 ||
        sh->n_kv < 1 || sh->head_dim < 8 || sh->head_dim > 256 || sh->head_dim % 8)
        return SD2_ERR_SHAPE;  // the attention kernels split a head's dimensions into eight equal parts
    if (sh->n_heads % sh->n_kv || (int64_t)sh->n_heads * sh->head_dim != sh->q_out ||
        (int64_t)sh->n_kv * sh->head_dim != sh->kv_out)
        return SD2_ERR_SHAPE;
    if (n_mats != 4 * sh->layers) return SD2_ERR_SHAPE;
    if (n_mats > 0 && !mats) return SD2_ERR_NULL;
    const int want[4][2] = {{sh->q_out + 2 * sh->kv_out, sh->hidden},
                            {sh->hidden, sh->q_out},
                            {2 * sh->inter, sh->hidden},
                            {sh->hidden, sh->inter}};
    for (int i = 0; i < n_mats; ++i) {
        const sd2_matrix_t* m = mats + i;
        if (m->kind != SD2_KIND_SPARSE && m->kind != SD2_KIND_DENSE) return SD2_ERR_FORMAT;
        int rc = check_matrix(m, m->kind);
        if (rc != SD2_OK) return rc;
        if (m->info.n_out != want[i % 4][0] || m->info.k_in != want[i % 4][1]) return SD2_ERR_SHAPE;
    }
    sd2_model* md = new (std::nothrow) sd2_model;
    if (!md) return SD2_ERR_BUFFER;
    md->shape = *sh;
    md->mats.assign(mats, mats + n_mats);
    *out = md;
    return SD2_OK;
}

int sd2_model_destroy(sd2_model_t* model) {
    delete model;
    return SD2_OK;
}

int sd2_drafter_workspace_size(const sd2_model_t* model, int32_t k_tok, size_t* bytes_out) {
    if (!model || !bytes_out) return SD2_ERR_NULL;
    int rc = check_tokens(k_tok);
    if (rc != SD2_OK) return rc;
    // the single-launch kernel's buffers count only where that kernel serves the model and the token count
    MegaGeo geo[4];
    const size_t mega = plan_mega_path(model, k_tok, geo) ? planned_layout(model, k_tok, geo).total : 0;
    *bytes_out = std::max(stack_layout(model, k_tok).total, mega);
    return SD2_OK;
}

struct TraceLayout {
    int kmax, smax;
    size_t x_off, src_off, time_off, total;
};

static TraceLayout trace_layout(const sd2_model* md, int k_tok) {
    const sd2_model_shape_t& sh = md->shape;
    TraceLayout T;
    T.kmax = std::max(std::max(sh.hidden, sh.q_out), sh.inter);
    T.smax = std::max(std::max(sh.hidden, sh.q_out + 2 * sh.kv_out), 2 * sh.inter);
    const size_t n_lin = (size_t)4 * sh.layers;
    T.x_off = 0;
    T.src_off = align256(n_lin * k_tok * T.kmax * sizeof(uint16_t));
    T.time_off = T.src_off + align256(n_lin * k_tok * T.smax * sizeof(float));
    // per workgroup and linear four timestamps (only the single-launch kernel fills them)
    T.total = T.time_off + align256((size_t)std::max(mega_grid_size(), 1) * n_lin * 8 * sizeof(unsigned long long));
    return T;
}

// Everything of the persistent kernel's argument block that the model, the token count and the workspace fix.
static void fill_mega_args(MegaArgs& ma, const sd2_model* md, int k_tok, const MegaLayout& ML, uint8_t* base, float* h_out) {
    const sd2_model_shape_t& sh = md->shape;
    ma.layers = sh.layers;
    ma.hidden = sh.hidden;
    ma.q_out = sh.q_out;
    ma.kv_out = sh.kv_out;
    ma.inter = sh.inter;
    ma.n_heads = sh.n_heads;
    ma.n_kv = sh.n_kv;
    ma.head_dim = sh.head_dim;
    ma.k_tok = k_tok;
    // about a second of polling per barrier before the forward is given up (SD2_OPT_SPIN_LIMIT overrides: tests)
    ma.spin_limit = option(SD2_OPT_SPIN_LIMIT) >= 0 ? option(SD2_OPT_SPIN_LIMIT) : 1 << 20;
    ma.h_out = h_out;
    ma.bar = reinterpret_cast<unsigned*>(base + ML.bar_off);
    ma.err = reinterpret_cast<unsigned*>(base + ML.err_off);
    ma.yqkv = reinterpret_cast<int*>(base + ML.yqkv_off);
    ma.ygu = reinterpret_cast<int*>(base + ML.ygu_off);
    ma.hv = reinterpret_cast<int*>(base + ML.hv_off);
    ma.h_stride = ML.h_stride;
    ma.yqkv_stride = ML.yqkv_stride;
    ma.ygu_stride = ML.ygu_stride;
    // fixed point of the sums that cross compute units: F fraction bits (SD2_OPT_FIXED_BITS), limits that exclude a wrap
    const int fbits = option(SD2_OPT_FIXED_BITS);
    ma.fix_scale = std::ldexp(1.0f, fbits);
    ma.fix_inv = std::ldexp(1.0f, -fbits);
    for (int kd = 0; kd < 4; ++kd) ma.fix_limit[kd] = std::ldexp(1.0f, 30) / (float)std::max(ma.geo[kd].n_bblk, 1);
    ma.h_limit_sq = std::ldexp(1.0f, 2 * (30 - fbits));
    for (size_t i = 0; i < md->mats.size(); ++i) ma.blob[i] = static_cast<const unsigned char*>(md->mats[i].data_dev);
}

static int forward_impl(const sd2_model_t* md, const uint16_t* h_in, int32_t k_tok, float* h_out, void* ws,
                        size_t ws_bytes, void* trace, void* stream) {
    if (!md || !h_in || !h_out || !ws) return SD2_ERR_NULL;
    int rc = check_tokens(k_tok);
    if (rc != SD2_OK) return rc;
    const StackLayout L = stack_layout(md, k_tok);
    const sd2_model_shape_t& sh = md->shape;
    hipStream_t s = static_cast<hipStream_t>(stream);
    MegaArgs ma;
    memset(&ma, 0, sizeof(ma));
    bool nm24 = false;
    const bool single_launch = plan_mega_path(md, k_tok, ma.geo, &nm24);
    MegaLayout ML;
    memset(&ML, 0, sizeof(ML));
    if (single_launch) ML = planned_layout(md, k_tok, ma.geo);
    if (!aligned16(h_in) || !aligned16(h_out) || !aligned16(ws) || ws_bytes < std::max(L.total, ML.total))
        return SD2_ERR_BUFFER;
    if (single_launch) {
        uint8_t* base = static_cast<uint8_t*>(ws);
        fill_mega_args(ma, md, k_tok, ML, base, h_out);
        bool probe = false;
        if (trace) {
            const TraceLayout T = trace_layout(md, k_tok);
            ma.trace_x = reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(trace) + T.x_off);
            ma.trace_src = reinterpret_cast<float*>(static_cast<uint8_t*>(trace) + T.src_off);
            ma.trace_kmax = T.kmax;
            ma.trace_smax = T.smax;
            ma.trace_time = reinterpret_cast<unsigned long long*>(static_cast<uint8_t*>(trace) + T.time_off);
            // SD2_OPT_MEGA_TIMING = 1: keep only the per-workgroup timestamps (profiling the production kernel);
            // = 2: the same plus wavefront 0's split into waiting for streams and decoding
            const int tonly = option(SD2_OPT_MEGA_TIMING);
            if (tonly) ma.trace_x = nullptr;
            probe = tonly == 2 && !nm24;  // the wait/decode split exists for the bitmask format only
        }
        return launch_mega_forward(ma, h_in, base, ML.hv_off, probe, nm24, s) == hipSuccess ? SD2_OK : SD2_ERR_HIP;
    }
    uint16_t* act = reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(ws) + L.act_off);
    uint16_t* act2 = reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(ws) + L.act2_off);
    float* part = reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + L.part_off);
    float* ssq = reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + L.ssq_off);
    float* h = h_out;  // the residual stream lives in the output buffer
#define SD2_TRY(expr) \
    if ((expr) != hipSuccess) return SD2_ERR_HIP
    const TraceLayout T = trace_layout(md, k_tok);
    // records what linear `lin` consumed: `width` fp32 source values per token (copied, or summed from partials)
    // and the `k_in` bf16 activations now sitting in `act`
    auto record = [&](int lin, const float* src_copy, const float* src_part, int n_splits, int width, int k_in) -> hipError_t {
        if (!trace) return hipSuccess;
        uint16_t* tx = reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(trace) + T.x_off) + (size_t)lin * k_tok * T.kmax;
        float* ts = reinterpret_cast<float*>(static_cast<uint8_t*>(trace) + T.src_off) + (size_t)lin * k_tok * T.smax;
        hipError_t e = hipMemcpy2DAsync(tx, (size_t)T.kmax * 2, act, (size_t)k_in * 2, (size_t)k_in * 2, k_tok,
                                        hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return e;
        if (src_copy)
            return hipMemcpy2DAsync(ts, (size_t)T.smax * 4, src_copy, (size_t)width * 4, (size_t)width * 4, k_tok,
                                    hipMemcpyDeviceToDevice, s);
        for (int t = 0; t < k_tok; ++t) {
            // partials are [split][token][width]: reduce one token row at a time into the padded trace row
            e = launch_reduce_partials_strided(src_part + (size_t)t * width, n_splits, (size_t)k_tok * width, (size_t)width,
                                               ts + (size_t)t * T.smax, s);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    };
    SD2_TRY(launch_residual_rmsnorm(h, h_in, nullptr, 0, k_tok, sh.hidden, sh.layers > 0 ? act : nullptr, ssq, s));
    for (int l = 0; l < sh.layers; ++l) {
        const sd2_matrix_t* qkv = &md->mats[4 * l + 0];
        const sd2_matrix_t* o = &md->mats[4 * l + 1];
        const sd2_matrix_t* gu = &md->mats[4 * l + 2];
        const sd2_matrix_t* dn = &md->mats[4 * l + 3];
        SD2_TRY(record(4 * l + 0, h, nullptr, 0, sh.hidden, sh.hidden));
        SD2_TRY(run_linear(qkv, act, k_tok, part, s));
        SD2_TRY(launch_inflight_attention(part, n_splits(qkv, k_tok), k_tok, sh.q_out, sh.kv_out, sh.n_heads, sh.n_kv,
                                          sh.head_dim, act, s));
        SD2_TRY(record(4 * l + 1, nullptr, part, n_splits(qkv, k_tok), sh.q_out + 2 * sh.kv_out, sh.q_out));
        SD2_TRY(run_linear(o, act, k_tok, part, s));
        SD2_TRY(launch_residual_rmsnorm(h, nullptr, part, n_splits(o, k_tok), k_tok, sh.hidden, act, ssq, s));
        SD2_TRY(record(4 * l + 2, h, nullptr, 0, sh.hidden, sh.hidden));
        if (!trace && gated_ok(gu, k_tok)) {
            // one launch: the gated product is written by the linear's own epilogue (act is read and written: the
            // kernel has taken its input columns into registers before the first result leaves)
            SD2_TRY(launch_sparse_strip_gated(mat_args(gu), act, k_tok, act2, s));
            std::swap(act, act2);
        } else {
            SD2_TRY(run_linear(gu, act, k_tok, part, s));
            SD2_TRY(launch_silu_mul(part, n_splits(gu, k_tok), k_tok, sh.inter, act, s));
        }
        SD2_TRY(record(4 * l + 3, nullptr, part, n_splits(gu, k_tok), 2 * sh.inter, sh.inter));
        SD2_TRY(run_linear(dn, act, k_tok, part, s));
        SD2_TRY(launch_residual_rmsnorm(h, nullptr, part, n_splits(dn, k_tok), k_tok, sh.hidden,
                                        l + 1 < sh.layers ? act : nullptr, ssq, s));
    }
#undef SD2_TRY
    return SD2_OK;
}

int sd2_sparse_drafter_forward(const sd2_model_t* md, const uint16_t* h_in, int32_t k_tok, float* h_out, void* ws,
                               size_t ws_bytes, void* stream) {
    return forward_impl(md, h_in, k_tok, h_out, ws, ws_bytes, nullptr, stream);
}

int sd2_drafter_forward_status(const sd2_model_t* md, int32_t k_tok, const void* ws, void* stream) {
    if (!md || !ws) return SD2_ERR_NULL;
    int rc = check_tokens(k_tok);
    if (rc != SD2_OK) return rc;
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return SD2_ERR_HIP;
    MegaGeo geo[4];
    if (!plan_mega_path(md, k_tok, geo)) return SD2_OK;  // the multi-launch path has no waits inside kernels
    const MegaLayout ML = planned_layout(md, k_tok, geo);
    unsigned flag = 0;
    if (hipMemcpy(&flag, static_cast<const uint8_t*>(ws) + ML.err_off, sizeof(flag), hipMemcpyDeviceToHost) != hipSuccess)
        return SD2_ERR_HIP;
    return (flag & 1u) ? SD2_ERR_TIMEOUT : ((flag & 2u) ? SD2_ERR_RANGE : SD2_OK);
}

int sd2_drafter_trace_size(const sd2_model_t* model, int32_t k_tok, size_t* bytes_out) {
    if (!model || !bytes_out) return SD2_ERR_NULL;
    int rc = check_tokens(k_tok);
    if (rc != SD2_OK) return rc;
    *bytes_out = std::max(trace_layout(model, k_tok).total, (size_t)256);
    return SD2_OK;
}

int sd2_sparse_drafter_forward_trace(const sd2_model_t* md, const uint16_t* h_in, int32_t k_tok, float* h_out, void* ws,
                                     size_t ws_bytes, void* trace, size_t trace_bytes, void* stream) {
    if (!md || !trace) return SD2_ERR_NULL;
    int rc = check_tokens(k_tok);
    if (rc != SD2_OK) return rc;
    if (!aligned16(trace) || trace_bytes < trace_layout(md, k_tok).total) return SD2_ERR_BUFFER;
    return forward_impl(md, h_in, k_tok, h_out, ws, ws_bytes, trace, stream);
}

// ------------------------------------------------------------------ decode step with a key/value cache

struct DecodeLayout {
    size_t q_off, table_off;               // one launch per step: rotated queries, angle table
    size_t mega_table_off, mega_part_off;  // single launch: angle table and partial attention results after its own workspace
    int chunks;                            // workgroups per (key/value head, token) of the single-launch attention step, 0: not served
    size_t total;
};

static DecodeLayout decode_layout(const sd2_model* md, int k_tok) {
    const sd2_model_shape_t& sh = md->shape;
    DecodeLayout D;
    D.q_off = stack_layout(md, k_tok).total;
    D.table_off = D.q_off + align256((size_t)k_tok * sh.q_out * sizeof(float));
    const size_t table_bytes = align256((size_t)k_tok * (sh.head_dim / 2 + 1) * sizeof(float2));
    D.total = D.table_off + table_bytes;
    D.chunks = 0;
    D.mega_table_off = D.mega_part_off = 0;
    MegaGeo geo[4];
    if (k_tok <= kMegaMaxTok && plan_mega_path(md, k_tok, geo)) {
        D.chunks = mega_attention_chunks(sh.n_heads, sh.n_kv, k_tok);
        if (D.chunks > 0) {
            D.mega_table_off = planned_layout(md, k_tok, geo).total;
            D.mega_part_off = D.mega_table_off + table_bytes;
            const size_t part = (size_t)sh.layers * k_tok * sh.n_heads * D.chunks * kMegaAttPartDw * sizeof(float);
            D.total = std::max(D.total, D.mega_part_off + align256(part));
        }
    }
    return D;
}

int sd2_drafter_decode_workspace_size(const sd2_model_t* model, int32_t k_tok, size_t* bytes_out) {
    if (!model || !bytes_out) return SD2_ERR_NULL;
    int rc = check_tokens(k_tok);
    if (rc != SD2_OK) return rc;
    *bytes_out = decode_layout(model, k_tok).total;
    return SD2_OK;
}

int sd2_drafter_decode_status(const sd2_model_t* md, int32_t k_tok, const void* ws, void* stream) {
    if (!md || !ws) return SD2_ERR_NULL;
    int rc = check_tokens(k_tok);
    if (rc != SD2_OK) return rc;
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return SD2_ERR_HIP;
    if (decode_layout(md, k_tok).chunks == 0) return SD2_OK;  // one launch per step: no waits inside kernels
    MegaGeo geo[4];
    if (!plan_mega_path(md, k_tok, geo)) return SD2_OK;
    const MegaLayout ML = planned_layout(md, k_tok, geo);
    unsigned flag = 0;
    if (hipMemcpy(&flag, static_cast<const uint8_t*>(ws) + ML.err_off, sizeof(flag), hipMemcpyDeviceToHost) != hipSuccess)
        return SD2_ERR_HIP;
    return (flag & 1u) ? SD2_ERR_TIMEOUT : ((flag & 2u) ? SD2_ERR_RANGE : SD2_OK);
}

int sd2_sparse_drafter_decode(const sd2_model_t* md, const uint16_t* h_in, int32_t k_tok, int32_t pos0, uint16_t* k_cache,
                              uint16_t* v_cache, int32_t max_pos, double rope_theta, float* h_out, void* ws, size_t ws_bytes,
                              void* stream) {
    if (!md || !h_in || !h_out || !ws || !k_cache || !v_cache) return SD2_ERR_NULL;
    int rc = check_tokens(k_tok);
    if (rc != SD2_OK) return rc;
    const sd2_model_shape_t& sh = md->shape;
    if (max_pos < 1 || pos0 < 0 || (int64_t)pos0 + k_tok > max_pos || !(rope_theta > 1.0)) return SD2_ERR_RANGE;
    if (!cached_attention_supported(sh.n_heads, sh.n_kv, sh.head_dim, max_pos)) return SD2_ERR_UNSUPPORTED;
    const StackLayout L = stack_layout(md, k_tok);
    const DecodeLayout DL = decode_layout(md, k_tok);
    if (!aligned16(h_in) || !aligned16(h_out) || !aligned16(ws) || !aligned16(k_cache) || !aligned16(v_cache) ||
        ws_bytes < DL.total)
        return SD2_ERR_BUFFER;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* base = static_cast<uint8_t*>(ws);
    if (DL.chunks > 0) {
        // single launch: the persistent kernel with an attention step over the cache after each q|k|v linear
        MegaArgs ma;
        memset(&ma, 0, sizeof(ma));
        bool nm24 = false;
        if (!plan_mega_path(md, k_tok, ma.geo, &nm24)) return SD2_ERR_UNSUPPORTED;
        const MegaLayout ML = planned_layout(md, k_tok, ma.geo);
        fill_mega_args(ma, md, k_tok, ML, base, h_out);
        float2* table = reinterpret_cast<float2*>(base + DL.mega_table_off);
        ma.k_cache = k_cache;
        ma.v_cache = v_cache;
        ma.rope = table;
        ma.att_part = reinterpret_cast<float*>(base + DL.mega_part_off);
        ma.max_pos = max_pos;
        ma.pos0 = pos0;
        // a stretch of about a hundred positions per workgroup (two passes of its loads), as far as the workgroups go
        ma.att_chunks = std::max(1, std::min(DL.chunks, (pos0 + 95) / 96));
        if (launch_rope_table(pos0, k_tok, sh.head_dim, rope_theta, table, s) != hipSuccess) return SD2_ERR_HIP;
        return launch_mega_forward(ma, h_in, base, ML.hv_off, false, nm24, s) == hipSuccess ? SD2_OK : SD2_ERR_HIP;
    }
    uint16_t* act = reinterpret_cast<uint16_t*>(base + L.act_off);
    uint16_t* act2 = reinterpret_cast<uint16_t*>(base + L.act2_off);
    float* part = reinterpret_cast<float*>(base + L.part_off);
    float* ssq = reinterpret_cast<float*>(base + L.ssq_off);
    float* q_rot = reinterpret_cast<float*>(base + DL.q_off);
    float2* table = reinterpret_cast<float2*>(base + DL.table_off);
    float* h = h_out;  // the residual stream lives in the output buffer
    const size_t layer_elems = (size_t)sh.n_kv * max_pos * sh.head_dim;
#define SD2_TRY(expr) \
    if ((expr) != hipSuccess) return SD2_ERR_HIP
    SD2_TRY(launch_rope_table(pos0, k_tok, sh.head_dim, rope_theta, table, s));
    SD2_TRY(launch_residual_rmsnorm(h, h_in, nullptr, 0, k_tok, sh.hidden, sh.layers > 0 ? act : nullptr, ssq, s));
    for (int l = 0; l < sh.layers; ++l) {
        const sd2_matrix_t* qkv = &md->mats[4 * l + 0];
        const sd2_matrix_t* o = &md->mats[4 * l + 1];
        const sd2_matrix_t* gu = &md->mats[4 * l + 2];
        const sd2_matrix_t* dn = &md->mats[4 * l + 3];
        uint16_t* kc = k_cache + (size_t)l * layer_elems;
        uint16_t* vc = v_cache + (size_t)l * layer_elems;
        SD2_TRY(run_linear(qkv, act, k_tok, part, s));
        SD2_TRY(launch_rope_append(part, n_splits(qkv, k_tok), k_tok, sh.q_out, sh.kv_out, sh.n_heads, sh.n_kv, sh.head_dim, table,
                                   pos0, max_pos, q_rot, kc, vc, s));
        SD2_TRY(launch_cached_attention(q_rot, kc, vc, max_pos, pos0, k_tok, sh.q_out, sh.n_heads, sh.n_kv, sh.head_dim, act, s));
        SD2_TRY(run_linear(o, act, k_tok, part, s));
        SD2_TRY(launch_residual_rmsnorm(h, nullptr, part, n_splits(o, k_tok), k_tok, sh.hidden, act, ssq, s));
        if (gated_ok(gu, k_tok)) {
            SD2_TRY(launch_sparse_strip_gated(mat_args(gu), act, k_tok, act2, s));
            std::swap(act, act2);
        } else {
            SD2_TRY(run_linear(gu, act, k_tok, part, s));
            SD2_TRY(launch_silu_mul(part, n_splits(gu, k_tok), k_tok, sh.inter, act, s));
        }
        SD2_TRY(run_linear(dn, act, k_tok, part, s));
        SD2_TRY(launch_residual_rmsnorm(h, nullptr, part, n_splits(dn, k_tok), k_tok, sh.hidden,
                                        l + 1 < sh.layers ? act : nullptr, ssq, s));
    }
#undef SD2_TRY
    return SD2_OK;
}

int sd2_greedy_verify(const int32_t* draft, const int32_t* target, int32_t batch, int32_t k, int32_t vocab,
                      int32_t* accepted, int32_t* out_tokens, void* stream) {
    if (batch < 0 || k < 0) return SD2_ERR_SHAPE;
    if (vocab < 1) return SD2_ERR_RANGE;
    if (batch == 0) return SD2_OK;
    if (!target || !accepted || !out_tokens || (k > 0 && !draft)) return SD2_ERR_NULL;
    if (launch_greedy_verify(draft, target, batch, k, accepted, out_tokens, static_cast<hipStream_t>(stream)) != hipSuccess)
        return SD2_ERR_HIP;
    return SD2_OK;
}

int sd2_improvement_factor(double mean_emitted, int32_t k, double cost_ratio, double* factor_out) {
    if (!factor_out) return SD2_ERR_NULL;
    if (!(mean_emitted >= 0.0) || !(cost_ratio >= 0.0) || k < 0 || !std::isfinite(mean_emitted) || !std::isfinite(cost_ratio))
        return SD2_ERR_RANGE;
    *factor_out = mean_emitted / ((double)k * cost_ratio + 1.0);
    return SD2_OK;
}

int sd2_greedy_verify_host(const int32_t* draft, const int32_t* target, int32_t batch, int32_t k, int32_t vocab,
                           int32_t* accepted, int32_t* out_tokens) {
    if (batch < 0 || k < 0) return SD2_ERR_SHAPE;
    if (vocab < 1) return SD2_ERR_RANGE;
    if (batch == 0) return SD2_OK;
    if (!target || !accepted || !out_tokens || (k > 0 && !draft)) return SD2_ERR_NULL;
    // ids are checked before anything is written
    for (int64_t i = 0; i < (int64_t)batch * k; ++i)
        if (draft[i] < 0 || draft[i] >= vocab) return SD2_ERR_RANGE;
    for (int64_t i = 0; i < (int64_t)batch * (k + 1); ++i)
        if (target[i] < 0 || target[i] >= vocab) return SD2_ERR_RANGE;
    for (int32_t b = 0; b < batch; ++b) {
        const int32_t* d = draft + (int64_t)b * k;
        const int32_t* t = target + (int64_t)b * (k + 1);
        int32_t* o = out_tokens + (int64_t)b * (k + 1);
        int32_t n = 0;
        while (n < k && d[n] == t[n]) ++n;  // the longest prefix on which the drafter agrees with the target
        accepted[b] = n;
        for (int32_t i = 0; i < n; ++i) o[i] = d[i];
        o[n] = t[n];                        // then the target's own token
        for (int32_t i = n + 1; i <= k; ++i) o[i] = -1;
    }
    return SD2_OK;
}

int sd2_check_token_ids_host(const int32_t* ids, size_t n, int32_t vocab) {
    if (n > 0 && !ids) return SD2_ERR_NULL;
    if (vocab < 1) return SD2_ERR_RANGE;
    for (size_t i = 0; i < n; ++i)
        if (ids[i] < 0 || ids[i] >= vocab) return SD2_ERR_RANGE;
    return SD2_OK;
}

int sd2_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (bytes == 0) return SD2_OK;
    if (!dst || !src) return SD2_ERR_NULL;
    if (bytes % 16 != 0 || !aligned16(dst) || !aligned16(src)) return SD2_ERR_BUFFER;
    if (launch_calibration_copy(dst, src, bytes, static_cast<hipStream_t>(stream)) != hipSuccess) return SD2_ERR_HIP;
    return SD2_OK;
}

int sd2_calibration_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
    if (!src || !sink) return SD2_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || !aligned16(src) || !aligned16(sink)) return SD2_ERR_BUFFER;
    if (launch_calibration_read(src, bytes, sink, static_cast<hipStream_t>(stream)) != hipSuccess) return SD2_ERR_HIP;
    return SD2_OK;
}

// ---- one-shot magnitude pruning

int sd2_prune_magnitude(uint16_t* w, int32_t n_out, int32_t k_in, int32_t sparsity_pct, int32_t pattern, void* stream) {
    if (!w) return SD2_ERR_NULL;
    if (!aligned16(w)) return SD2_ERR_BUFFER;
    if (n_out < 1 || k_in < 64 || k_in % 64 || (uint64_t)n_out * (uint64_t)k_in > (1ull << 36)) return SD2_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (pattern == SD2_PRUNE_2OF4) {
        if (sparsity_pct != 50) return SD2_ERR_RANGE;
        return launch_prune_2of4(w, n_out, k_in, s) == hipSuccess ? SD2_OK : SD2_ERR_HIP;
    }
    if (pattern != SD2_PRUNE_ROWS) return SD2_ERR_FORMAT;
    if (sparsity_pct < 0 || sparsity_pct > 99) return SD2_ERR_RANGE;
    if (k_in % 256 || k_in > 9216) return SD2_ERR_UNSUPPORTED;
    const int n_keep = k_in - (int)(((int64_t)sparsity_pct * k_in) / 100);
    return launch_prune_rows(w, n_out, k_in, n_keep, s) == hipSuccess ? SD2_OK : SD2_ERR_HIP;
}

// ---- masked gradient of sparse fine-tuning

int sd2_mask_gradient(const sd2_matrix_t* m, void* grad, int32_t grad_is_bf16, void* stream) {
    int rc = check_matrix(m, SD2_KIND_SPARSE);
    if (rc != SD2_OK) return rc;
    if (m->info.format != SD2_FORMAT_BITMASK) return SD2_ERR_UNSUPPORTED;
    if (!grad) return SD2_ERR_NULL;
    if (!aligned16(grad)) return SD2_ERR_BUFFER;
    if (grad_is_bf16 != 0 && grad_is_bf16 != 1) return SD2_ERR_RANGE;
    return launch_mask_gradient(mat_args(m), grad, grad_is_bf16 != 0, static_cast<hipStream_t>(stream)) == hipSuccess
               ? SD2_OK
               : SD2_ERR_HIP;
}

// ---- LM head with greedy choice

static int lm_head_check(int32_t vocab, int32_t hidden, int32_t k_tok) {
    if (vocab < 1 || hidden < 128 || hidden % 128 != 0 || hidden > kLmMaxHidden) return SD2_ERR_SHAPE;
    if (k_tok < 1 || k_tok > SD2_MAX_TOKENS) return SD2_ERR_RANGE;
    return SD2_OK;
}

int sd2_lm_head_workspace_size(int32_t vocab, int32_t hidden, int32_t k_tok, size_t* bytes_out) {
    if (!bytes_out) return SD2_ERR_NULL;
    const int rc = lm_head_check(vocab, hidden, k_tok);
    if (rc != SD2_OK) return rc;
    *bytes_out = (size_t)kLmMaxWorkgroups * 16 * 8;
    return SD2_OK;
}

int sd2_lm_head_argmax(const uint16_t* w_lm, int32_t vocab, int32_t hidden, const float* h, int32_t k_tok,
                       int32_t* token_ids, float* max_logit, float* logits, void* workspace, size_t workspace_bytes,
                       void* stream) {
    if (!w_lm || !h || !token_ids || !workspace) return SD2_ERR_NULL;
    const int rc = lm_head_check(vocab, hidden, k_tok);
    if (rc != SD2_OK) return rc;
    if (!aligned16(w_lm) || !aligned16(h) || !aligned16(workspace)) return SD2_ERR_BUFFER;
    if (workspace_bytes < (size_t)kLmMaxWorkgroups * 16 * 8) return SD2_ERR_BUFFER;
    // the matrix cores take 16 tokens at a time; a larger k_tok streams the head once per group of 16
    for (int32_t t0 = 0; t0 < k_tok; t0 += 16) {
        const int32_t kt = std::min<int32_t>(16, k_tok - t0);
        if (launch_lm_head(w_lm, h + (size_t)t0 * hidden, vocab, hidden, kt, workspace, token_ids + t0,
                           max_logit ? max_logit + t0 : nullptr, logits ? logits + (size_t)t0 * vocab : nullptr,
                           static_cast<hipStream_t>(stream)) != hipSuccess)
            return SD2_ERR_HIP;
    }
    return SD2_OK;
}

// ---- drafting round

namespace {
struct RoundLayout {
    size_t hin_off, hout_off, flag_off, lm_off, fwd_off, fwd_bytes, total;
};

int round_layout(const sd2_model_t* md, int32_t vocab, int32_t k, RoundLayout* L) {
    if (!md) return SD2_ERR_NULL;
    if (k < 1 || k > SD2_MAX_TOKENS) return SD2_ERR_RANGE;
    const sd2_model_shape_t& sh = md->shape;
    int rc = lm_head_check(vocab, sh.hidden, 1);
    if (rc != SD2_OK) return rc;
    size_t fwd = 0;
    for (int32_t kt = 1; kt <= k; ++kt) {
        size_t b = 0;
        if ((rc = sd2_drafter_workspace_size(md, kt, &b)) != SD2_OK) return rc;
        fwd = std::max(fwd, b);
    }
    L->hin_off = 0;
    L->hout_off = align256((size_t)k * sh.hidden * sizeof(uint16_t));
    L->flag_off = L->hout_off + align256((size_t)k * sh.hidden * sizeof(float));
    L->lm_off = L->flag_off + 256;
    L->fwd_off = L->lm_off + align256((size_t)kLmMaxWorkgroups * 16 * 8);
    L->fwd_bytes = fwd;
    L->total = L->fwd_off + align256(fwd);
    return SD2_OK;
}
}  // namespace

int sd2_draft_round_workspace_size(const sd2_model_t* model, int32_t vocab, int32_t k, size_t* bytes_out) {
    if (!bytes_out) return SD2_ERR_NULL;
    RoundLayout L;
    const int rc = round_layout(model, vocab, k, &L);
    if (rc != SD2_OK) return rc;
    *bytes_out = L.total;
    return SD2_OK;
}

int sd2_draft_round(const sd2_model_t* model, const uint16_t* emb, int32_t vocab, const int32_t* start_token, int32_t k,
                    int32_t* draft_ids, void* ws, size_t ws_bytes, void* stream) {
    RoundLayout L;
    int rc = round_layout(model, vocab, k, &L);
    if (rc != SD2_OK) return rc;
    if (!emb || !start_token || !draft_ids || !ws) return SD2_ERR_NULL;
    if (!aligned16(emb) || !aligned16(ws) || ws_bytes < L.total) return SD2_ERR_BUFFER;
    const sd2_model_shape_t& sh = model->shape;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* base = static_cast<uint8_t*>(ws);
    uint16_t* h_in = reinterpret_cast<uint16_t*>(base + L.hin_off);
    float* h_out = reinterpret_cast<float*>(base + L.hout_off);
    unsigned* round_flag = reinterpret_cast<unsigned*>(base + L.flag_off);
    void* lm_ws = base + L.lm_off;
    void* fwd_ws = base + L.fwd_off;
    // cleared by a kernel, not a memset: the caller may capture this call in a graph
    if (launch_fold_flag(nullptr, round_flag, s) != hipSuccess) return SD2_ERR_HIP;
    for (int32_t i = 0; i < k; ++i) {
        // step i: the window so far goes through the stack, the head reads its last position
        if (launch_embed_window(emb, vocab, sh.hidden, start_token, draft_ids, i + 1, h_in, s) != hipSuccess) return SD2_ERR_HIP;
        rc = forward_impl(model, h_in, i + 1, h_out, fwd_ws, L.fwd_bytes, nullptr, stream);
        if (rc != SD2_OK) return rc;
        MegaGeo geo[4];
        if (plan_mega_path(model, i + 1, geo)) {  // keep a give-up flag beyond the next forward's set-up
            const MegaLayout ML = planned_layout(model, i + 1, geo);
            if (launch_fold_flag(reinterpret_cast<const unsigned*>(static_cast<uint8_t*>(fwd_ws) + ML.err_off), round_flag, s) !=
                hipSuccess)
                return SD2_ERR_HIP;
        }
        if (launch_lm_head(emb, h_out + (size_t)i * sh.hidden, vocab, sh.hidden, 1, lm_ws, draft_ids + i, nullptr, nullptr,
                           s) != hipSuccess)
            return SD2_ERR_HIP;
    }
    return SD2_OK;
}

int sd2_draft_round_status(const sd2_model_t* model, int32_t vocab, int32_t k, const void* ws, void* stream) {
    RoundLayout L;
    const int rc = round_layout(model, vocab, k, &L);
    if (rc != SD2_OK) return rc;
    if (!ws) return SD2_ERR_NULL;
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return SD2_ERR_HIP;
    unsigned flag = 0;
    if (hipMemcpy(&flag, static_cast<const uint8_t*>(ws) + L.flag_off, sizeof(flag), hipMemcpyDeviceToHost) != hipSuccess)
        return SD2_ERR_HIP;
    return (flag & 1u) ? SD2_ERR_TIMEOUT : ((flag & 2u) ? SD2_ERR_RANGE : SD2_OK);
}

// ---- the round against a key/value cache: k single-token decode steps

namespace {
int cached_round_layout(const sd2_model_t* md, int32_t vocab, int32_t k, RoundLayout* L) {
    if (!md) return SD2_ERR_NULL;
    if (k < 1 || k > SD2_MAX_TOKENS) return SD2_ERR_RANGE;
    const sd2_model_shape_t& sh = md->shape;
    int rc = lm_head_check(vocab, sh.hidden, 1);
    if (rc != SD2_OK) return rc;
    L->hin_off = 0;
    L->hout_off = align256((size_t)sh.hidden * sizeof(uint16_t));
    L->flag_off = L->hout_off + align256((size_t)sh.hidden * sizeof(float));
    L->lm_off = L->flag_off + 256;
    L->fwd_off = L->lm_off + align256((size_t)kLmMaxWorkgroups * 16 * 8);
    L->fwd_bytes = decode_layout(md, 1).total;
    L->total = L->fwd_off + align256(L->fwd_bytes);
    return SD2_OK;
}
}  // namespace

int sd2_draft_round_cached_workspace_size(const sd2_model_t* model, int32_t vocab, int32_t k, size_t* bytes_out) {
    if (!bytes_out) return SD2_ERR_NULL;
    RoundLayout L;
    const int rc = cached_round_layout(model, vocab, k, &L);
    if (rc != SD2_OK) return rc;
    *bytes_out = L.total;
    return SD2_OK;
}

int sd2_draft_round_cached(const sd2_model_t* model, const uint16_t* emb, int32_t vocab, const int32_t* start_token, int32_t k,
                           int32_t pos0, uint16_t* k_cache, uint16_t* v_cache, int32_t max_pos, double rope_theta,
                           int32_t* draft_ids, void* ws, size_t ws_bytes, void* stream) {
    RoundLayout L;
    int rc = cached_round_layout(model, vocab, k, &L);
    if (rc != SD2_OK) return rc;
    if (!emb || !start_token || !draft_ids || !ws || !k_cache || !v_cache) return SD2_ERR_NULL;
    if (max_pos < 1 || pos0 < 0 || (int64_t)pos0 + k > max_pos || !(rope_theta > 1.0)) return SD2_ERR_RANGE;
    const sd2_model_shape_t& sh = model->shape;
    if (!cached_attention_supported(sh.n_heads, sh.n_kv, sh.head_dim, max_pos)) return SD2_ERR_UNSUPPORTED;
    if (!aligned16(emb) || !aligned16(ws) || !aligned16(k_cache) || !aligned16(v_cache) || ws_bytes < L.total)
        return SD2_ERR_BUFFER;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* base = static_cast<uint8_t*>(ws);
    uint16_t* h_in = reinterpret_cast<uint16_t*>(base + L.hin_off);
    float* h_out = reinterpret_cast<float*>(base + L.hout_off);
    unsigned* round_flag = reinterpret_cast<unsigned*>(base + L.flag_off);
    void* lm_ws = base + L.lm_off;
    void* dec_ws = base + L.fwd_off;
    MegaGeo geo1[4];
    const bool single_launch = decode_layout(model, 1).chunks > 0 && plan_mega_path(model, 1, geo1);
    MegaLayout ML;
    memset(&ML, 0, sizeof(ML));
    if (single_launch) ML = planned_layout(model, 1, geo1);
    if (launch_fold_flag(nullptr, round_flag, s) != hipSuccess) return SD2_ERR_HIP;
    for (int32_t i = 0; i < k; ++i) {
        // step i: one token (the start token, then the one chosen at step i - 1) at position pos0 + i
        if (launch_embed_window(emb, vocab, sh.hidden, i == 0 ? start_token : draft_ids + (i - 1), nullptr, 1, h_in, s) != hipSuccess)
            return SD2_ERR_HIP;
        rc = sd2_sparse_drafter_decode(model, h_in, 1, pos0 + i, k_cache, v_cache, max_pos, rope_theta, h_out, dec_ws, L.fwd_bytes,
                                       stream);
        if (rc != SD2_OK) return rc;
        if (single_launch &&
            launch_fold_flag(reinterpret_cast<const unsigned*>(static_cast<uint8_t*>(dec_ws) + ML.err_off), round_flag, s) != hipSuccess)
            return SD2_ERR_HIP;
        if (launch_lm_head(emb, h_out, vocab, sh.hidden, 1, lm_ws, draft_ids + i, nullptr, nullptr, s) != hipSuccess)
            return SD2_ERR_HIP;
    }
    return SD2_OK;
}

int sd2_draft_round_cached_status(const sd2_model_t* model, int32_t vocab, int32_t k, const void* ws, void* stream) {
    RoundLayout L;
    const int rc = cached_round_layout(model, vocab, k, &L);
    if (rc != SD2_OK) return rc;
    if (!ws) return SD2_ERR_NULL;
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return SD2_ERR_HIP;
    unsigned flag = 0;
    if (hipMemcpy(&flag, static_cast<const uint8_t*>(ws) + L.flag_off, sizeof(flag), hipMemcpyDeviceToHost) != hipSuccess)
        return SD2_ERR_HIP;
    return (flag & 1u) ? SD2_ERR_TIMEOUT : ((flag & 2u) ? SD2_ERR_RANGE : SD2_OK);
}

}  // extern "C"
