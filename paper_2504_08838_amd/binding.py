"""ctypes binding of libsd2.so: argument marshalling only, same names as the C ABI.

Device pointers are plain integers (``tensor.data_ptr()``); ``stream`` is the raw
``hipStream_t`` value (``torch.cuda.current_stream().cuda_stream``) or 0.
The library is loaded from this directory and there is no fallback: a missing or
unloadable ``libsd2.so`` raises at import of the first call.
"""

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class SD2Error(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {strerror(status)} ({status})")


class BlobInfo(C.Structure):
    _fields_ = [
        ("format", C.c_int32), ("n_out", C.c_int32), ("k_in", C.c_int32),
        ("n_strips", C.c_int32), ("n_slabs", C.c_int32), ("n_tiles", C.c_int32),
        ("max_tile_nnz", C.c_int32), ("reserved0", C.c_int32),
        ("nnz", C.c_uint64), ("total_bytes", C.c_uint64), ("useful_bytes", C.c_uint64),
        ("mask_off", C.c_uint64), ("val_off", C.c_uint64),
        ("checksum", C.c_uint32), ("reserved", C.c_uint32),
    ]

    def asdict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_ if not n.startswith("reserved")}


class Matrix(C.Structure):
    _fields_ = [("kind", C.c_int32), ("reserved", C.c_int32), ("data_dev", C.c_void_p), ("info", BlobInfo)]


class ModelShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("layers", "hidden", "q_out", "kv_out", "inter", "n_heads", "n_kv", "head_dim")]


class Model:
    """Owns an sd2_model_t*; keeps the descriptors' device tensors alive via ``keep``."""

    def __init__(self, handle, keep=None):
        self.handle = handle
        self.keep = keep

    def close(self):
        if self.handle:
            lib().sd2_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def lib_path():
    return os.path.join(_HERE, "libsd2.so")


def lib():
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -m paper_2504_08838_amd.build` (there is no CPU fallback)")
        # One HIP runtime per process: torch ships its own copy, and streams and device pointers of one runtime
        # mean nothing to another.  Loading torch first makes libsd2 bind the runtime torch uses.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(path)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        psz = C.POINTER(C.c_size_t)
        pinfo, pmat = C.POINTER(BlobInfo), C.POINTER(Matrix)
        sig = {
            "sd2_strerror": (C.c_char_p, [C.c_int]),
            "sd2_version": (C.c_int, []),
            "sd2_set_option": (C.c_int, [i32, i32]),
            "sd2_get_option": (C.c_int, [i32, C.POINTER(C.c_int32)]),
            "sd2_pack_sparse_size": (C.c_int, [vp, i32, i32, i32, psz]),
            "sd2_pack_sparse": (C.c_int, [vp, i32, i32, i32, vp, sz, psz]),
            "sd2_unpack_sparse": (C.c_int, [vp, sz, vp, i32, i32]),
            "sd2_blob_info": (C.c_int, [vp, sz, pinfo]),
            "sd2_blob_validate": (C.c_int, [vp, sz]),
            "sd2_matrix_init_sparse": (C.c_int, [pmat, vp, sz, vp]),
            "sd2_matrix_init_dense": (C.c_int, [pmat, vp, i32, i32]),
            "sd2_linear_workspace_size": (C.c_int, [pmat, i32, psz]),
            "sd2_sparse_linear": (C.c_int, [pmat, vp, i32, vp, vp, sz, vp]),
            "sd2_sparse_linear_partials": (C.c_int, [pmat, vp, i32, vp, sz, vp]),
            "sd2_sparse_linear_static": (C.c_int, [pmat, vp, i32, vp, vp]),
            "sd2_static_scratch_bytes": (C.c_int, [psz]),
            "sd2_dense_linear": (C.c_int, [pmat, vp, i32, vp, vp, sz, vp]),
            "sd2_mlp_workspace_size": (C.c_int, [pmat, pmat, i32, psz]),
            "sd2_sparse_mlp_forward": (C.c_int, [pmat, pmat, vp, i32, vp, vp, sz, vp]),
            "sd2_model_create": (C.c_int, [C.POINTER(ModelShape), pmat, i32, C.POINTER(vp)]),
            "sd2_model_destroy": (C.c_int, [vp]),
            "sd2_drafter_workspace_size": (C.c_int, [vp, i32, psz]),
            "sd2_sparse_drafter_forward": (C.c_int, [vp, vp, i32, vp, vp, sz, vp]),
            "sd2_drafter_trace_size": (C.c_int, [vp, i32, psz]),
            "sd2_sparse_drafter_forward_trace": (C.c_int, [vp, vp, i32, vp, vp, sz, vp, sz, vp]),
            "sd2_greedy_verify": (C.c_int, [vp, vp, i32, i32, i32, vp, vp, vp]),
            "sd2_check_token_ids_host": (C.c_int, [vp, sz, i32]),
            "sd2_greedy_verify_host": (C.c_int, [vp, vp, i32, i32, i32, vp, vp]),
            "sd2_drafter_forward_status": (C.c_int, [vp, i32, vp, vp]),
            "sd2_calibration_copy": (C.c_int, [vp, vp, sz, vp]),
            "sd2_calibration_read": (C.c_int, [vp, sz, vp, vp]),
            "sd2_mask_gradient": (C.c_int, [vp, vp, i32, vp]),
            "sd2_improvement_factor": (C.c_int, [C.c_double, i32, C.c_double, C.POINTER(C.c_double)]),
            "sd2_draft_round_cached_workspace_size": (C.c_int, [vp, i32, i32, C.POINTER(sz)]),
            "sd2_draft_round_cached": (C.c_int, [vp, vp, i32, vp, i32, i32, vp, vp, i32, C.c_double, vp, vp, sz, vp]),
            "sd2_draft_round_cached_status": (C.c_int, [vp, i32, i32, vp, vp]),
            "sd2_drafter_decode_workspace_size": (C.c_int, [vp, i32, C.POINTER(sz)]),
            "sd2_drafter_decode_status": (C.c_int, [vp, i32, vp, vp]),
            "sd2_sparse_drafter_decode": (C.c_int, [vp, vp, i32, i32, vp, vp, i32, C.c_double, vp, vp, sz, vp]),
            "sd2_draft_round_workspace_size": (C.c_int, [vp, i32, i32, C.POINTER(sz)]),
            "sd2_draft_round": (C.c_int, [vp, vp, i32, vp, i32, vp, vp, sz, vp]),
            "sd2_draft_round_status": (C.c_int, [vp, i32, i32, vp, vp]),
            "sd2_prune_magnitude": (C.c_int, [vp, i32, i32, i32, i32, vp]),
            "sd2_lm_head_workspace_size": (C.c_int, [i32, i32, i32, C.POINTER(sz)]),
            "sd2_lm_head_argmax": (C.c_int, [vp, i32, i32, vp, i32, vp, vp, vp, vp, sz, vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _LIB = L
    return _LIB


def _check(status, where):
    if status != 0:
        raise SD2Error(status, where)


def _host_ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def strerror(status):
    return lib().sd2_strerror(int(status)).decode()


def version():
    return lib().sd2_version()


OPT_FORWARD_MULTI, OPT_LINEAR_PARTIALS, OPT_SPIN_LIMIT, OPT_MEGA_TIMING, OPT_FIXED_BITS = 0, 1, 2, 3, 4


def set_option(which, value):
    _check(lib().sd2_set_option(int(which), int(value)), "sd2_set_option")


def get_option(which):
    v = C.c_int32()
    _check(lib().sd2_get_option(int(which), C.byref(v)), "sd2_get_option")
    return v.value


def _w_host(w_bits):
    w = np.ascontiguousarray(w_bits, dtype=np.uint16)
    if w.ndim != 2:
        raise ValueError("w_bits must be [n_out][k_in]")
    return w


def pack_sparse_size(w_bits, fmt=0):
    w = _w_host(w_bits)
    n = C.c_size_t()
    _check(lib().sd2_pack_sparse_size(_host_ptr(w), w.shape[0], w.shape[1], fmt, C.byref(n)), "sd2_pack_sparse_size")
    return n.value


def pack_sparse(w_bits, fmt=0, out=None):
    """Returns the blob as a numpy uint8 array (host)."""
    w = _w_host(w_bits)
    if out is None:
        out = np.empty(pack_sparse_size(w, fmt), dtype=np.uint8)
    written = C.c_size_t()
    _check(lib().sd2_pack_sparse(_host_ptr(w), w.shape[0], w.shape[1], fmt, _host_ptr(out), out.nbytes,
                                 C.byref(written)), "sd2_pack_sparse")
    return out[:written.value]


def unpack_sparse(blob, n_out, k_in):
    b = np.ascontiguousarray(blob, dtype=np.uint8)
    w = np.empty((n_out, k_in), dtype=np.uint16)
    _check(lib().sd2_unpack_sparse(_host_ptr(b), b.nbytes, _host_ptr(w), n_out, k_in), "sd2_unpack_sparse")
    return w


def blob_info(blob):
    b = np.ascontiguousarray(blob, dtype=np.uint8)
    info = BlobInfo()
    _check(lib().sd2_blob_info(_host_ptr(b), b.nbytes, C.byref(info)), "sd2_blob_info")
    return info


def blob_validate(blob):
    b = np.ascontiguousarray(blob, dtype=np.uint8)
    _check(lib().sd2_blob_validate(_host_ptr(b), b.nbytes), "sd2_blob_validate")


def matrix_init_sparse(blob_host, blob_dev_ptr):
    b = np.ascontiguousarray(blob_host, dtype=np.uint8)
    m = Matrix()
    _check(lib().sd2_matrix_init_sparse(C.byref(m), _host_ptr(b), b.nbytes, C.c_void_p(blob_dev_ptr)),
           "sd2_matrix_init_sparse")
    return m


def matrix_init_dense(w_dev_ptr, n_out, k_in):
    m = Matrix()
    _check(lib().sd2_matrix_init_dense(C.byref(m), C.c_void_p(w_dev_ptr), n_out, k_in), "sd2_matrix_init_dense")
    return m


def linear_workspace_size(m, k_tok):
    n = C.c_size_t()
    _check(lib().sd2_linear_workspace_size(C.byref(m), k_tok, C.byref(n)), "sd2_linear_workspace_size")
    return n.value


def sparse_linear(m, x_ptr, k_tok, y_ptr, ws_ptr=0, ws_bytes=0, stream=0):
    _check(lib().sd2_sparse_linear(C.byref(m), C.c_void_p(x_ptr), k_tok, C.c_void_p(y_ptr), C.c_void_p(ws_ptr),
                                   ws_bytes, C.c_void_p(stream)), "sd2_sparse_linear")


def sparse_linear_static(m, x_ptr, k_tok, y_ptr, stream=0):
    _check(lib().sd2_sparse_linear_static(C.byref(m), C.c_void_p(x_ptr), k_tok, C.c_void_p(y_ptr), C.c_void_p(stream)),
           "sd2_sparse_linear_static")


def static_scratch_bytes():
    n = C.c_size_t()
    _check(lib().sd2_static_scratch_bytes(C.byref(n)), "sd2_static_scratch_bytes")
    return n.value


def sparse_linear_partials(m, x_ptr, k_tok, part_ptr, part_bytes, stream=0):
    _check(lib().sd2_sparse_linear_partials(C.byref(m), C.c_void_p(x_ptr), k_tok, C.c_void_p(part_ptr), part_bytes,
                                            C.c_void_p(stream)), "sd2_sparse_linear_partials")


def dense_linear(m, x_ptr, k_tok, y_ptr, ws_ptr=0, ws_bytes=0, stream=0):
    _check(lib().sd2_dense_linear(C.byref(m), C.c_void_p(x_ptr), k_tok, C.c_void_p(y_ptr), C.c_void_p(ws_ptr),
                                  ws_bytes, C.c_void_p(stream)), "sd2_dense_linear")


def mlp_workspace_size(gate_up, down, k_tok):
    n = C.c_size_t()
    _check(lib().sd2_mlp_workspace_size(C.byref(gate_up), C.byref(down), k_tok, C.byref(n)), "sd2_mlp_workspace_size")
    return n.value


def sparse_mlp_forward(gate_up, down, x_ptr, k_tok, y_ptr, ws_ptr, ws_bytes, stream=0):
    _check(lib().sd2_sparse_mlp_forward(C.byref(gate_up), C.byref(down), C.c_void_p(x_ptr), k_tok, C.c_void_p(y_ptr),
                                        C.c_void_p(ws_ptr), ws_bytes, C.c_void_p(stream)), "sd2_sparse_mlp_forward")


def model_create(shape, mats, keep=None):
    """shape: ModelShape; mats: sequence of Matrix (4 per layer: qkv, o, gate_up, down)."""
    arr = (Matrix * max(len(mats), 1))(*mats)
    handle = C.c_void_p()
    _check(lib().sd2_model_create(C.byref(shape), arr, len(mats), C.byref(handle)), "sd2_model_create")
    return Model(handle, keep)


def model_destroy(model):
    model.close()


def drafter_workspace_size(model, k_tok):
    n = C.c_size_t()
    _check(lib().sd2_drafter_workspace_size(model.handle, k_tok, C.byref(n)), "sd2_drafter_workspace_size")
    return n.value


def sparse_drafter_forward(model, h_in_ptr, k_tok, h_out_ptr, ws_ptr, ws_bytes, stream=0):
    _check(lib().sd2_sparse_drafter_forward(model.handle, C.c_void_p(h_in_ptr), k_tok, C.c_void_p(h_out_ptr),
                                            C.c_void_p(ws_ptr), ws_bytes, C.c_void_p(stream)),
           "sd2_sparse_drafter_forward")


def drafter_trace_size(model, k_tok):
    n = C.c_size_t()
    _check(lib().sd2_drafter_trace_size(model.handle, k_tok, C.byref(n)), "sd2_drafter_trace_size")
    return n.value


def sparse_drafter_forward_trace(model, h_in_ptr, k_tok, h_out_ptr, ws_ptr, ws_bytes, trace_ptr, trace_bytes, stream=0):
    _check(lib().sd2_sparse_drafter_forward_trace(model.handle, C.c_void_p(h_in_ptr), k_tok, C.c_void_p(h_out_ptr),
                                                  C.c_void_p(ws_ptr), ws_bytes, C.c_void_p(trace_ptr), trace_bytes,
                                                  C.c_void_p(stream)), "sd2_sparse_drafter_forward_trace")


def drafter_forward_status(model, k_tok, ws_ptr, stream=0):
    _check(lib().sd2_drafter_forward_status(model.handle, k_tok, C.c_void_p(ws_ptr), C.c_void_p(stream)),
           "sd2_drafter_forward_status")


def greedy_verify(draft_ptr, target_ptr, batch, k, vocab, accepted_ptr, out_tokens_ptr, stream=0):
    _check(lib().sd2_greedy_verify(C.c_void_p(draft_ptr), C.c_void_p(target_ptr), batch, k, vocab,
                                   C.c_void_p(accepted_ptr), C.c_void_p(out_tokens_ptr), C.c_void_p(stream)),
           "sd2_greedy_verify")


def greedy_verify_host(draft, target, vocab):
    """Host arrays draft [batch][k], target [batch][k+1] -> (accepted_len [batch], out_tokens [batch][k+1])."""
    d = np.ascontiguousarray(draft, dtype=np.int32)
    t = np.ascontiguousarray(target, dtype=np.int32)
    batch, k = t.shape[0], t.shape[1] - 1
    if d.shape != (batch, k):
        raise ValueError("draft must be [batch][k] for target [batch][k+1]")
    acc = np.empty(batch, dtype=np.int32)
    out = np.empty((batch, k + 1), dtype=np.int32)
    _check(lib().sd2_greedy_verify_host(_host_ptr(d), _host_ptr(t), batch, k, vocab, _host_ptr(acc), _host_ptr(out)),
           "sd2_greedy_verify_host")
    return acc, out


def lm_head_workspace_size(vocab, hidden, k_tok):
    n = C.c_size_t(0)
    _check(lib().sd2_lm_head_workspace_size(vocab, hidden, k_tok, C.byref(n)), "sd2_lm_head_workspace_size")
    return n.value


def lm_head_argmax(w_ptr, vocab, hidden, h_ptr, k_tok, token_ids_ptr, ws_ptr, ws_bytes, stream=0, max_logit_ptr=0,
                   logits_ptr=0):
    """Device pointers as integers; max_logit_ptr / logits_ptr 0 = not wanted."""
    _check(lib().sd2_lm_head_argmax(C.c_void_p(w_ptr), vocab, hidden, C.c_void_p(h_ptr), k_tok,
                                    C.c_void_p(token_ids_ptr), C.c_void_p(max_logit_ptr or None),
                                    C.c_void_p(logits_ptr or None), C.c_void_p(ws_ptr), ws_bytes, C.c_void_p(stream)),
           "sd2_lm_head_argmax")


def drafter_decode_workspace_size(model, k_tok):
    n = C.c_size_t(0)
    _check(lib().sd2_drafter_decode_workspace_size(model.handle, k_tok, C.byref(n)), "sd2_drafter_decode_workspace_size")
    return n.value


def drafter_decode_status(model, k_tok, ws_ptr, stream=0):
    _check(lib().sd2_drafter_decode_status(model.handle, k_tok, C.c_void_p(ws_ptr), C.c_void_p(stream)),
           "sd2_drafter_decode_status")


def sparse_drafter_decode(model, h_in_ptr, k_tok, pos0, k_cache_ptr, v_cache_ptr, max_pos, rope_theta, h_out_ptr, ws_ptr,
                          ws_bytes, stream=0):
    _check(lib().sd2_sparse_drafter_decode(model.handle, C.c_void_p(h_in_ptr), k_tok, pos0, C.c_void_p(k_cache_ptr),
                                           C.c_void_p(v_cache_ptr), max_pos, float(rope_theta), C.c_void_p(h_out_ptr),
                                           C.c_void_p(ws_ptr), ws_bytes, C.c_void_p(stream)),
           "sd2_sparse_drafter_decode")


def draft_round_workspace_size(model, vocab, k):
    n = C.c_size_t(0)
    _check(lib().sd2_draft_round_workspace_size(model.handle, vocab, k, C.byref(n)), "sd2_draft_round_workspace_size")
    return n.value


def draft_round(model, emb_ptr, vocab, start_token_ptr, k, draft_ids_ptr, ws_ptr, ws_bytes, stream=0):
    _check(lib().sd2_draft_round(model.handle, C.c_void_p(emb_ptr), vocab, C.c_void_p(start_token_ptr), k,
                                 C.c_void_p(draft_ids_ptr), C.c_void_p(ws_ptr), ws_bytes, C.c_void_p(stream)),
           "sd2_draft_round")


def draft_round_status(model, vocab, k, ws_ptr, stream=0):
    _check(lib().sd2_draft_round_status(model.handle, vocab, k, C.c_void_p(ws_ptr), C.c_void_p(stream)),
           "sd2_draft_round_status")


def draft_round_cached_workspace_size(model, vocab, k):
    n = C.c_size_t(0)
    _check(lib().sd2_draft_round_cached_workspace_size(model.handle, vocab, k, C.byref(n)),
           "sd2_draft_round_cached_workspace_size")
    return n.value


def draft_round_cached(model, emb_ptr, vocab, start_token_ptr, k, pos0, k_cache_ptr, v_cache_ptr, max_pos, rope_theta,
                       draft_ids_ptr, ws_ptr, ws_bytes, stream=0):
    _check(lib().sd2_draft_round_cached(model.handle, C.c_void_p(emb_ptr), vocab, C.c_void_p(start_token_ptr), k, pos0,
                                        C.c_void_p(k_cache_ptr), C.c_void_p(v_cache_ptr), max_pos, float(rope_theta),
                                        C.c_void_p(draft_ids_ptr), C.c_void_p(ws_ptr), ws_bytes, C.c_void_p(stream)),
           "sd2_draft_round_cached")


def draft_round_cached_status(model, vocab, k, ws_ptr, stream=0):
    _check(lib().sd2_draft_round_cached_status(model.handle, vocab, k, C.c_void_p(ws_ptr), C.c_void_p(stream)),
           "sd2_draft_round_cached_status")


def prune_magnitude(w_ptr, n_out, k_in, sparsity_pct, pattern=0, stream=0):
    """In place on the device; pattern 0 = per row, 1 = 2:4."""
    _check(lib().sd2_prune_magnitude(C.c_void_p(w_ptr), n_out, k_in, sparsity_pct, pattern, C.c_void_p(stream)),
           "sd2_prune_magnitude")


def mask_gradient(m, grad_ptr, grad_is_bf16, stream=0):
    _check(lib().sd2_mask_gradient(C.byref(m), C.c_void_p(grad_ptr), int(grad_is_bf16), C.c_void_p(stream)),
           "sd2_mask_gradient")


def calibration_copy(dst_ptr, src_ptr, nbytes, stream=0):
    _check(lib().sd2_calibration_copy(C.c_void_p(dst_ptr), C.c_void_p(src_ptr), nbytes, C.c_void_p(stream)),
           "sd2_calibration_copy")


def calibration_read(src_ptr, nbytes, sink_ptr, stream=0):
    _check(lib().sd2_calibration_read(C.c_void_p(src_ptr), nbytes, C.c_void_p(sink_ptr), C.c_void_p(stream)),
           "sd2_calibration_read")


def improvement_factor(mean_emitted, k, cost_ratio):
    """Eq. 3 on the host."""
    out = C.c_double(0.0)
    _check(lib().sd2_improvement_factor(float(mean_emitted), int(k), float(cost_ratio), C.byref(out)), "sd2_improvement_factor")
    return out.value


def check_token_ids_host(ids, vocab):
    a = np.ascontiguousarray(ids, dtype=np.int32)
    _check(lib().sd2_check_token_ids_host(_host_ptr(a), a.size, vocab), "sd2_check_token_ids_host")
