"""Helpers for the GPU parity tests: torch owns device memory, the library does the work."""
import numpy as np
import torch

import paper_2504_08838_amd as sd2


def dev(a: np.ndarray) -> torch.Tensor:
    """Upload a numpy array bit for bit (uint16 travels as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    if a.dtype == np.uint8:
        return torch.from_numpy(a).cuda()
    return torch.from_numpy(a).cuda()


def stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


class SparseMat:
    def __init__(self, w_bits, fmt=1):
        self.blob = sd2.pack_sparse(w_bits, fmt)
        self.blob_dev = dev(self.blob)
        self.m = sd2.matrix_init_sparse(self.blob, self.blob_dev.data_ptr())
        self.n_out, self.k_in = w_bits.shape


class DenseMat:
    def __init__(self, w_bits):
        self.w_dev = dev(w_bits)
        self.n_out, self.k_in = w_bits.shape
        self.m = sd2.matrix_init_dense(self.w_dev.data_ptr(), self.n_out, self.k_in)


def run_linear(mat, x_bits, sparse=True) -> np.ndarray:
    k_tok = x_bits.shape[0]
    x = dev(x_bits)
    y = torch.full((k_tok, mat.n_out), float("nan"), dtype=torch.float32, device="cuda")
    ws_bytes = sd2.linear_workspace_size(mat.m, k_tok)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    fn = sd2.sparse_linear if sparse else sd2.dense_linear
    fn(mat.m, x.data_ptr(), k_tok, y.data_ptr(), ws.data_ptr(), ws_bytes, stream_ptr())
    torch.cuda.synchronize()
    return y.cpu().numpy()


def build_model(shape, weight_bits, sparse=True, n_layers=None, fmt=1):
    """shape: sd2_workload.StackShape-like; weight_bits(layer, proj) -> bf16 bits.  Returns (Model, keep-alive list)."""
    layers = shape.layers if n_layers is None else n_layers
    mats, keep = [], []
    for l in range(layers):
        fused = [
            np.concatenate([weight_bits(l, "q"), weight_bits(l, "k"), weight_bits(l, "v")], axis=0),
            weight_bits(l, "o"),
            np.concatenate([weight_bits(l, "gate"), weight_bits(l, "up")], axis=0),
            weight_bits(l, "down"),
        ]
        for w in fused:
            mat = SparseMat(w, fmt) if sparse else DenseMat(w)
            keep.append(mat)
            mats.append(mat.m)
    ms = sd2.ModelShape(layers, shape.hidden, shape.q_out, shape.kv_out, shape.inter, shape.n_heads, shape.n_kv,
                        shape.head_dim)
    return sd2.model_create(ms, mats, keep=keep)


def run_forward(model, h_in_bits, hidden) -> np.ndarray:
    k_tok = h_in_bits.shape[0]
    h_in = dev(h_in_bits)
    h_out = torch.full((k_tok, hidden), float("nan"), dtype=torch.float32, device="cuda")
    ws_bytes = sd2.drafter_workspace_size(model, k_tok)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    sd2.sparse_drafter_forward(model, h_in.data_ptr(), k_tok, h_out.data_ptr(), ws.data_ptr(), ws_bytes, stream_ptr())
    sd2.drafter_forward_status(model, k_tok, ws.data_ptr(), stream_ptr())  # waits; raises if a bounded wait ran out
    return h_out.cpu().numpy()


def run_forward_trace(model, h_in_bits, shape):
    """-> (h_out, x [n_lin][k][kmax] bf16 bits, src [n_lin][k][smax] fp32) from the step-recording forward."""
    k_tok = h_in_bits.shape[0]
    n_lin = 4 * shape.layers
    kmax = max(shape.hidden, shape.q_out, shape.inter)
    smax = max(shape.hidden, shape.q_out + 2 * shape.kv_out, 2 * shape.inter)
    h_in = dev(h_in_bits)
    h_out = torch.full((k_tok, shape.hidden), float("nan"), dtype=torch.float32, device="cuda")
    ws_bytes = sd2.drafter_workspace_size(model, k_tok)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    tb = sd2.drafter_trace_size(model, k_tok)
    trace = torch.zeros(tb, dtype=torch.uint8, device="cuda")
    sd2.sparse_drafter_forward_trace(model, h_in.data_ptr(), k_tok, h_out.data_ptr(), ws.data_ptr(), ws_bytes,
                                     trace.data_ptr(), tb, stream_ptr())
    torch.cuda.synchronize()
    raw = trace.cpu().numpy()
    x_bytes = n_lin * k_tok * kmax * 2
    src_off = (x_bytes + 255) // 256 * 256
    x = raw[:x_bytes].view(np.uint16).reshape(n_lin, k_tok, kmax)
    src = raw[src_off:src_off + n_lin * k_tok * smax * 4].view(np.float32).reshape(n_lin, k_tok, smax)
    return h_out.cpu().numpy(), x, src


def run_lm_head(w_dev, vocab, hidden, h: np.ndarray, want_logits=True):
    """-> (token ids int32 [k], max logit fp32 [k], logits fp32 [k][vocab] or None) through the C ABI."""
    k_tok = h.shape[0]
    h_dev = torch.from_numpy(np.ascontiguousarray(h, dtype=np.float32)).cuda()
    ids = torch.full((k_tok,), -7, dtype=torch.int32, device="cuda")
    mx = torch.full((k_tok,), float("nan"), dtype=torch.float32, device="cuda")
    logits = torch.full((k_tok, vocab), float("nan"), dtype=torch.float32, device="cuda") if want_logits else None
    ws_bytes = sd2.lm_head_workspace_size(vocab, hidden, k_tok)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    sd2.lm_head_argmax(w_dev.data_ptr(), vocab, hidden, h_dev.data_ptr(), k_tok, ids.data_ptr(), ws.data_ptr(), ws_bytes,
                       stream_ptr(), max_logit_ptr=mx.data_ptr(), logits_ptr=logits.data_ptr() if want_logits else 0)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), mx.cpu().numpy(), (logits.cpu().numpy() if want_logits else None)
