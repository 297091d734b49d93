"""Decode step with rotary embedding and a key/value cache on the GPU against the oracle.

Per call: the residuals (rel-L2 <= 1e-3, the bar of the stack) and the cache contents.  A cache entry is a bf16
decided by floating point (fp32 on the GPU, fp64 in the oracle): entries must be equal or neighbours, and
neighbours must be rare."""
from types import SimpleNamespace

import numpy as np
import pytest

import sd2_workload as wl
from oracle import decode as od
from oracle.bf16 import bits_to_f64
from oracle.linear import rel_l2

pytestmark = pytest.mark.gpu

THETA = 500000.0
SMALL = SimpleNamespace(layers=2, hidden=512, q_out=512, kv_out=256, inter=1024, n_heads=4, n_kv=2, head_dim=128)


def _model(shape, seed, fmt=1, pattern="row", sparse=True):
    import gpu_util as gu
    table = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(shape)}
    cache = {}

    def get(layer, proj):
        if (layer, proj) not in cache:
            cache[(layer, proj)] = wl.gen_weight(seed, layer, proj, table[proj][0], table[proj][1], 50, pattern=pattern)
        return cache[(layer, proj)]

    return get, gu.build_model(shape, get, sparse=sparse, fmt=fmt)


def _decode(model, shape, h_bits, kc_dev, vc_dev, max_pos, pos0, theta=THETA):
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    k_tok = h_bits.shape[0]
    h_in = gu.dev(h_bits)
    h_out = torch.full((k_tok, shape.hidden), float("nan"), dtype=torch.float32, device="cuda")
    nb = sd2.drafter_decode_workspace_size(model, k_tok)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    sd2.sparse_drafter_decode(model, h_in.data_ptr(), k_tok, pos0, kc_dev.data_ptr(), vc_dev.data_ptr(), max_pos, theta,
                              h_out.data_ptr(), ws.data_ptr(), nb, gu.stream_ptr())
    sd2.drafter_decode_status(model, k_tok, ws.data_ptr(), gu.stream_ptr())  # waits; raises if a bounded wait ran out
    return h_out.cpu().numpy()


def _cache_close(got_bits, want_bits):
    """bf16 bit patterns equal, or neighbours (one step apart, or both tiny) in at most 1 % of the entries.  Tiny: the
    single-launch kernel hands the q|k|v sums over in fixed point with 17 fraction bits, each slab block rounding its
    share by at most 2^-18, so an entry may sit 2^-16 from the oracle's whatever its size."""
    g, w = got_bits.astype(np.int64), want_bits.astype(np.int64)
    diff = g != w
    if not diff.any():
        return 0.0
    gv, wv = bits_to_f64(got_bits), bits_to_f64(want_bits)
    ok = (np.abs(g - w) <= 1) | (np.abs(gv - wv) <= 2.0 ** -8 * np.maximum(np.abs(wv), 1e-3) + 2.0 ** -16)
    assert ok[diff].all()
    frac = diff.mean()
    assert frac <= 0.01, frac
    return frac


@pytest.fixture(params=["single-launch", "multi-launch"])
def forward(request, sd2_options):
    """Both implementations: the persistent kernel with its attention step, and one launch per linear and glue step."""
    if request.param == "multi-launch":
        sd2_options.set("forward_multi", 1)
    else:
        sd2_options.set("forward_multi", 0)
    return request.param


@pytest.mark.parametrize("n_hist,k_tok", [(0, 1), (0, 5), (1, 1), (37, 5), (300, 8), (555, 1), (700, 16), (191, 3), (193, 8)])
def test_decode_matches_oracle(n_hist, k_tok, forward):
    import gpu_util as gu
    shape, max_pos = SMALL, 768
    get, model = _model(shape, 81)
    kc, vc = wl.gen_kv_history(81, shape.layers, shape.n_kv, max_pos, shape.head_dim, n_hist)
    h_bits = wl.gen_x(81, 0, "q", k_tok, shape.hidden)
    kc_dev, vc_dev = gu.dev(kc), gu.dev(vc)
    got = _decode(model, shape, h_bits, kc_dev, vc_dev, max_pos, n_hist)
    want = od.drafter_decode(shape, get, h_bits, kc, vc, n_hist, THETA)  # updates kc, vc
    assert rel_l2(got, want) <= 1e-3
    assert np.isfinite(got).all()
    kg = kc_dev.cpu().numpy().view(np.uint16)
    vg = vc_dev.cpu().numpy().view(np.uint16)
    # history and the positions after the call are untouched, bit for bit
    assert np.array_equal(kg[:, :, :n_hist], kc[:, :, :n_hist]) and np.array_equal(vg[:, :, :n_hist], vc[:, :, :n_hist])
    assert not kg[:, :, n_hist + k_tok:].any() and not vg[:, :, n_hist + k_tok:].any()
    _cache_close(kg[0, :, n_hist:n_hist + k_tok], kc[0, :, n_hist:n_hist + k_tok])  # layer 0: inputs are identical
    _cache_close(vg[0, :, n_hist:n_hist + k_tok], vc[0, :, n_hist:n_hist + k_tok])
    assert rel_l2(bits_to_f64(kg[:, :, n_hist:n_hist + k_tok]), bits_to_f64(kc[:, :, n_hist:n_hist + k_tok])) <= 4e-3
    assert rel_l2(bits_to_f64(vg[:, :, n_hist:n_hist + k_tok]), bits_to_f64(vc[:, :, n_hist:n_hist + k_tok])) <= 4e-3


def test_token_by_token_equals_one_call_on_the_device(forward):
    # five calls of one token leave the same cache and give the same residuals as one call of five tokens
    import gpu_util as gu
    shape, max_pos, n_hist = SMALL, 128, 40
    get, model = _model(shape, 82)
    kc, vc = wl.gen_kv_history(82, shape.layers, shape.n_kv, max_pos, shape.head_dim, n_hist)
    h_bits = wl.gen_x(82, 0, "q", 5, shape.hidden)
    k1, v1 = gu.dev(kc), gu.dev(vc)
    a = _decode(model, shape, h_bits, k1, v1, max_pos, n_hist)
    k2, v2 = gu.dev(kc), gu.dev(vc)
    b = np.concatenate([_decode(model, shape, h_bits[t:t + 1], k2, v2, max_pos, n_hist + t) for t in range(5)])
    assert rel_l2(b, a) <= 2e-5  # kernels pick other split counts for one token: summation order only
    ka, kb = k1.cpu().numpy().view(np.uint16), k2.cpu().numpy().view(np.uint16)
    va, vb = v1.cpu().numpy().view(np.uint16), v2.cpu().numpy().view(np.uint16)
    _cache_close(kb, ka)
    _cache_close(vb, va)


@pytest.mark.parametrize("fmt,pattern,sparse", [(3, "2:4", True), (1, "row", False)])
def test_decode_other_matrix_kinds(fmt, pattern, sparse, forward):
    import gpu_util as gu
    shape, max_pos, n_hist, k_tok = SMALL, 128, 50, 3
    get, model = _model(shape, 83, fmt, pattern, sparse)
    kc, vc = wl.gen_kv_history(83, shape.layers, shape.n_kv, max_pos, shape.head_dim, n_hist)
    h_bits = wl.gen_x(83, 0, "q", k_tok, shape.hidden)
    got = _decode(model, shape, h_bits, gu.dev(kc), gu.dev(vc), max_pos, n_hist)
    want = od.drafter_decode(shape, get, h_bits, kc, vc, n_hist, THETA)
    assert rel_l2(got, want) <= 1e-3


def test_grouped_heads_six_per_kv_head_and_other_theta():
    # the Qwen-1.5B grouping (12 query heads on 2 key/value heads) and its rotary base
    import gpu_util as gu
    shape = SimpleNamespace(layers=1, hidden=512, q_out=1536, kv_out=256, inter=1024, n_heads=12, n_kv=2, head_dim=128)
    max_pos, n_hist, k_tok = 256, 200, 4
    get, model = _model(shape, 84)
    kc, vc = wl.gen_kv_history(84, shape.layers, shape.n_kv, max_pos, shape.head_dim, n_hist)
    h_bits = wl.gen_x(84, 0, "q", k_tok, shape.hidden)
    got = _decode(model, shape, h_bits, gu.dev(kc), gu.dev(vc), max_pos, n_hist, theta=1.0e6)
    want = od.drafter_decode(shape, get, h_bits, kc, vc, n_hist, 1.0e6)
    assert rel_l2(got, want) <= 1e-3


@pytest.mark.parametrize("head_dim,n_heads,n_kv", [(64, 8, 2), (256, 2, 1), (64, 16, 2)])
def test_other_head_sizes(head_dim, n_heads, n_kv):
    import gpu_util as gu
    shape = SimpleNamespace(layers=1, hidden=512, q_out=n_heads * head_dim, kv_out=n_kv * head_dim, inter=1024,
                            n_heads=n_heads, n_kv=n_kv, head_dim=head_dim)
    max_pos, n_hist, k_tok = 192, 131, 3
    get, model = _model(shape, 87)
    kc, vc = wl.gen_kv_history(87, shape.layers, shape.n_kv, max_pos, shape.head_dim, n_hist)
    h_bits = wl.gen_x(87, 0, "q", k_tok, shape.hidden)
    kc_dev, vc_dev = gu.dev(kc), gu.dev(vc)
    got = _decode(model, shape, h_bits, kc_dev, vc_dev, max_pos, n_hist)
    want = od.drafter_decode(shape, get, h_bits, kc, vc, n_hist, THETA)
    assert rel_l2(got, want) <= 1e-3
    _cache_close(kc_dev.cpu().numpy().view(np.uint16)[0, :, n_hist:n_hist + k_tok], kc[0, :, n_hist:n_hist + k_tok])


def test_far_positions_keep_their_angles(forward):
    # position 8000: a float product pos * frequency would be off by 5e-4 rad; the table is built in double precision
    import gpu_util as gu
    shape = SimpleNamespace(layers=1, hidden=512, q_out=512, kv_out=256, inter=1024, n_heads=4, n_kv=2, head_dim=128)
    max_pos, n_hist, k_tok = 8192, 8000, 2
    get, model = _model(shape, 85)
    kc, vc = wl.gen_kv_history(85, shape.layers, shape.n_kv, max_pos, shape.head_dim, n_hist)
    h_bits = wl.gen_x(85, 0, "q", k_tok, shape.hidden)
    kc_dev, vc_dev = gu.dev(kc), gu.dev(vc)
    got = _decode(model, shape, h_bits, kc_dev, vc_dev, max_pos, n_hist)
    want = od.drafter_decode(shape, get, h_bits, kc, vc, n_hist, THETA)
    assert rel_l2(got, want) <= 1e-3
    frac = _cache_close(kc_dev.cpu().numpy().view(np.uint16)[0, :, n_hist:n_hist + k_tok], kc[0, :, n_hist:n_hist + k_tok])
    assert frac <= 0.01


def test_decode_in_a_graph_replays(forward):
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    shape, max_pos, n_hist, k_tok = SMALL, 128, 30, 2
    get, model = _model(shape, 86)
    kc, vc = wl.gen_kv_history(86, shape.layers, shape.n_kv, max_pos, shape.head_dim, n_hist)
    h_bits = wl.gen_x(86, 0, "q", k_tok, shape.hidden)
    kc_dev, vc_dev = gu.dev(kc), gu.dev(vc)
    eager = _decode(model, shape, h_bits, kc_dev, vc_dev, max_pos, n_hist)
    h_in = gu.dev(h_bits)
    h_out = torch.zeros((k_tok, shape.hidden), dtype=torch.float32, device="cuda")
    nb = sd2.drafter_decode_workspace_size(model, k_tok)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        sd2.sparse_drafter_decode(model, h_in.data_ptr(), k_tok, n_hist, kc_dev.data_ptr(), vc_dev.data_ptr(), max_pos, THETA,
                                  h_out.data_ptr(), ws.data_ptr(), nb, side.cuda_stream)  # warm-up outside the capture
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            sd2.sparse_drafter_decode(model, h_in.data_ptr(), k_tok, n_hist, kc_dev.data_ptr(), vc_dev.data_ptr(), max_pos,
                                      THETA, h_out.data_ptr(), ws.data_ptr(), nb, side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        h_out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = h_out.cpu().numpy()
        if forward == "multi-launch":
            assert np.array_equal(got, eager)
        else:  # the single-launch kernel sums its split-K parts with float atomics: the order varies from run to run
            assert rel_l2(got, eager) <= 1e-5


def test_bounded_wait_gives_up_and_recovers(sd2_options):
    """Failure handling of the single-launch path: with a spin limit of zero every grid barrier (the attention step's
    included) gives up at its first unsuccessful poll.  Every wavefront still runs to the end, the status call reports
    the step as invalid, and the next step on a fresh cache is right again."""
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    sd2_options.set("forward_multi", 0)
    shape, max_pos, n_hist, k_tok = SMALL, 128, 50, 3
    get, model = _model(shape, 88)
    kc, vc = wl.gen_kv_history(88, shape.layers, shape.n_kv, max_pos, shape.head_dim, n_hist)
    h_bits = wl.gen_x(88, 0, "q", k_tok, shape.hidden)
    h_in = gu.dev(h_bits)
    h_out = torch.zeros((k_tok, shape.hidden), dtype=torch.float32, device="cuda")
    nb = sd2.drafter_decode_workspace_size(model, k_tok)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    kc_bad, vc_bad = gu.dev(kc), gu.dev(vc)
    sd2_options.set("spin_limit", 0)
    sd2.sparse_drafter_decode(model, h_in.data_ptr(), k_tok, n_hist, kc_bad.data_ptr(), vc_bad.data_ptr(), max_pos, THETA,
                              h_out.data_ptr(), ws.data_ptr(), nb, gu.stream_ptr())
    with pytest.raises(sd2.SD2Error):
        sd2.drafter_decode_status(model, k_tok, ws.data_ptr(), gu.stream_ptr())
    sd2_options.set("spin_limit", -1)
    got = _decode(model, shape, h_bits, gu.dev(kc), gu.dev(vc), max_pos, n_hist)
    want = od.drafter_decode(shape, get, h_bits, kc, vc, n_hist, THETA)
    assert rel_l2(got, want) <= 1e-3
