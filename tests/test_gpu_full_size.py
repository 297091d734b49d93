"""The benchmark's own configuration at full size: 3B-shape stack, 28 layers, 50 % sparse, k = 5.

Link by link (every linear and every glue step of all 28 layers against the oracle on the GPU's own recorded
inputs, bar 1e-3 per linear), and end to end through the entry point and launch configuration that bench.py
times (the forward captured in a HIP graph on a side stream and replayed).
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import sd2_workload as wl
from oracle import linear as ol
from oracle import stack as os_

pytestmark = pytest.mark.gpu

# After 28 layers (112 bf16 re-rounding points) a handful of activations that sit within fp32 error of a rounding
# boundary round the other way than in the fp64 oracle; each such flip moves the output by ~1e-4 of its norm and
# they add up like a random walk.  Observed at 28 layers: 8.0e-3 (printed by the test below); the bound is 2.5 times
# that.  The link-by-link part below is the contract; this bound only catches a broken run.
FULL_E2E_TOL = 2e-2


@pytest.fixture(scope="module")
def cfg3():
    import gpu_util as gu
    shape = wl.CONFIGS[3]["shape"]
    jobs = [(l, p, n, k) for l in range(shape.layers) for p, n, k in wl.layer_matrix_shapes(shape)]
    with ThreadPoolExecutor(max_workers=16) as ex:
        mats = list(ex.map(lambda j: wl.gen_weight(3, j[0], j[1], j[2], j[3], 50), jobs))
    weights = {(l, p): w for (l, p, _, _), w in zip(jobs, mats)}
    get = lambda l, p: weights[(l, p)]
    h_in = wl.gen_x(3, 0, "q", 5, shape.hidden)
    return shape, get, h_in, gu.build_model(shape, get)


def test_cfg3_every_link_of_28_layers(cfg3):
    import gpu_util as gu
    from test_gpu_stack import _verify_steps
    shape, get, h_in, model = cfg3
    h_out, x, src = gu.run_forward_trace(model, h_in, shape)
    assert np.isfinite(h_out).all()
    _verify_steps(shape, get, h_in, h_out, x, src)


def test_cfg3_graph_replays_as_timed_by_the_benchmark(cfg3):
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    shape, get, h_in_bits, model = cfg3
    ref = os_.drafter_forward(shape, get, h_in_bits)

    k_tok = h_in_bits.shape[0]
    h_in = gu.dev(h_in_bits)
    h_out = torch.full((k_tok, shape.hidden), float("nan"), dtype=torch.float32, device="cuda")
    ws_bytes = sd2.drafter_workspace_size(model, k_tok)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()  # default priority
    outs = []
    with torch.cuda.stream(stream):
        sd2.sparse_drafter_forward(model, h_in.data_ptr(), k_tok, h_out.data_ptr(), ws.data_ptr(), ws_bytes,
                                   stream.cuda_stream)
        stream.synchronize()
        outs.append(h_out.cpu().numpy().copy())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            sd2.sparse_drafter_forward(model, h_in.data_ptr(), k_tok, h_out.data_ptr(), ws.data_ptr(), ws_bytes,
                                       torch.cuda.current_stream().cuda_stream)
        for _ in range(20):
            h_out.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            outs.append(h_out.cpu().numpy().copy())
    assert np.isfinite(outs[0]).all()
    err = ol.rel_l2(outs[0], ref)
    print(f"28-layer end-to-end rel-L2 against the fp64 oracle: {err:.3e}")
    assert err <= FULL_E2E_TOL
    # nothing in the forward depends on the order in which workgroups finish: every replay reproduces the eager
    # call bit for bit (partial results are added in a fixed order, the residual stream by exact integer adds)
    for i, o in enumerate(outs[1:]):
        assert np.array_equal(o.view(np.uint32), outs[0].view(np.uint32)), f"replay {i} differs from the eager call"


# ---- the decode step at full size (the configuration bench.py times: one token at position 428 of a 1024-slot cache)

THETA = 500000.0


def _decode_once(model, shape, h_bits, kc_dev, vc_dev, max_pos, pos0, graph=False):
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    k_tok = h_bits.shape[0]
    h_in = gu.dev(h_bits)
    h_out = torch.full((k_tok, shape.hidden), float("nan"), dtype=torch.float32, device="cuda")
    nb = sd2.drafter_decode_workspace_size(model, k_tok)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()  # default priority
    call = lambda sp: sd2.sparse_drafter_decode(model, h_in.data_ptr(), k_tok, pos0, kc_dev.data_ptr(), vc_dev.data_ptr(), max_pos,
                                                THETA, h_out.data_ptr(), ws.data_ptr(), nb, sp)
    outs = []
    with torch.cuda.stream(stream):
        call(stream.cuda_stream)
        sd2.drafter_decode_status(model, k_tok, ws.data_ptr(), stream.cuda_stream)
        outs.append(h_out.cpu().numpy().copy())
        if graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                call(torch.cuda.current_stream().cuda_stream)
            for _ in range(2):
                h_out.fill_(float("nan"))
                g.replay()
                sd2.drafter_decode_status(model, k_tok, ws.data_ptr(), stream.cuda_stream)
                outs.append(h_out.cpu().numpy().copy())
    return outs


@pytest.mark.parametrize("k_tok", [1, 5])
@pytest.mark.parametrize("forward", ["single-launch", "multi-launch"])
def test_cfg3_decode_two_layers_at_full_width(cfg3, k_tok, forward, sd2_options):
    """Full-size matrices, two layers, both implementations.  End to end through eight bf16 rounding points: the bar is
    the stack's end-to-end one (5e-3; a few activations within fp32 error of a rounding boundary round the other way
    than in the fp64 oracle, observed ~1e-3), the cache rows of the first layer are checked entry by entry."""
    import gpu_util as gu
    from oracle import decode as od
    from oracle.bf16 import bits_to_f64
    if forward == "multi-launch":
        sd2_options.set("forward_multi", 1)
    else:
        sd2_options.set("forward_multi", 0)
    shape, get, _, _ = cfg3
    two = wl.StackShape("two-layers", 2, shape.hidden, shape.q_out, shape.kv_out, shape.inter, shape.n_heads, shape.n_kv,
                        shape.head_dim, shape.vocab)
    model = gu.build_model(two, get)
    max_pos, pos0 = 1024, 428
    kc, vc = wl.gen_kv_history(3, 2, shape.n_kv, max_pos, shape.head_dim, pos0)
    kc_dev, vc_dev = gu.dev(kc), gu.dev(vc)
    h_bits = wl.gen_x(3, 1, "q", k_tok, shape.hidden)
    got = _decode_once(model, two, h_bits, kc_dev, vc_dev, max_pos, pos0)[0]
    want = od.drafter_decode(two, get, h_bits, kc, vc, pos0, THETA)
    assert ol.rel_l2(got, want) <= 5e-3
    kg = kc_dev.cpu().numpy().view(np.uint16)
    vg = vc_dev.cpu().numpy().view(np.uint16)
    sl = slice(pos0, pos0 + k_tok)
    assert np.array_equal(kg[:, :, :pos0], kc[:, :, :pos0]) and not kg[:, :, pos0 + k_tok:].any()
    assert ol.rel_l2(bits_to_f64(kg[:, :, sl]), bits_to_f64(kc[:, :, sl])) <= 4e-3
    assert ol.rel_l2(bits_to_f64(vg[:, :, sl]), bits_to_f64(vc[:, :, sl])) <= 4e-3
    assert (kg[0, :, sl] != kc[0, :, sl]).mean() <= 0.01 and (vg[0, :, sl] != vc[0, :, sl]).mean() <= 0.01


def test_cfg3_decode_28_layers_as_timed_by_the_benchmark(cfg3):
    import gpu_util as gu
    from oracle import decode as od
    shape, get, _, model = cfg3
    max_pos, pos0 = 1024, 428
    kc, vc = wl.gen_kv_history(3, shape.layers, shape.n_kv, max_pos, shape.head_dim, pos0)
    kc_dev, vc_dev = gu.dev(kc), gu.dev(vc)
    h_bits = wl.gen_x(3, 1, "q", 1, shape.hidden)
    outs = _decode_once(model, shape, h_bits, kc_dev, vc_dev, max_pos, pos0, graph=True)
    want = od.drafter_decode(shape, get, h_bits, kc, vc, pos0, THETA)
    for o in outs:
        assert np.isfinite(o).all()
        assert ol.rel_l2(o, want) <= FULL_E2E_TOL
    # The forward itself is order-independent, but a replay starts from the cache the call before it left: the step's
    # own key/value rows are rewritten with the same bits, so the replays agree bit for bit as well.
    for o in outs[1:]:
        assert np.array_equal(o.view(np.uint32), outs[0].view(np.uint32))
