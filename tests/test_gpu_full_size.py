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
# they add up like a random walk.  The link-by-link part below is the contract; this bound only catches a broken run.
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
        for _ in range(3):
            h_out.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            outs.append(h_out.cpu().numpy().copy())
    for o in outs:
        assert np.isfinite(o).all()
        assert ol.rel_l2(o, ref) <= FULL_E2E_TOL
    # replays agree with the eager call up to the order of the float atomics (and the rounding flips that can follow)
    for o in outs[1:]:
        assert ol.rel_l2(o, outs[0]) <= FULL_E2E_TOL
