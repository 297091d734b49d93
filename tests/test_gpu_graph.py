"""The drafter forward under HIP graph replay: every replay must reproduce the eager result bit for bit,
with eager work and synchronisations in between (the forward records kernels only, no memset nodes)."""
from types import SimpleNamespace

import numpy as np
import pytest

import sd2_workload as wl

pytestmark = pytest.mark.gpu

SHAPE = SimpleNamespace(layers=2, hidden=512, q_out=512, kv_out=256, inter=1024, n_heads=4, n_kv=2, head_dim=128)


@pytest.mark.parametrize("path", ["single-launch", "multi-launch"])
def test_forward_graph_replays_match_eager(path, sd2_options):
    # both forward paths add partial results in a fixed order (the single-launch kernel sums the residual stream
    # with exact integer atomics), so a replay must reproduce the eager call bit for bit
    sd2_options.set("forward_multi", 1 if path == "multi-launch" else 0)
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    table = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(SHAPE)}
    get = lambda l, p: wl.gen_weight(16, l, p, table[p][0], table[p][1], 50)
    model = gu.build_model(SHAPE, get)
    k_tok = 5
    h_in = gu.dev(wl.gen_x(16, 0, "q", k_tok, SHAPE.hidden))
    h_out = torch.zeros((k_tok, SHAPE.hidden), dtype=torch.float32, device="cuda")
    nb = sd2.drafter_workspace_size(model, k_tok)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        sd2.sparse_drafter_forward(model, h_in.data_ptr(), k_tok, h_out.data_ptr(), ws.data_ptr(), nb, stream.cuda_stream)
        stream.synchronize()
        eager = h_out.cpu().numpy().copy()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            sd2.sparse_drafter_forward(model, h_in.data_ptr(), k_tok, h_out.data_ptr(), ws.data_ptr(), nb,
                                       torch.cuda.current_stream().cuda_stream)
        for i in range(4):
            h_out.fill_(float(i))            # eager work between replays, also proves the replay rewrites the output
            ws.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(h_out.cpu().numpy(), eager), i
