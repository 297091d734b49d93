"""One drafting round on the GPU (embedding rows -> stack -> LM head -> next token, k times) against the oracle.

The tokens are integers decided by floating point: the GPU's ids are compared with the oracle run teacher-forced on
the GPU's own earlier ids (so one near-tie cannot cascade), and each id must be the oracle's id or lie within the
fp32 error bound of the oracle's maximum logit at that step."""
from types import SimpleNamespace

import numpy as np
import pytest

import sd2_workload as wl
from oracle import draft_round as odr

pytestmark = pytest.mark.gpu


def _model(shape, seed, fmt=1, pattern="row"):
    import gpu_util as gu
    table = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(shape)}
    cache = {}

    def get(layer, proj):
        if (layer, proj) not in cache:
            cache[(layer, proj)] = wl.gen_weight(seed, layer, proj, table[proj][0], table[proj][1], 50, pattern=pattern)
        return cache[(layer, proj)]

    return get, gu.build_model(shape, get, sparse=True, fmt=fmt)


def _run_round(model, emb_dev, vocab, t_start, k):
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    start = torch.tensor([t_start], dtype=torch.int32, device="cuda")
    ids = torch.full((k,), -7, dtype=torch.int32, device="cuda")
    nb = sd2.draft_round_workspace_size(model, vocab, k)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    sd2.draft_round(model, emb_dev.data_ptr(), vocab, start.data_ptr(), k, ids.data_ptr(), ws.data_ptr(), nb, gu.stream_ptr())
    sd2.draft_round_status(model, vocab, k, ws.data_ptr(), gu.stream_ptr())
    return ids.cpu().numpy(), (start, ids, ws, nb)


def _check(shape, get, emb, t_start, ids):
    k = ids.size
    assert ((ids >= 0) & (ids < emb.shape[0])).all()
    ref_ids, ref_logits = odr.draft_round(shape, get, emb, t_start, k, forced=ids)
    for i in range(k):
        gap = ref_logits[i, ref_ids[i]] - ref_logits[i, ids[i]]
        assert 0 <= gap <= 5e-3 * np.abs(ref_logits[i]).max(), (i, ids[i], ref_ids[i], gap)
    return int((ids == ref_ids).sum())


@pytest.mark.parametrize("forward", ["single-launch", "multi-launch"])
@pytest.mark.parametrize("fmt,pattern", [(1, "row"), (3, "2:4")])
def test_round_matches_oracle(forward, fmt, pattern, monkeypatch):
    import gpu_util as gu
    if forward == "multi-launch":
        monkeypatch.setenv("SD2_FORWARD", "multi")
    else:
        monkeypatch.delenv("SD2_FORWARD", raising=False)
    shape = SimpleNamespace(layers=2, hidden=512, q_out=512, kv_out=256, inter=1024, n_heads=4, n_kv=2, head_dim=128)
    vocab, k = 3000, 5
    get, model = _model(shape, 78, fmt, pattern)
    emb = wl.gen_lm_head(78, vocab, shape.hidden)
    ids, _ = _run_round(model, gu.dev(emb), vocab, 17, k)
    assert _check(shape, get, emb, 17, ids) >= k - 1


def test_round_k1_and_k8_and_out_of_range_start():
    import gpu_util as gu
    shape = SimpleNamespace(layers=1, hidden=256, q_out=256, kv_out=128, inter=512, n_heads=2, n_kv=1, head_dim=128)
    vocab = 777
    get, model = _model(shape, 79)
    emb = wl.gen_lm_head(79, vocab, shape.hidden)
    emb_dev = gu.dev(emb)
    for k in (1, 8):
        ids, _ = _run_round(model, emb_dev, vocab, 5, k)
        _check(shape, get, emb, 5, ids)
    ids_hi, _ = _run_round(model, emb_dev, vocab, vocab + 100, 3)   # clamped to the last id
    ids_ok, _ = _run_round(model, emb_dev, vocab, vocab - 1, 3)
    assert np.array_equal(ids_hi, ids_ok)


def test_round_in_a_graph_replays_identically_and_feeds_verify():
    """Captured once, replayed three times with the start token changed in place; the drafts then go through
    sd2_greedy_verify against themselves (everything accepted) and against a target that differs at position 2."""
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    shape = SimpleNamespace(layers=2, hidden=512, q_out=512, kv_out=256, inter=1024, n_heads=4, n_kv=2, head_dim=128)
    vocab, k = 2000, 5
    get, model = _model(shape, 80)
    emb = wl.gen_lm_head(80, vocab, shape.hidden)
    emb_dev = gu.dev(emb)
    eager = {t: _run_round(model, emb_dev, vocab, t, k)[0] for t in (3, 1234)}
    start = torch.tensor([3], dtype=torch.int32, device="cuda")
    ids = torch.full((k,), -7, dtype=torch.int32, device="cuda")
    nb = sd2.draft_round_workspace_size(model, vocab, k)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        call = lambda sp: sd2.draft_round(model, emb_dev.data_ptr(), vocab, start.data_ptr(), k, ids.data_ptr(), ws.data_ptr(), nb, sp)
        call(stream.cuda_stream)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            call(torch.cuda.current_stream().cuda_stream)
        for t in (3, 1234, 3):
            start.fill_(t)
            ids.fill_(-7)
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(ids.cpu().numpy(), eager[t])
    drafts = ids.reshape(1, k).contiguous()
    target = torch.cat([drafts, torch.tensor([[9]], dtype=torch.int32, device="cuda")], dim=1).contiguous()
    acc = torch.empty(1, dtype=torch.int32, device="cuda")
    out = torch.empty((1, k + 1), dtype=torch.int32, device="cuda")
    sd2.greedy_verify(drafts.data_ptr(), target.data_ptr(), 1, k, vocab, acc.data_ptr(), out.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    assert acc.item() == k and out.cpu().numpy()[0, -1] == 9
    target[0, 2] = (target[0, 2] + 1) % vocab
    sd2.greedy_verify(drafts.data_ptr(), target.data_ptr(), 1, k, vocab, acc.data_ptr(), out.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    assert acc.item() == 2
