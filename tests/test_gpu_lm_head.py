"""LM head with greedy choice on the GPU against the oracle (Eq. 1; the head is the drafter's one dense linear).

Floating point decides an integer here.  The checks therefore split in three:
  * the logits themselves against the fp64 oracle (rel-L2 <= 1e-3, the bar of every linear);
  * the choice against the kernel's own fp32 logits: exactly numpy's first argmax of them, bit for bit;
  * the choice against the oracle's: equal, except where the oracle's own top two are closer than the fp32
    error bound -- then the chosen id must be one of those near-maximal ids.
"""
import numpy as np
import pytest

import sd2_workload as wl
from oracle import linear as ol
from oracle import lm_head as olm

pytestmark = pytest.mark.gpu

TOL = 1e-3


def _check(w_bits, h, ids, mx, logits, ref_ids, ref_logits):
    k_tok = h.shape[0]
    assert ids.shape == (k_tok,) and ids.dtype == np.int32
    if logits is not None:
        assert np.isfinite(logits).all()
        assert ol.rel_l2(logits, ref_logits) <= TOL
        # the integer decision, taken in the kernel's precision on both sides
        assert np.array_equal(ids, np.argmax(logits, axis=-1).astype(np.int32))
        assert np.array_equal(mx, logits[np.arange(k_tok), ids])
    # against the oracle: an id whose fp64 logit is within the error bound of the fp64 maximum
    scale = np.abs(ref_logits).max(axis=-1)
    for t in range(k_tok):
        gap = ref_logits[t, ref_ids[t]] - ref_logits[t, ids[t]]
        assert 0 <= gap <= 2e-3 * scale[t], (t, ids[t], ref_ids[t], gap)
        if gap > 0:
            continue
        assert ids[t] == ref_ids[t] or ref_logits[t, ids[t]] == ref_logits[t, ref_ids[t]]
    assert np.abs(mx - ref_logits[np.arange(k_tok), ids]).max() <= 2e-3 * scale.max()
    return int((ids == ref_ids).sum())


@pytest.mark.parametrize(
    "vocab,hidden,k_tok",
    [
        (1000, 1024, 5),    # ragged last strip
        (1000, 3072, 1),    # the drafting shape: one token, three chunks per wavefront
        (4099, 2048, 16),   # a full token block, odd vocabulary
        (20000, 1024, 5),   # several strips per workgroup
        (777, 640, 3),      # fewer column chunks than wavefronts
        (2048, 1152, 7),    # ragged column chunks (9 over 8 wavefronts)
        (513, 4096, 2),
        (300, 8192, 4),
        (200, 9216, 3),     # the widest supported hidden size
        (5, 128, 1),        # less than one strip, one chunk
        (1, 256, 2),
        (3000, 1024, 17),   # more than one token block: the head is streamed per 16 tokens
        (1500, 2048, 40),
    ],
)
def test_lm_head_matches_oracle(vocab, hidden, k_tok):
    import gpu_util as gu
    w_bits = wl.gen_lm_head(21, vocab, hidden)
    h = wl.gen_final_hidden(21, k_tok, hidden)
    ref_ids, ref_logits = olm.lm_head_argmax(w_bits, h)
    w_dev = gu.dev(w_bits)
    ids, mx, logits = gu.run_lm_head(w_dev, vocab, hidden, h, want_logits=True)
    same = _check(w_bits, h, ids, mx, logits, ref_ids, ref_logits)
    assert same >= k_tok - 1  # random logits: a near-tie at the top is rare
    # without the logits output nothing else changes
    ids2, mx2, _ = gu.run_lm_head(w_dev, vocab, hidden, h, want_logits=False)
    assert np.array_equal(ids, ids2) and np.array_equal(mx, mx2)


def test_exact_ties_take_the_lowest_index():
    """Copies of the winning row planted before and after it, in other strips and other workgroups."""
    import gpu_util as gu
    vocab, hidden, k_tok = 9000, 1024, 4
    w_bits = wl.gen_lm_head(22, vocab, hidden)
    h = wl.gen_final_hidden(22, k_tok, hidden)
    ref_ids, _ = olm.lm_head_argmax(w_bits, h)
    planted = {}
    for t in range(k_tok):
        r = int(ref_ids[t])
        lo, hi = (r * 7 + 13 * t) % max(r, 1), r + 1 + (t * 997 + 31) % (vocab - r - 1)
        if r == 0 or lo in planted or hi in planted or lo in ref_ids or hi in ref_ids:
            continue
        w_bits[lo] = w_bits[r]
        w_bits[hi] = w_bits[r]
        planted[lo] = planted[hi] = r
    assert planted
    ref_ids2, ref_logits2 = olm.lm_head_argmax(w_bits, h)
    ids, mx, logits = gu.run_lm_head(gu.dev(w_bits), vocab, hidden, h, want_logits=True)
    _check(w_bits, h, ids, mx, logits, ref_ids2, ref_logits2)
    assert np.array_equal(ids, ref_ids2)
    for t in range(k_tok):
        # identical rows give bit-identical fp32 logits: the tie is exact on the GPU too
        dup = [v for v, r in planted.items() if r == int(ref_ids[t])]
        for v in dup:
            assert logits[t, v] == logits[t, int(ref_ids[t])]
            assert ids[t] <= v


def test_all_equal_logits_choose_token_zero():
    import gpu_util as gu
    vocab, hidden, k_tok = 4000, 1024, 3
    w_bits = np.zeros((vocab, hidden), dtype=np.uint16)
    h = wl.gen_final_hidden(23, k_tok, hidden)
    ids, mx, logits = gu.run_lm_head(gu.dev(w_bits), vocab, hidden, h, want_logits=True)
    assert np.array_equal(ids, np.zeros(k_tok, dtype=np.int32))
    assert np.array_equal(mx, np.zeros(k_tok, dtype=np.float32)) and not logits.any()


def test_last_row_can_win():
    """The winner sits in the ragged last strip."""
    import gpu_util as gu
    vocab, hidden, k_tok = 4099, 1024, 2
    w_bits = wl.gen_lm_head(24, vocab, hidden)
    h = wl.gen_final_hidden(24, k_tok, hidden)
    a = olm.round_to_bf16(olm.rmsnorm(h.astype(np.float64)))
    # last row = 0.25 * sign(a[0]): its logit for token 0 is 0.25 * sum |a[0]|, far above the random rows
    w_bits[vocab - 1] = wl.f32_to_bf16_bits((0.25 * np.sign(a[0])).astype(np.float32))
    ref_ids, ref_logits = olm.lm_head_argmax(w_bits, h)
    assert ref_ids[0] == vocab - 1
    ids, mx, logits = gu.run_lm_head(gu.dev(w_bits), vocab, hidden, h, want_logits=True)
    _check(w_bits, h, ids, mx, logits, ref_ids, ref_logits)
    assert ids[0] == vocab - 1


def test_full_size_head_eager_and_graph_replays():
    """The 3B drafter's head (vocabulary 128256 x hidden 3072, k = 5) in the launch configuration bench.py times:
    captured in a HIP graph on a side stream, without the logits output; and once eagerly with it."""
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    shape = wl.CONFIGS[3]["shape"]
    vocab, hidden, k_tok = shape.vocab, shape.hidden, 5
    assert (vocab, hidden) == (128256, 3072)
    w_bits = wl.gen_lm_head(3, vocab, hidden)
    h = wl.gen_final_hidden(3, k_tok, hidden)
    ref_ids, ref_logits = olm.lm_head_argmax(w_bits, h)
    w_dev = gu.dev(w_bits)
    ids, mx, logits = gu.run_lm_head(w_dev, vocab, hidden, h, want_logits=True)
    _check(w_bits, h, ids, mx, logits, ref_ids, ref_logits)

    h_dev = torch.from_numpy(h).cuda()
    ids_dev = torch.full((k_tok,), -7, dtype=torch.int32, device="cuda")
    mx_dev = torch.full((k_tok,), float("nan"), dtype=torch.float32, device="cuda")
    ws_bytes = sd2.lm_head_workspace_size(vocab, hidden, k_tok)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()  # default priority
    with torch.cuda.stream(stream):
        call = lambda s: sd2.lm_head_argmax(w_dev.data_ptr(), vocab, hidden, h_dev.data_ptr(), k_tok, ids_dev.data_ptr(),
                                            ws.data_ptr(), ws_bytes, s, max_logit_ptr=mx_dev.data_ptr())
        call(stream.cuda_stream)  # loads the kernels before the capture
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            call(torch.cuda.current_stream().cuda_stream)
        for _ in range(3):
            ids_dev.fill_(-7)
            mx_dev.fill_(float("nan"))
            ws.fill_(0xFF)  # the workspace carries nothing from call to call
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(ids_dev.cpu().numpy(), ids)
            assert np.array_equal(mx_dev.cpu().numpy(), mx)
