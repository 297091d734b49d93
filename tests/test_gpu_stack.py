"""Drafter stack through the C ABI against the oracle's glue, plus greedy verification (bit-exact)."""
from types import SimpleNamespace

import numpy as np
import pytest

import sd2_workload as wl
from oracle import linear as ol
from oracle import stack as os_
from oracle import verify as ov
from oracle.bf16 import f64_to_bits

pytestmark = pytest.mark.gpu
TOL = 1e-3

SMALL = SimpleNamespace(layers=3, hidden=512, q_out=512, kv_out=256, inter=1024, n_heads=4, n_kv=2, head_dim=128)


def _weights(shape, cfg, pct=50):
    table = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(shape)}
    cache = {}

    def get(layer, proj):
        if (layer, proj) not in cache:
            n, k = table[proj]
            cache[(layer, proj)] = wl.gen_weight(cfg, layer, proj, n, k, pct)
        return cache[(layer, proj)]
    return get


@pytest.mark.parametrize("k_tok,sparse", [(1, True), (5, True), (8, True), (5, False), (20, True)])
def test_small_stack_end_to_end(k_tok, sparse):
    import gpu_util as gu
    get = _weights(SMALL, 14)
    h_in = wl.gen_x(14, 0, "q", k_tok, SMALL.hidden)
    ref = os_.drafter_forward(SMALL, get, h_in)
    model = gu.build_model(SMALL, get, sparse=sparse)
    out = gu.run_forward(model, h_in, SMALL.hidden)
    assert ol.rel_l2(out, ref) <= TOL


def test_zero_layers_returns_input():
    import gpu_util as gu
    z = SimpleNamespace(**{**SMALL.__dict__, "layers": 0})
    h_in = wl.gen_x(14, 0, "q", 3, SMALL.hidden)
    model = gu.build_model(z, None)
    out = gu.run_forward(model, h_in, SMALL.hidden)
    assert np.array_equal(out, wl.bf16_bits_to_f32(h_in))


def test_teacher_forced_linears_on_oracle_activations():
    """Each linear group fed the oracle's own bf16 activations: the 1e-3 bar without compounding."""
    import gpu_util as gu
    get = _weights(SMALL, 14)
    h_in = wl.gen_x(14, 0, "q", 5, SMALL.hidden)
    trace = []
    os_.drafter_forward(SMALL, get, h_in, trace=trace)
    fused = {
        "qkv": lambda l: np.concatenate([get(l, "q"), get(l, "k"), get(l, "v")], axis=0),
        "o": lambda l: get(l, "o"),
        "gateup": lambda l: np.concatenate([get(l, "gate"), get(l, "up")], axis=0),
        "down": lambda l: get(l, "down"),
    }
    for layer, name, x_f64, y_ref in trace:
        mat = gu.SparseMat(fused[name](layer))
        y = gu.run_linear(mat, f64_to_bits(x_f64))
        assert ol.rel_l2(y, y_ref) <= TOL, (layer, name)


def test_greedy_verify_bit_exact():
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    for batch, k, stream in [(64, 5, 0), (1, 1, 1), (1000, 8, 2), (7, 0, 3)]:
        draft, target = wl.gen_verify(5, batch, k, 128256, 0.85, stream=stream)
        acc_ref, out_ref = ov.greedy_verify(draft, target, vocab=128256)
        d = gu.dev(draft) if k > 0 else torch.empty(0, dtype=torch.int32, device="cuda")
        t = gu.dev(target)
        acc = torch.full((batch,), -7, dtype=torch.int32, device="cuda")
        out = torch.full((batch, k + 1), -7, dtype=torch.int32, device="cuda")
        sd2.greedy_verify(d.data_ptr() if k > 0 else 0x10, t.data_ptr(), batch, k, 128256, acc.data_ptr(), out.data_ptr(),
                          gu.stream_ptr())
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy(), acc_ref)
        assert np.array_equal(out.cpu().numpy(), out_ref)


def test_greedy_verify_hand_cases(golden_dir):
    import os
    import torch
    import paper_2504_08838_amd as sd2
    import gpu_util as gu
    with open(os.path.join(golden_dir, "verify_hand_cases.txt")) as f:
        lines = [l for l in f if l.strip() and not l.startswith("#")]
    for line in lines:
        d, t, n, o = [[int(v) for v in p.split()] for p in line.split("|")]
        k = len(d)
        dd = gu.dev(np.array(d, dtype=np.int32).reshape(1, k)) if k else None
        tt = gu.dev(np.array(t, dtype=np.int32).reshape(1, k + 1))
        acc = torch.zeros(1, dtype=torch.int32, device="cuda")
        out = torch.zeros((1, k + 1), dtype=torch.int32, device="cuda")
        sd2.greedy_verify(dd.data_ptr() if k else 0, tt.data_ptr(), 1, k, 128256, acc.data_ptr(), out.data_ptr(), gu.stream_ptr())
        torch.cuda.synchronize()
        assert acc.cpu().tolist() == n and out.cpu().tolist() == [o]
