#!/usr/bin/env python3
"""Headline benchmark: microseconds per sparse drafter forward (k = 5) on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input: the 28-layer,
3B-shape drafter linear stack at 50 % unstructured sparsity on k = 5 in-flight tokens
(sd2_sparse_drafter_forward), followed by greedy verification of a 64 x 5 batch of draft ids
(sd2_greedy_verify).  Inputs and packed weights are resident in HBM before the timed region.
Forward and verify are each captured once into a HIP graph and replayed K times; an event pair
on the same stream brackets every forward inside the timed region.

Prints one JSON line.  `value` is the step above and nothing else.  Beside it:
* `roofline`: the dominant kernel -- algorithmic bytes per launch divided by the live event-timed duration, against
  the published 8 TB/s of HBM3E (`traffic` = HBM bytes per launch measured with profiler counters in separate runs)
  and against a measured pure read stream of 2 GiB;
* `config.dense_stack_us`, `speedup_vs_dense`, `linears_only_us`: the same stack with the same masked weights stored
  densely, and every linear of the stack as an independent call (sparse and dense);
* `configs`: the other benchmark configurations, each with microseconds per call, useful and stored bytes, effective
  GB/s, fraction of peak and the dense kernel's time: the single 512 x 512 linear (latency-bound), the 1B-shape MLP
  block run cold over distinct matrices, the twelve cells of the 1.5B-shape stack, the wide regime (16/32/64 tokens);
* `cpu_baseline`: the NumPy fp64 oracle timed on the host's cores;
* further kernels timed on their own (`lm_head`, `draft_round`, `decode`, `draft_round_cached`, `nm24_linear`,
  `mask_gradient`).
"""

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
# HBM bytes per launch of the forward kernel (and of the gate+up sparse linear) from rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs, scaled by the plain copy kernel of --calibrate; None until measured.
MEASURED_TRAFFIC_BYTES = 3425351415
MEASURED_LINEAR_TRAFFIC_BYTES = 61258973
MEASURED_LM_HEAD_TRAFFIC_BYTES = 788238775
MEASURED_NM24_TRAFFIC_BYTES = 57259560
MEASURED_DECODE_TRAFFIC_BYTES = 3359744520
CALIBRATION_BYTES = 256 << 20  # size of the plain copies launched by --calibrate
STREAM_BYTES = 2 << 30         # the pure read stream that serves as the measured ceiling


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="3 = Llama-3B-shape stack (headline), 4 = Qwen-1.5B-shape")
    ap.add_argument("--sparsity", type=int, default=50)
    ap.add_argument("--k-tok", type=int, default=5)
    ap.add_argument("--pattern", default="row", choices=["row", "global"],
                    help="mask of the synthetic weights: per-row magnitude (headline) or one threshold per matrix (rows of unequal population)")
    ap.add_argument("--layers", type=int, default=0, help="debug: fewer layers (reported as such)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense bf16 stack and the linears-only comparison")
    ap.add_argument("--no-configs", action="store_true", help="skip the other benchmark configurations (`configs`)")
    ap.add_argument("--no-lm-head", action="store_true", help="skip the separately timed LM head, drafting rounds and decode step")
    ap.add_argument("--no-nm24", action="store_true", help="skip the separately timed 2:4 semi-structured gate+up linear")
    ap.add_argument("--nm24-stack", action="store_true", help="also time the whole stack with 2:4 matrices")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch three plain 256 MiB copies (reference dispatches for profiler HBM counters)")
    return ap.parse_args()


FUSED_GROUPS = (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))


def build_weights(shape, cfg_id, pcts, layers, workers, pattern="row"):
    """Per sparsity the per-layer fused bf16 matrices (qkv, o, gate_up, down) from the seed recipe.  The random draw
    of a matrix does not depend on the sparsity, so several sparsities share it and differ in the mask only."""
    import sd2_workload as wl

    table = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(shape)}
    mask_fn = wl.magnitude_mask_per_row if pattern == "row" else wl.magnitude_mask_global

    def one(job):
        layer, projs = job
        per_pct = {p: [] for p in pcts}
        for proj in projs:
            dense = wl.gen_weight_dense(cfg_id, layer, proj, table[proj][0], table[proj][1])
            for p in pcts:
                w = np.where(mask_fn(dense, p), dense, np.uint16(0)).astype(np.uint16)
                per_pct[p].append(w)
        return {p: (m[0] if len(m) == 1 else np.concatenate(m, axis=0)) for p, m in per_pct.items()}

    jobs = [(l, g) for l in range(layers) for g in FUSED_GROUPS]
    with ThreadPoolExecutor(max_workers=workers) as ex:
        done = list(ex.map(one, jobs))
    return {p: [d[p] for d in done] for p in pcts}


class Bench:
    """Shared state of one benchmark process: device, stream, small helpers."""

    def __init__(self, args):
        import torch
        import paper_2504_08838_amd as sd2
        import sd2_workload as wl

        self.torch, self.sd2, self.wl, self.args = torch, sd2, wl, args
        self.dev = torch.device("cuda:0")
        torch.cuda.set_device(self.dev)
        self.stream = torch.cuda.Stream()  # default priority
        self.workers = min(16, os.cpu_count() or 8)

    def to_dev(self, a):
        a = np.ascontiguousarray(a)
        return self.torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(self.dev)

    def pack_model(self, fused, shape, layers, sparse=True):
        """-> (model, descriptors, useful bytes, stored bytes); the model keeps its device tensors alive."""
        sd2, torch = self.sd2, self.torch
        keep, mats, useful, total = [], [], 0, 0
        if sparse:
            with ThreadPoolExecutor(max_workers=self.workers) as ex:
                blobs = list(ex.map(lambda w: sd2.pack_sparse(w, 1), fused))
            for blob in blobs:
                d = torch.from_numpy(blob).to(self.dev)
                keep.append(d)
                mats.append(sd2.matrix_init_sparse(blob, d.data_ptr()))
        else:
            for w in fused:
                d = self.to_dev(w)
                keep.append(d)
                mats.append(sd2.matrix_init_dense(d.data_ptr(), w.shape[0], w.shape[1]))
        for m in mats:
            useful += int(m.info.useful_bytes)
            total += int(m.info.total_bytes)
        ms = sd2.ModelShape(layers, shape.hidden, shape.q_out, shape.kv_out, shape.inter, shape.n_heads, shape.n_kv, shape.head_dim)
        return sd2.model_create(ms, mats, keep=keep), mats, useful, total

    def graph_us(self, call, reps, warm=3, graph=True):
        """Event-timed microseconds per call (list), the call captured once into a HIP graph and replayed."""
        torch, stream = self.torch, self.stream
        with torch.cuda.stream(stream):
            call(stream.cuda_stream)
            stream.synchronize()
            g = None
            if graph:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    call(torch.cuda.current_stream().cuda_stream)
                run = g.replay
            else:
                run = lambda: call(stream.cuda_stream)
            for _ in range(warm):
                run()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for e0, e1 in ev:
                e0.record(stream)
                run()
                e1.record(stream)
            stream.synchronize()
            del g
        return [e0.elapsed_time(e1) * 1e3 for e0, e1 in ev]

    def forward_us(self, model, shape, k_tok, reps, cfg_id=3):
        """Mean microseconds of sd2_sparse_drafter_forward on k_tok tokens (graph replays), output checked finite."""
        sd2, torch, wl = self.sd2, self.torch, self.wl
        h_in = self.to_dev(wl.gen_x(cfg_id, 0, "q", k_tok, shape.hidden))
        h_out = torch.empty((k_tok, shape.hidden), dtype=torch.float32, device=self.dev)
        nb = sd2.drafter_workspace_size(model, k_tok)
        ws = torch.empty(nb, dtype=torch.uint8, device=self.dev)
        us = self.graph_us(lambda sp: sd2.sparse_drafter_forward(model, h_in.data_ptr(), k_tok, h_out.data_ptr(), ws.data_ptr(), nb, sp), reps)
        sd2.drafter_forward_status(model, k_tok, ws.data_ptr(), self.stream.cuda_stream)
        assert torch.isfinite(h_out).all(), "non-finite drafter output"
        return float(np.mean(us))

    def linears_us(self, mats, layers, k_tok, fn, cfg_id=3):
        """Every linear of a stack as an independent call on its own seeded input, event-timed per kind; microseconds summed."""
        sd2, torch, wl, stream = self.sd2, self.torch, self.wl, self.stream
        tot = 0.0
        with torch.cuda.stream(stream):
            spp = stream.cuda_stream
            for kind in range(4):
                ms_k = [mats[4 * l + kind] for l in range(layers)]
                info = ms_k[0].info
                xk = self.to_dev(wl.gen_x(cfg_id, 0, ("q", "o", "gate", "down")[kind], k_tok, int(info.k_in)))
                yk = torch.empty((k_tok, int(info.n_out)), dtype=torch.float32, device=self.dev)
                wsb = max(sd2.linear_workspace_size(ms_k[0], k_tok), 16)
                wsk = torch.empty(wsb, dtype=torch.uint8, device=self.dev)
                best = None
                for rep in range(3):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    for m in ms_k:
                        fn(m, xk.data_ptr(), k_tok, yk.data_ptr(), wsk.data_ptr(), wsb, spp)
                    e1.record(stream)
                    stream.synchronize()
                    t = e0.elapsed_time(e1) * 1e3
                    best = t if best is None or (rep and t < best) else best
                tot += best
        return tot


def rate(nbytes, us):
    gbs = nbytes / us / 1e3
    return {"GBps": round(gbs, 1), "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)}


def other_configs(B, fused3, model3, mats3, dmodel3, dmats3, useful3, total3, layers3):
    """The benchmark's other configurations.  None of them enters `value`."""
    sd2, torch, wl, args = B.sd2, B.torch, B.wl, B.args
    out = []

    # --- config 1: one 512 x 512 linear, 50 %, one token.  0.29 MB: launch latency, not bandwidth.
    c1 = wl.CONFIGS[1]
    w1 = wl.gen_weight(1, 0, "q", c1["n_out"], c1["k_in"], c1["sparsity"])
    b1 = sd2.pack_sparse(w1, 1)
    b1_dev = torch.from_numpy(b1).to(B.dev)
    m1 = sd2.matrix_init_sparse(b1, b1_dev.data_ptr())
    w1_dev = B.to_dev(w1)
    d1 = sd2.matrix_init_dense(w1_dev.data_ptr(), c1["n_out"], c1["k_in"])
    x1 = B.to_dev(wl.gen_x(1, 0, "q", c1["k_tok"], c1["k_in"]))
    y1 = torch.empty((c1["k_tok"], c1["n_out"]), dtype=torch.float32, device=B.dev)
    ws1 = torch.empty(max(sd2.linear_workspace_size(m1, c1["k_tok"]), sd2.linear_workspace_size(d1, c1["k_tok"]), 16), dtype=torch.uint8, device=B.dev)
    us_s = float(np.median(B.graph_us(lambda sp: sd2.sparse_linear(m1, x1.data_ptr(), c1["k_tok"], y1.data_ptr(), ws1.data_ptr(), ws1.numel(), sp), 100)))
    us_d = float(np.median(B.graph_us(lambda sp: sd2.dense_linear(d1, x1.data_ptr(), c1["k_tok"], y1.data_ptr(), ws1.data_ptr(), ws1.numel(), sp), 100)))
    out.append({"config": 1, "what": "single sparse linear 512x512, 50 %, k=1", "us": round(us_s, 2), "dense_us": round(us_d, 2),
                "speedup_vs_dense": round(us_d / us_s, 3), "useful_bytes": int(m1.info.useful_bytes), "stored_bytes": int(m1.info.total_bytes),
                "bound": "launch latency: 0.3 MB is 0.04 us of traffic at peak, so GB/s says nothing here", **rate(int(m1.info.useful_bytes), us_s)})

    # --- config 2: the 1B-shape MLP block, 50 %, k = 5, cold: ten distinct blocks (566 MB packed, 1 GB dense), so that
    # no call finds its matrices in the last-level cache left by the call before
    c2 = wl.CONFIGS[2]
    n_blk = 10

    def gen2(i):
        gu = np.concatenate([wl.gen_weight(2, i, p, c2["inter"], c2["hidden"], c2["sparsity"]) for p in ("gate", "up")], axis=0)
        dn = wl.gen_weight(2, i, "down", c2["hidden"], c2["inter"], c2["sparsity"])
        return gu, dn, sd2.pack_sparse(gu, 1), sd2.pack_sparse(dn, 1)

    with ThreadPoolExecutor(max_workers=B.workers) as ex:
        blocks = list(ex.map(gen2, range(n_blk)))
    keep2, sp2, de2, useful2, stored2 = [], [], [], 0, 0
    for gu, dn, bgu, bdn in blocks:
        dg, dd = torch.from_numpy(bgu).to(B.dev), torch.from_numpy(bdn).to(B.dev)
        wg, wd = B.to_dev(gu), B.to_dev(dn)
        keep2 += [dg, dd, wg, wd]
        sp2.append((sd2.matrix_init_sparse(bgu, dg.data_ptr()), sd2.matrix_init_sparse(bdn, dd.data_ptr())))
        de2.append((sd2.matrix_init_dense(wg.data_ptr(), gu.shape[0], gu.shape[1]), sd2.matrix_init_dense(wd.data_ptr(), dn.shape[0], dn.shape[1])))
    useful2 = sum(int(a.info.useful_bytes) + int(b.info.useful_bytes) for a, b in sp2) // n_blk
    stored2 = sum(int(a.info.total_bytes) + int(b.info.total_bytes) for a, b in sp2) // n_blk
    x2 = B.to_dev(wl.gen_x(2, 0, "gate", c2["k_tok"], c2["hidden"]))
    y2 = torch.empty((c2["k_tok"], c2["hidden"]), dtype=torch.float32, device=B.dev)
    nb2 = max(sd2.mlp_workspace_size(sp2[0][0], sp2[0][1], c2["k_tok"]), sd2.mlp_workspace_size(de2[0][0], de2[0][1], c2["k_tok"]))
    ws2 = torch.empty(nb2, dtype=torch.uint8, device=B.dev)

    def cold(pairs):
        d = []
        with torch.cuda.stream(B.stream):
            for rep in range(3):
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * n_blk)]
                for i, (a, b) in enumerate(pairs):
                    ev[2 * i].record(B.stream)
                    sd2.sparse_mlp_forward(a, b, x2.data_ptr(), c2["k_tok"], y2.data_ptr(), ws2.data_ptr(), nb2, B.stream.cuda_stream)
                    ev[2 * i + 1].record(B.stream)
                B.stream.synchronize()
                if rep:
                    d += [ev[2 * i].elapsed_time(ev[2 * i + 1]) * 1e3 for i in range(n_blk)]
        return float(np.mean(d))

    us_s, us_d = cold(sp2), cold(de2)
    out.append({"config": 2, "what": f"1B-shape MLP block (gate|up 16384x2048, down 2048x8192), 50 %, k=5, cold over {n_blk} distinct blocks "
                                     "(sparse: 2 launches per call, gate|up with the gated product in its epilogue, then down; dense: 3)",
                "us": round(us_s, 2), "dense_us": round(us_d, 2), "speedup_vs_dense": round(us_d / us_s, 3), "useful_bytes": useful2,
                "stored_bytes": stored2, **rate(useful2, us_s)})
    del keep2, sp2, de2, blocks

    # --- config 4: the 1.5B-shape stack, 28 layers, 50 / 60 / 70 % x k = 1, 3, 5, 8, against the dense stack of the same shape
    c4 = wl.CONFIGS[4]
    shape4 = c4["shape"]
    fused4 = build_weights(shape4, 4, list(c4["sparsity"]), shape4.layers, B.workers)
    dmodel4, _, _, _ = B.pack_model(fused4[c4["sparsity"][0]], shape4, shape4.layers, sparse=False)
    dense4 = {k: B.forward_us(dmodel4, shape4, k, 10, cfg_id=4) for k in c4["k_tok"]}
    sd2.model_destroy(dmodel4)
    for pct in c4["sparsity"]:
        model4, _, useful4, stored4 = B.pack_model(fused4[pct], shape4, shape4.layers)
        for k in c4["k_tok"]:
            us = B.forward_us(model4, shape4, k, 30, cfg_id=4)
            out.append({"config": 4, "what": f"1.5B-shape stack, 28 layers, {pct} %, k={k}", "sparsity_pct": pct, "k_tok": k, "us": round(us, 1),
                        "dense_us": round(dense4[k], 1), "speedup_vs_dense": round(dense4[k] / us, 3), "useful_bytes": useful4,
                        "stored_bytes": stored4, **rate(useful4, us)})
        sd2.model_destroy(model4)
    del fused4

    # --- config 5: the 3B-shape stack on 16 / 32 / 64 tokens, sparse against dense: the whole stack and the linears alone
    for k in wl.CONFIGS[5]["k_tok"]:
        us_s = B.forward_us(model3, wl.CONFIGS[3]["shape"], k, 10)
        entry = {"config": 5, "what": f"3B-shape stack, {layers3} layers, 50 %, k={k} (wide regime)", "k_tok": k, "us": round(us_s, 1),
                 "useful_bytes": useful3, "stored_bytes": total3, **rate(useful3, us_s)}
        lin_s = B.linears_us(mats3, layers3, k, sd2.sparse_linear)
        entry["linears_only_us"] = {"sparse": round(lin_s, 1)}
        if dmodel3 is not None:
            us_d = B.forward_us(dmodel3, wl.CONFIGS[3]["shape"], k, 5)
            lin_d = B.linears_us(dmats3, layers3, k, sd2.dense_linear)
            entry.update({"dense_us": round(us_d, 1), "speedup_vs_dense": round(us_d / us_s, 3)})
            entry["linears_only_us"].update({"dense": round(lin_d, 1), "speedup": round(lin_d / lin_s, 3),
                                             **{"sparse_" + a: b for a, b in rate(useful3, lin_s).items()}})
        out.append(entry)
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the sparse drafter is replicated per GPU and requests are "
              "sharded across them, so there is no multi-GPU figure to report; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2504_08838_amd as sd2
    import sd2_workload as wl

    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(1)
    B = Bench(args)
    dev, stream, to_dev, workers = B.dev, B.stream, B.to_dev, B.workers

    cfg = wl.CONFIGS[args.config]
    shape = cfg["shape"]
    layers = args.layers or shape.layers
    k_tok, pct = args.k_tok, args.sparsity
    headline = args.config == 3 and layers == shape.layers and pct == 50 and k_tok == 5 and args.pattern == "row"

    t_setup = time.time()
    fused = build_weights(shape, args.config, [pct], layers, workers, args.pattern)[pct]
    model, mats, useful, total = B.pack_model(fused, shape, layers)
    ms = sd2.ModelShape(layers, shape.hidden, shape.q_out, shape.kv_out, shape.inter, shape.n_heads, shape.n_kv, shape.head_dim)

    h_in = to_dev(wl.gen_x(args.config, 0, "q", k_tok, shape.hidden))
    h_out = torch.empty((k_tok, shape.hidden), dtype=torch.float32, device=dev)
    ws_bytes = sd2.drafter_workspace_size(model, k_tok)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    vcfg = wl.CONFIGS[5]["verify"]
    draft_np, target_np = wl.gen_verify(5, vcfg["batch"], vcfg["k"], vcfg["vocab"], vcfg["alpha"])
    draft, target = to_dev(draft_np), to_dev(target_np)
    acc = torch.empty(vcfg["batch"], dtype=torch.int32, device=dev)
    out_tok = torch.empty((vcfg["batch"], vcfg["k"] + 1), dtype=torch.int32, device=dev)
    setup_s = time.time() - t_setup

    def fwd(sp):
        sd2.sparse_drafter_forward(model, h_in.data_ptr(), k_tok, h_out.data_ptr(), ws.data_ptr(), ws_bytes, sp)

    def ver(sp):
        sd2.greedy_verify(draft.data_ptr(), target.data_ptr(), vcfg["batch"], vcfg["k"], vcfg["vocab"],
                          acc.data_ptr(), out_tok.data_ptr(), sp)

    # A step is forward + verify.  Each half is captured into a HIP graph of its own so that an event pair
    # recorded on the same stream brackets the forward inside the timed region: the forward is one persistent
    # kernel (plus a tiny set-up launch), and that pair is the live duration the roofline entry uses.
    use_graph = not args.no_graph
    with torch.cuda.stream(stream):
        sp = stream.cuda_stream
        fwd(sp)
        ver(sp)
        stream.synchronize()
        if use_graph:
            g_fwd, g_ver = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_fwd, stream=stream):
                fwd(torch.cuda.current_stream().cuda_stream)
            with torch.cuda.graph(g_ver, stream=stream):
                ver(torch.cuda.current_stream().cuda_stream)
            run_fwd, run_ver = g_fwd.replay, g_ver.replay
        else:
            run_fwd, run_ver = (lambda: fwd(sp)), (lambda: ver(sp))
        for _ in range(args.warmup):
            run_fwd()
            run_ver()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for e0, e1 in evs:
            e0.record(stream)
            run_fwd()
            e1.record(stream)
            run_ver()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    us_per_step = wall / args.steps * 1e6
    fwd_all = np.array([e0.elapsed_time(e1) for e0, e1 in evs]) * 1e3
    fwd_us = float(fwd_all.mean())
    fwd_p10, fwd_p50, fwd_p90 = (float(np.percentile(fwd_all, q)) for q in (10, 50, 90))

    # sanity: no bounded wait ran out, the output of the timed configuration is finite, the verify result plausible
    sd2.drafter_forward_status(model, k_tok, ws.data_ptr(), stream.cuda_stream)
    h_host = h_out.cpu().numpy()
    assert np.isfinite(h_host).all(), "non-finite drafter output"
    acc_host = acc.cpu().numpy()
    assert acc_host.min() >= 0 and acc_host.max() <= vcfg["k"]

    # --- roofline of the dominant kernel.  With the single-launch forward that kernel is the whole stack:
    # algorithmic bytes = every matrix's useful bytes (2 B per nonzero + 1 mask bit per weight) plus the
    # activations each linear reads (bf16) and the sums it produces (fp32).
    # the single-launch kernel serves up to 8 tokens (and is switched off by SD2_FORWARD=multi)
    forward_path = "multi" if (sd2.get_option(sd2.OPT_FORWARD_MULTI) or k_tok > 8) else "single-launch"
    act_bytes = 0
    for m in mats:
        act_bytes += 2 * k_tok * int(m.info.k_in) + 4 * k_tok * int(m.info.n_out)
    fwd_alg_bytes = useful + act_bytes
    fwd_achieved = fwd_alg_bytes / fwd_us / 1e3  # GB/s

    # --- the stand-alone sparse linear kernel on the largest matrix (fused gate+up), timed per launch with
    # events on the stream it runs on, over the distinct layers (each launch streams a different matrix).
    gu = [mats[4 * l + 2] for l in range(layers)]
    x_act = to_dev(wl.gen_x(args.config, 0, "gate", k_tok, shape.hidden))
    part = torch.empty(max(sd2.linear_workspace_size(gu[0], k_tok), 16), dtype=torch.uint8, device=dev)
    durs, durs_part = [], []
    y_lin = torch.empty((k_tok, int(gu[0].info.n_out)), dtype=torch.float32, device=dev)
    with torch.cuda.stream(stream):
        sp = stream.cuda_stream
        for rep in range(3):
            evl = [torch.cuda.Event(enable_timing=True) for _ in range(2 * layers)]
            for l in range(layers):
                evl[2 * l].record(stream)
                # final results in one launch (the slabs are added up inside the workgroup)
                sd2.sparse_linear(gu[l], x_act.data_ptr(), k_tok, y_lin.data_ptr(), part.data_ptr(), part.numel(), sp)
                evl[2 * l + 1].record(stream)
            stream.synchronize()
            if rep:
                durs += [evl[2 * l].elapsed_time(evl[2 * l + 1]) * 1e3 for l in range(layers)]
        for rep in range(3):
            evl = [torch.cuda.Event(enable_timing=True) for _ in range(2 * layers)]
            for l in range(layers):
                evl[2 * l].record(stream)
                # the older kernel: one partial result per slab, added up by whatever kernel comes next
                sd2.sparse_linear_partials(gu[l], x_act.data_ptr(), k_tok, part.data_ptr(), part.numel(), sp)
                evl[2 * l + 1].record(stream)
            stream.synchronize()
            if rep:
                durs_part += [evl[2 * l].elapsed_time(evl[2 * l + 1]) * 1e3 for l in range(layers)]
        # the same per-slab kernel with the multiply on the vector ALU (packed bf16 dot products) instead of the matrix cores
        durs_valu = []
        sd2.set_option(sd2.OPT_LINEAR_PARTIALS, 2)
        if k_tok <= 8:
            for rep in range(3):
                evl = [torch.cuda.Event(enable_timing=True) for _ in range(2 * layers)]
                for l in range(layers):
                    evl[2 * l].record(stream)
                    sd2.sparse_linear_partials(gu[l], x_act.data_ptr(), k_tok, part.data_ptr(), part.numel(), sp)
                    evl[2 * l + 1].record(stream)
                stream.synchronize()
                if rep:
                    durs_valu += [evl[2 * l].elapsed_time(evl[2 * l + 1]) * 1e3 for l in range(layers)]
        sd2.set_option(sd2.OPT_LINEAR_PARTIALS, 0)
        if args.calibrate:
            # plain copies of known size: the scale for the profiler's HBM counters
            cal_src = torch.empty(CALIBRATION_BYTES, dtype=torch.uint8, device=dev).fill_(1)
            cal_dst = torch.empty_like(cal_src)
            for _ in range(3):
                sd2.calibration_copy(cal_dst.data_ptr(), cal_src.data_ptr(), CALIBRATION_BYTES, sp)
            stream.synchronize()
            del cal_src, cal_dst
    kern_us, part_us = float(np.mean(durs)), float(np.mean(durs_part))
    gi = gu[0].info
    alg_bytes = int(gi.useful_bytes) + 2 * k_tok * gi.k_in + 4 * k_tok * gi.n_out
    achieved = alg_bytes / kern_us / 1e3  # GB/s

    # --- measured ceiling: a pure read stream of 2 GiB (more than the last-level cache holds), event-timed per launch
    src = torch.empty(STREAM_BYTES, dtype=torch.uint8, device=dev).fill_(3)
    sink = torch.empty(2048, dtype=torch.int32, device=dev)
    rd = B.graph_us(lambda spp: sd2.calibration_read(src.data_ptr(), STREAM_BYTES, sink.data_ptr(), spp), 10, graph=False)
    stream_gbs = STREAM_BYTES / float(np.mean(rd)) / 1e3
    del src

    single = forward_path != "multi"
    record = {
        "metric": f"us per sparse drafter forward (k={args.k_tok}) and effective HBM GB/s vs peak",
        "value": round(us_per_step, 2),
        "unit": "us",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(us_per_step / 1e3, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{shape.name} drafter linear stack, {layers} layers, {pct}% unstructured sparse bf16, "
                        f"k={k_tok} tokens + greedy verify batch {vcfg['batch']} k={vcfg['k']}",
            "config_id": args.config,
            "mask_pattern": args.pattern,
            "hip_graph": use_graph,
            "forward_path": forward_path,
            "forward_us": round(fwd_us, 2),
            "forward_us_p10_p50_p90": [round(fwd_p10, 2), round(fwd_p50, 2), round(fwd_p90, 2)],
            "packed_useful_bytes": useful,
            "packed_total_bytes": total,
            "effective_GBps": round(useful / us_per_step / 1e3, 1),
            "effective_frac_of_peak": round(useful / us_per_step / 1e3 / HBM_PEAK_GBS, 4),
            "setup_s": round(setup_s, 1),
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "mega_forward_kernel (whole stack, one launch)" if single else "forward (multi-launch)",
            "achieved": round(fwd_achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(fwd_achieved / HBM_PEAK_GBS, 4),
            "traffic": MEASURED_TRAFFIC_BYTES if (single and headline) else None,
            "kernel_us": round(fwd_us, 2),
            "algorithmic_bytes": fwd_alg_bytes,
            "measured_read_stream_GBps": round(stream_gbs, 1),
            "measured_read_stream_what": f"pure read of {STREAM_BYTES >> 20} MiB (sd2_calibration_read), event-timed",
            "frac_of_measured_stream": round(fwd_achieved / stream_gbs, 4),
            "linear_kernel": {
                "kernel": f"sparse_strip_kernel (fused gate+up, {gi.n_out}x{gi.k_in}, final results in one launch)",
                "achieved": round(achieved, 1),
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "kernel_us": round(kern_us, 2),
                "algorithmic_bytes": alg_bytes,
                "traffic": MEASURED_LINEAR_TRAFFIC_BYTES if headline else None,
                "partials_kernel_us": round(part_us, 2),
                "partials_kernel_vector_alu_us": round(float(np.mean(durs_valu)), 2) if durs_valu else None,
            },
        },
    }

    # --- the same stack with the same masked weights stored densely (the hand-written dense bf16 baseline), and every
    # linear of the stack as an independent call without any glue: sparse against dense, like for like
    dmodel = dmats = None
    if not args.no_dense:
        dmodel, dmats, _, _ = B.pack_model(fused, shape, layers, sparse=False)
        dense_us = B.forward_us(dmodel, shape, k_tok, max(args.steps // 8, 10), cfg_id=args.config)
        record["config"]["dense_stack_us"] = round(dense_us, 2)
        record["config"]["dense_stack_path"] = "multi-launch (the single-launch kernel is written for the packed format)"
        record["config"]["speedup_vs_dense"] = round(dense_us / fwd_us, 3)
        sd2.set_option(sd2.OPT_FORWARD_MULTI, 1)  # the sparse stack on the dense stack's launch structure
        try:
            multi_us = B.forward_us(model, shape, k_tok, max(args.steps // 8, 10), cfg_id=args.config)
        finally:
            sd2.set_option(sd2.OPT_FORWARD_MULTI, 0)
        record["config"]["sparse_stack_multi_launch_us"] = round(multi_us, 2)
        record["config"]["speedup_vs_dense_same_launch_structure"] = round(dense_us / multi_us, 3)
        sp_lin = B.linears_us(mats, layers, k_tok, sd2.sparse_linear, cfg_id=args.config)
        de_lin = B.linears_us(dmats, layers, k_tok, sd2.dense_linear, cfg_id=args.config)
        record["config"]["linears_only_us"] = {"sparse": round(sp_lin, 1), "dense": round(de_lin, 1), "speedup": round(de_lin / sp_lin, 3),
                                               **{"sparse_" + a: b for a, b in rate(useful, sp_lin).items()}}

    if not args.no_configs and headline:
        record["configs"] = other_configs(B, fused, model, mats, dmodel, dmats, useful, total, layers)

    if dmodel is not None:
        sd2.model_destroy(dmodel)
        dmodel = dmats = None

    if not args.no_lm_head:
        # The drafter's dense LM head with the final norm and the greedy choice fused in, timed on its own
        # (it is not part of `value`): one graph replay per call, an event pair around each.
        vocab = shape.vocab
        w_lm = to_dev(wl.gen_lm_head(args.config, vocab, shape.hidden))
        lm_ws_bytes = sd2.lm_head_workspace_size(vocab, shape.hidden, k_tok)
        lm_ws = torch.empty(lm_ws_bytes, dtype=torch.uint8, device=dev)
        lm = {}
        for kt in sorted({1, k_tok}):
            h_fin = torch.from_numpy(wl.gen_final_hidden(args.config, kt, shape.hidden)).to(dev)
            ids = torch.empty(kt, dtype=torch.int32, device=dev)
            us = float(np.mean(B.graph_us(lambda spp: sd2.lm_head_argmax(w_lm.data_ptr(), vocab, shape.hidden, h_fin.data_ptr(), kt,
                                                                        ids.data_ptr(), lm_ws.data_ptr(), lm_ws_bytes, spp), 30)))
            lm_bytes = 2 * vocab * shape.hidden + 4 * kt * shape.hidden + 8 * kt
            lm[f"k{kt}"] = {"us": round(us, 2), "achieved_GBps": round(lm_bytes / us / 1e3, 1),
                            "frac": round(lm_bytes / us / 1e3 / HBM_PEAK_GBS, 4), "algorithmic_bytes": lm_bytes}
            ids_host = ids.cpu().numpy()
            assert ids_host.min() >= 0 and ids_host.max() < vocab
        record["lm_head"] = {"kernel": f"lm_head_kernel (dense bf16 {vocab}x{shape.hidden}, final norm + argmax fused)",
                             "bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "traffic": MEASURED_LM_HEAD_TRAFFIC_BYTES if (args.config == 3) else None, **lm}
        # One drafting round: k forwards on a growing window (1..k tokens), each followed by the head on the last
        # position, everything on the device, captured in one graph.  The head's matrix doubles as the embedding.
        kr = vcfg["k"]
        dr_bytes = sd2.draft_round_workspace_size(model, vocab, kr)
        dr_ws = torch.empty(dr_bytes, dtype=torch.uint8, device=dev)
        start_tok = torch.tensor([1], dtype=torch.int32, device=dev)
        dr_ids = torch.full((kr,), -1, dtype=torch.int32, device=dev)
        dr_us = float(np.mean(B.graph_us(lambda spp: sd2.draft_round(model, w_lm.data_ptr(), vocab, start_tok.data_ptr(), kr, dr_ids.data_ptr(),
                                                                     dr_ws.data_ptr(), dr_bytes, spp), 20, warm=2)))
        sd2.draft_round_status(model, vocab, kr, dr_ws.data_ptr(), stream.cuda_stream)
        ids_host = dr_ids.cpu().numpy()
        assert ids_host.min() >= 0 and ids_host.max() < vocab
        dr_alg = kr * (useful + 2 * vocab * shape.hidden)  # every step streams the stack and the head once
        record["draft_round"] = {"what": f"k={kr} greedy draft tokens: per step embedding rows, stack forward on the window so far, "
                                         "LM head on its last position", "us": round(dr_us, 1),
                                 "us_per_token": round(dr_us / kr, 1), "algorithmic_bytes": dr_alg,
                                 "achieved_GBps": round(dr_alg / dr_us / 1e3, 1),
                                 "frac": round(dr_alg / dr_us / 1e3 / HBM_PEAK_GBS, 4)}

        # One decode step with rotary embedding and a key/value cache: one new token at position 428 (a 300-token prompt
        # and 128 generated tokens: the middle of the request shape of the paper's serving measurements), synthetic history.
        # The single-launch kernel with its attention step over the cache.  Beside it: the window forward (no cache, no
        # rotary embedding) on one token.  Not part of `value`.
        dpos, dmax = 428, 1024
        kc_np, vc_np = wl.gen_kv_history(args.config, layers, shape.n_kv, dmax, shape.head_dim, dpos)
        kc_dev, vc_dev = to_dev(kc_np), to_dev(vc_np)
        del kc_np, vc_np
        dh_in = to_dev(wl.gen_x(args.config, 1, "q", 1, shape.hidden))
        dh_out = torch.empty((1, shape.hidden), dtype=torch.float32, device=dev)
        dec_bytes = sd2.drafter_decode_workspace_size(model, 1)
        dec_ws = torch.empty(dec_bytes, dtype=torch.uint8, device=dev)
        w1_bytes = sd2.drafter_workspace_size(model, 1)
        w1_ws = torch.empty(w1_bytes, dtype=torch.uint8, device=dev)
        dec_call = lambda spp: sd2.sparse_drafter_decode(model, dh_in.data_ptr(), 1, dpos, kc_dev.data_ptr(), vc_dev.data_ptr(),
                                                         dmax, 500000.0, dh_out.data_ptr(), dec_ws.data_ptr(), dec_bytes, spp)
        win_call = lambda spp: sd2.sparse_drafter_forward(model, dh_in.data_ptr(), 1, dh_out.data_ptr(), w1_ws.data_ptr(),
                                                          w1_bytes, spp)
        dec_us = {}
        for name, call in (("decode", dec_call), ("window", win_call)):
            dec_us[name] = float(np.mean(B.graph_us(call, 30)))
            assert torch.isfinite(dh_out).all()
        sd2.drafter_forward_status(model, 1, w1_ws.data_ptr(), stream.cuda_stream)
        sd2.drafter_decode_status(model, 1, dec_ws.data_ptr(), stream.cuda_stream)
        kv_bytes = 2 * 2 * layers * shape.n_kv * (dpos + 1) * shape.head_dim  # keys and values of the positions read, bf16
        dec_alg = useful + kv_bytes
        record["decode"] = {"what": f"one token at position {dpos}: rotary embedding, append to the bf16 key/value cache, attention "
                                    f"over {dpos + 1} positions, single launch",
                            "us": round(dec_us["decode"], 1), "algorithmic_bytes": dec_alg, "kv_cache_bytes_read": kv_bytes,
                            "achieved_GBps": round(dec_alg / dec_us["decode"] / 1e3, 1),
                            "frac": round(dec_alg / dec_us["decode"] / 1e3 / HBM_PEAK_GBS, 4),
                            "window_forward_k1_us": round(dec_us["window"], 1),
                            "traffic": MEASURED_DECODE_TRAFFIC_BYTES if (args.config == 3) else None}
        # The drafting round against the cache: k single-token decode steps from position dpos, each followed by the head.
        rc_bytes = sd2.draft_round_cached_workspace_size(model, vocab, kr)
        rc_ws = torch.empty(rc_bytes, dtype=torch.uint8, device=dev)
        rc_ids = torch.full((kr,), -1, dtype=torch.int32, device=dev)
        rc_us = float(np.mean(B.graph_us(lambda spp: sd2.draft_round_cached(model, w_lm.data_ptr(), vocab, start_tok.data_ptr(), kr, dpos,
                                                                            kc_dev.data_ptr(), vc_dev.data_ptr(), dmax, 500000.0,
                                                                            rc_ids.data_ptr(), rc_ws.data_ptr(), rc_bytes, spp), 20, warm=2)))
        sd2.draft_round_cached_status(model, vocab, kr, rc_ws.data_ptr(), stream.cuda_stream)
        ids_host = rc_ids.cpu().numpy()
        assert ids_host.min() >= 0 and ids_host.max() < vocab
        rc_alg = kr * (useful + 2 * vocab * shape.hidden) + sum(
            2 * 2 * layers * shape.n_kv * (dpos + i + 1) * shape.head_dim for i in range(kr))
        record["draft_round_cached"] = {"what": f"k={kr} greedy draft tokens from position {dpos}: per step one embedding row, one "
                                                "decode step against the cache, LM head", "us": round(rc_us, 1),
                                        "us_per_token": round(rc_us / kr, 1), "algorithmic_bytes": rc_alg,
                                        "achieved_GBps": round(rc_alg / rc_us / 1e3, 1),
                                        "frac": round(rc_alg / rc_us / 1e3 / HBM_PEAK_GBS, 4)}
        del w_lm, kc_dev, vc_dev

        # Masked-gradient step of sparse fine-tuning on the fused gate+up shape (fp32 gradient, in place), two
        # gradient buffers alternating so that the last-level cache cannot hold the working set.  Not part of `value`.
        gsh = (int(gi.n_out), int(gi.k_in))
        grads = [torch.randn(gsh, dtype=torch.float32, device=dev) for _ in range(2)]
        dmg = []
        with torch.cuda.stream(stream):
            for rep in range(3):
                evg = [torch.cuda.Event(enable_timing=True) for _ in range(2 * 8)]
                for i in range(8):
                    evg[2 * i].record(stream)
                    sd2.mask_gradient(gu[i % layers], grads[i & 1].data_ptr(), False, stream.cuda_stream)
                    evg[2 * i + 1].record(stream)
                stream.synchronize()
                if rep:
                    dmg += [evg[2 * i].elapsed_time(evg[2 * i + 1]) * 1e3 for i in range(8)]
        us_mg = float(np.mean(dmg))
        b_mg = 2 * 4 * gsh[0] * gsh[1] + gsh[0] * gsh[1] // 8
        record["mask_gradient"] = {"kernel": f"mask_gradient_kernel (fp32 gradient {gsh[0]}x{gsh[1]}, in place)", "bound": "hbm",
                                   "peak": HBM_PEAK_GBS, "unit": "GB/s", "kernel_us": round(us_mg, 2),
                                   "achieved": round(b_mg / us_mg / 1e3, 1), "frac": round(b_mg / us_mg / 1e3 / HBM_PEAK_GBS, 4),
                                   "algorithmic_bytes": b_mg, "traffic": None}
        del grads

    if not args.no_nm24:
        # The 2:4 semi-structured variant of the largest linear (fused gate+up), timed like the unstructured kernel
        # above: one launch per distinct matrix (8 of them, 453 MB, more than the last-level cache holds), event pairs
        # on the launch stream.  Not part of `value`.
        n_gu, k_gu = 2 * shape.inter, shape.hidden

        def gen24(l):
            w24 = np.concatenate([wl.gen_weight(args.config, l, p, shape.inter, shape.hidden, 50, pattern="2:4")
                                  for p in ("gate", "up")], axis=0)
            return sd2.pack_sparse(w24, 3)

        with ThreadPoolExecutor(max_workers=workers) as ex:
            blobs24 = list(ex.map(gen24, range(8)))
        keep24 = [torch.from_numpy(b).to(dev) for b in blobs24]
        mats24 = [sd2.matrix_init_sparse(b, d.data_ptr()) for b, d in zip(blobs24, keep24)]
        y24 = torch.empty((k_tok, n_gu), dtype=torch.float32, device=dev)
        d24 = []
        with torch.cuda.stream(stream):
            for rep in range(4):
                ev24 = [torch.cuda.Event(enable_timing=True) for _ in range(2 * len(mats24))]
                for i, m in enumerate(mats24):
                    ev24[2 * i].record(stream)
                    sd2.sparse_linear(m, x_act.data_ptr(), k_tok, y24.data_ptr(), 0, 0, stream.cuda_stream)
                    ev24[2 * i + 1].record(stream)
                stream.synchronize()
                if rep:
                    d24 += [ev24[2 * i].elapsed_time(ev24[2 * i + 1]) * 1e3 for i in range(len(mats24))]
        us24 = float(np.mean(d24))
        b24 = int(mats24[0].info.useful_bytes) + 2 * k_tok * k_gu + 4 * k_tok * n_gu
        record["nm24_linear"] = {"kernel": f"nm24_linear_kernel (2:4 semi-structured fused gate+up, {n_gu}x{k_gu}, "
                                           "structured-sparse matrix instruction)",
                                 "bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s", "kernel_us": round(us24, 2),
                                 "achieved": round(b24 / us24 / 1e3, 1), "frac": round(b24 / us24 / 1e3 / HBM_PEAK_GBS, 4),
                                 "algorithmic_bytes": b24,
                                 "traffic": MEASURED_NM24_TRAFFIC_BYTES if (args.config == 3 and k_tok == 5) else None}
        assert np.isfinite(y24.cpu().numpy()).all()
        del keep24, mats24, blobs24

    if args.nm24_stack:
        table_nk = {p: (n, k) for p, n, k in wl.layer_matrix_shapes(shape)}

        def gen24_fused(job):
            l, projs = job
            return np.concatenate([wl.gen_weight(args.config, l, p, table_nk[p][0], table_nk[p][1], 50, pattern="2:4") for p in projs], axis=0)

        jobs = [(l, g) for l in range(layers) for g in FUSED_GROUPS]
        with ThreadPoolExecutor(max_workers=workers) as ex:
            fused24 = list(ex.map(gen24_fused, jobs))
            sblobs = list(ex.map(lambda w: sd2.pack_sparse(w, 3), fused24))
        skeep = [torch.from_numpy(b).to(dev) for b in sblobs]
        smats = [sd2.matrix_init_sparse(b, d.data_ptr()) for b, d in zip(sblobs, skeep)]
        smodel = sd2.model_create(ms, smats, keep=skeep)
        s24_us = B.forward_us(smodel, shape, k_tok, max(args.steps // 4, 10), cfg_id=args.config)
        sbytes = sum(int(m.info.useful_bytes) for m in smats)
        record["config"]["nm24_stack_us"] = round(s24_us, 2)
        record["config"]["nm24_stack_GBps"] = round(sbytes / s24_us / 1e3, 1)
        sd2.model_destroy(smodel)
        del skeep, fused24

    if not args.no_cpu_baseline:
        from oracle import stack as ostack

        split = {"q": (0, 0, shape.q_out), "k": (0, shape.q_out, shape.q_out + shape.kv_out),
                 "v": (0, shape.q_out + shape.kv_out, shape.q_out + 2 * shape.kv_out), "o": (1, 0, shape.hidden),
                 "gate": (2, 0, shape.inter), "up": (2, shape.inter, 2 * shape.inter), "down": (3, 0, shape.hidden)}

        def wfn(layer, proj):
            idx, a, b = split[proj]
            return fused[4 * layer + idx][a:b]

        h_bits = wl.gen_x(args.config, 0, "q", k_tok, shape.hidden)
        # one layer first to size the sample: about 15 s of oracle work, at most the whole stack
        t0 = time.perf_counter()
        ostack.drafter_forward(shape, wfn, h_bits, n_layers=1)
        one_s = time.perf_counter() - t0
        sample_layers = int(min(layers, max(1, round(15.0 / max(one_s, 1e-3)))))
        t0 = time.perf_counter()
        ostack.drafter_forward(shape, wfn, h_bits, n_layers=sample_layers)
        cpu_s = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([int(i.get("num_threads", 1)) for i in threadpool_info()] or [1])
        except Exception:
            cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        record["cpu_baseline"] = {
            "value": round(cpu_s / sample_layers * layers * 1e6, 0),
            "unit": "us",
            "cores": cores,
            "kind": "oracle",
            "sample": f"{sample_layers} of {layers} layers of the same stack and input (fp64 NumPy masked-dense oracle, "
                      f"bf16->fp64 conversion included), scaled to {layers} layers; measured {cpu_s:.1f} s",
        }

    print(json.dumps(record), flush=True)
    # orderly teardown while the runtime is still up: graphs first, then the model
    if use_graph:
        del run_fwd, run_ver, g_fwd, g_ver
    sd2.model_destroy(model)
    torch.cuda.synchronize()


if __name__ == "__main__":
    main()
