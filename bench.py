#!/usr/bin/env python3
"""Benchmark of the fused mixed-precision linear layer on one MI355X.

One step = one pass of the whole hot path over synthetic inputs with the Llama-2 7B layer
shapes (4-bit, group 128, k = 128 weak columns):

  decode     decoder blocks at M = 1: the seven layers of a block (q, k, v, o, gate, up, down), each
             stored and packed on its own, in the four launches the block's dataflow allows -
             q / k / v read the same input and go out together (qeft_linear_fwd_group), so do gate
             and up; over 10 distinct packed copies of the block in a row (> 1 GB, so the weights
             come from HBM, not from the 256 MB last-level cache); the 40 launches are replayed
             from one HIP graph so that the GPU, not Python, sets the pace
  fine-tune  M = 4096 tokens on the three layer shapes: forward, dX through the full mixed
             weight, dW of the weak columns
  pack       min-max round-to-nearest quantization + packing of one 4096 x 4096 layer

`value` is the decode figure of the metric (stored weight bytes of the block / time of the
decode segment); the fine-tune TFLOP/s is reported beside it.  Everything is timed with HIP
events on the stream the kernels run on.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_F16_PEAK_TF = 2500.0   # MI355X dense fp16 MFMA
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, scaled by the
# same counters' reading for its 256 MiB device copy (profiles/bench_7b_hbm_traffic.md): averages over
# the launches of the kernel in one step.  They are NOT measured in this run (counters need the profiler).
TRAFFIC_DX_BYTES = (439.7e6 + 45.6e6 + 374.0e6 + 99.3e6) / 2      # gemm_dx_dw_kernel, read + written, mean of the two MLP shapes
TRAFFIC_GEMV_BYTES = (29.24e6 + 9.84e6 + 52.28e6 + 25.09e6) / 4    # gemv_w4_dot_kernel, mean of the four launches of a block
TRAFFIC_SOURCE = "profiles/bench_7b_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script; not measured in this run)"
# every stored byte of one 7B block with rows padded to 4 words and unpadded group parameters: the figure a
# reader derives from the format alone; block_bytes below is what this build stores (rows padded to 16 words)
ALGORITHMIC_BLOCK_BYTES = 115501056


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-models", action="store_true", help="skip the 13B / 70B timings (a profile of the 7B workload alone)")
    ap.add_argument("--sustained-seconds", type=float, default=2.0, help="length of the back-to-back fine-tune leg")
    args = ap.parse_args()

    def progress(what):   # one line per leg on stderr: a profiled run is slow, and a silent one looks hung
        print(f"[bench] {what}", file=sys.stderr, flush=True)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2410_08661_amd import binding as B
    from paper_2410_08661_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    bits, g, k = 4, 128, 128
    block_shapes = synth.LLAMA_7B_BLOCK            # 7 launches of one decoder block
    ft_shapes = synth.LLAMA_7B                     # the three distinct shapes
    M_ft = 4096

    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.seed_for(2, 0))

    def synth_weight(oc, ic):
        return (torch.randn((oc, ic), generator=gen, device=dev, dtype=torch.float32) * 0.02).half()

    def synth_x(m, ic):
        x = torch.randn((m, ic), generator=gen, device=dev, dtype=torch.float32)
        x[:, ic - k:] *= 20.0                      # the outlier channels that make columns weak
        return x.half()

    progress("packing the decode blocks")
    # ---- decode: enough distinct packed blocks to exceed 1 GB ------------------------------------
    descs = {s: B.make_desc(s[0], s[1], k, bits, g) for s in set(block_shapes)}
    block_bytes = 0
    blocks = []
    n_blocks = 10
    for b in range(n_blocks):
        layers = []
        for s in block_shapes:
            layers.append(B.qeft_pack(descs[s], synth_weight(*s)))
        blocks.append(layers)
    block_bytes = sum(l.nbytes() for l in blocks[0])
    x1 = {ic: synth_x(1, ic) for ic in {s[1] for s in block_shapes}}
    y1 = [torch.empty((1, s[0]), dtype=torch.float16, device=dev) for s in block_shapes]   # one output per layer
    # the launches of a block, as lists of layer indices: q/k/v share their input, and so do gate/up
    assert block_shapes == [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
    launches = [("q/k/v", [0, 1, 2]), ("o", [3]), ("gate/up", [4, 5]), ("down", [6])]
    groups = [[B.Group([descs[block_shapes[i]] for i in idx], [layers[i] for i in idx], [y1[i] for i in idx])
               for _, idx in launches] for layers in blocks]

    def decode_launch(b, li):
        idx = launches[li][1]
        x = x1[block_shapes[idx[0]][1]]
        if len(idx) == 1:
            B.qeft_linear_fwd(descs[block_shapes[idx[0]]], blocks[b][idx[0]], x, y1[idx[0]])
        else:
            B.qeft_linear_fwd_group(None, None, x, group=groups[b][li])

    def decode_block(b):
        for li in range(len(launches)):
            decode_launch(b, li)

    decode_block(0)                                # first launch sets kernel attributes: outside capture
    torch.cuda.synchronize()
    # one graph = one decode token of the 32-block model: 32 blocks in a row, cycling through the distinct packed
    # blocks (1.16 GB apart, so none is still cached when its turn comes again)
    graph_blocks = 32
    cap_stream = torch.cuda.Stream()
    decode_graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(decode_graph, stream=cap_stream):
        for b in range(graph_blocks):
            decode_block(b % n_blocks)

    progress("fine-tune operands")
    # ---- fine-tune operands -----------------------------------------------------------------------
    ft = []
    for s in ft_shapes:
        oc, ic = s
        d = descs[s]
        x = synth_x(M_ft, ic)
        dy = (torch.randn((M_ft, oc), generator=gen, device=dev, dtype=torch.float32) * 0.01).half()
        ws_n = B.qeft_workspace_bytes(d, B.QEFT_OP_BWD, M_ft)
        ft.append(dict(shape=s, desc=d, w=blocks[0][block_shapes.index(s)], x=x, dy=dy,
                       y=torch.empty((M_ft, oc), dtype=torch.float16, device=dev),
                       dx=torch.empty((M_ft, ic), dtype=torch.float16, device=dev),
                       dw=torch.zeros((oc, k), dtype=torch.float32, device=dev),
                       ws=torch.empty(max(ws_n, 1), dtype=torch.uint8, device=dev) if ws_n else None))
    pack_w = synth_weight(4096, 4096)
    pack_out = B.Weight(descs[(4096, 4096)])

    def call_us(call, n=5):
        for _ in range(2):
            call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            call()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n

    # the backward's two steps as calls of their own (outside the timed step, which takes them in one call)
    ft_split = [(call_us(lambda f=f: B.qeft_linear_bwd_dx(f["desc"], f["w"], f["dy"], f["dx"])),
                 call_us(lambda f=f: B.qeft_weak_grad(f["desc"], f["dy"], f["x"][:, f["shape"][1] - k:], dW=f["dw"], ws=f["ws"])))
                for f in ft]

    ev = lambda: torch.cuda.Event(enable_timing=True)
    records = []

    def one_step(i, timed):
        marks = [ev()]
        marks[0].record()
        decode_graph.replay()
        marks.append(ev()); marks[-1].record()
        for f in ft:
            B.qeft_linear_fwd(f["desc"], f["w"], f["x"], f["y"])
            marks.append(ev()); marks[-1].record()
            B.qeft_linear_bwd(f["desc"], f["w"], f["dy"], f["x"][:, f["shape"][1] - k:], dX=f["dx"], dW=f["dw"], ws=f["ws"])
            marks.append(ev()); marks[-1].record()
        B.qeft_pack(descs[(4096, 4096)], pack_w, pack_out)
        marks.append(ev()); marks[-1].record()
        if timed:
            records.append(marks)

    progress("timed steps")
    for i in range(args.warmup):
        one_step(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(args.warmup + i, True)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3

    progress("decode launches, one graph each")
    # ---- the decode kernel by launch: one graph per launch of the block holding that launch of every
    # rotating block, so that the launch periods can be told apart (host launch overhead would
    # dominate eager launches this short)
    decode_kernels = []
    gemv_bytes, gemv_ms = 0.0, 0.0
    for li, (name, idx) in enumerate(launches):
        gs = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gs, stream=cap_stream):
            for b in range(n_blocks):
                decode_launch(b, li)
        gs.replay()
        torch.cuda.synchronize()
        n_rep = max(args.steps, 5)
        e0, e1 = ev(), ev()
        e0.record()
        for r in range(n_rep):
            gs.replay()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (n_rep * n_blocks)
        nb = sum(blocks[0][i].nbytes() for i in idx)
        s0 = block_shapes[idx[0]]
        gemv_bytes += nb
        gemv_ms += us * 1e-3
        decode_kernels.append(dict(launch=name, layers=f"{len(idx)} x {s0[0]}x{s0[1]}", bytes=nb, us=round(us, 2),
                                   gbs=round(nb / us / 1e3, 1)))
    gemv_kernel_gbs = gemv_bytes / (gemv_ms * 1e-3) / 1e9

    def graph_period_us(fn, n_copies):
        """fn(c) enqueues one launch on copy c; period of one launch inside a graph over all copies."""
        fn(0)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=cap_stream):
            for c in range(n_copies):
                fn(c)
        gr.replay()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(n_rep):
            gr.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / (n_rep * n_copies)

    # the same four launches at M = 8 (config 2 names M = 1 and M = 8)
    x8 = {ic: synth_x(8, ic) for ic in {s[1] for s in block_shapes}}
    y8 = [torch.empty((8, s[0]), dtype=torch.float16, device=dev) for s in block_shapes]
    groups8 = [[B.Group([descs[block_shapes[i]] for i in idx], [layers[i] for i in idx], [y8[i] for i in idx])
                for _, idx in launches] for layers in blocks]
    decode_m8 = []
    for li, (name, idx) in enumerate(launches):
        def l8(c, li=li, idx=idx):
            x = x8[block_shapes[idx[0]][1]]
            if len(idx) == 1:
                B.qeft_linear_fwd(descs[block_shapes[idx[0]]], blocks[c][idx[0]], x, y8[idx[0]])
            else:
                B.qeft_linear_fwd_group(None, None, x, group=groups8[c][li])
        us = graph_period_us(l8, n_blocks)
        decode_m8.append(dict(launch=name, us=round(us, 2), vs_M1=round(us / decode_kernels[li]["us"], 2)))
    del x8, y8, groups8

    progress("irregular projection, 3-bit layouts")
    # ---- the attention output projection with its weak columns left in place (the layout the offline
    # reordering cannot reach): the same stored layer behind an on-the-fly gather of the activations
    d_o = descs[(4096, 4096)]
    widx = torch.randperm(4096, generator=torch.Generator().manual_seed(7))[:k].sort().values
    is_weak = torch.zeros(4096, dtype=torch.bool)
    is_weak[widx] = True
    perm_o = torch.cat([torch.nonzero(~is_weak).flatten(), widx]).to(torch.int32).to(dev)
    ws_irr = torch.empty(B.qeft_workspace_bytes(d_o, B.QEFT_OP_FWD_IRREGULAR, M_ft), dtype=torch.uint8, device=dev)
    B.qeft_linear_fwd_irregular(d_o, blocks[0][3], perm_o, x1[4096], y1[3], ws=ws_irr)
    gi = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gi, stream=cap_stream):
        for b in range(n_blocks):
            B.qeft_linear_fwd_irregular(d_o, blocks[b][3], perm_o, x1[4096], y1[3], ws=ws_irr)
    gi.replay()
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record()
    for r in range(n_rep):
        gi.replay()
    e1.record()
    torch.cuda.synchronize()
    irr_decode_us = e0.elapsed_time(e1) * 1e3 / (n_rep * n_blocks)
    f0 = ft[0]
    for _ in range(2):
        B.qeft_linear_fwd_irregular(d_o, f0["w"], perm_o, f0["x"], f0["y"], ws=ws_irr)
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(5):
        B.qeft_linear_fwd_irregular(d_o, f0["w"], perm_o, f0["x"], f0["y"], ws=ws_irr)
    e1.record()
    torch.cuda.synchronize()
    irr_ft_us = e0.elapsed_time(e1) * 1e3 / 5
    del ws_irr
    # the grid-search quantizer (80 candidates per group) on the same layer as the pack segment
    for _ in range(2):
        B.qeft_pack_search(descs[(4096, 4096)], pack_w, 80, 0.01, pack_out)
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(5):
        B.qeft_pack_search(descs[(4096, 4096)], pack_w, 80, 0.01, pack_out)
    e1.record()
    torch.cuda.synchronize()
    pack_search_us = e0.elapsed_time(e1) * 1e3 / 5

    # 3-bit storage of the same up-projection (Tab. 5's 3-bit models), both layouts: decode over rotating packed
    # copies, and the forward at M = 4096 through the dequantized fp16 copy
    three_bit = {"layer": "11008x4096, w3 g128 k=128"}
    w3 = synth_weight(11008, 4096)
    f1 = ft[1]
    for lname, lid in (("canonical", B.QEFT_LAYOUT_CANONICAL), ("dense", B.QEFT_LAYOUT_DENSE3)):
        d3 = B.make_desc(11008, 4096, k, 3, g, layout=lid)
        copies = [B.qeft_pack(d3, w3) for _ in range(n_blocks)]
        B.qeft_linear_fwd(d3, copies[0], x1[4096], y1[4])
        g3 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g3, stream=cap_stream):
            for b in range(n_blocks):
                B.qeft_linear_fwd(d3, copies[b], x1[4096], y1[4])
        g3.replay()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for r in range(n_rep):
            g3.replay()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (n_rep * n_blocks)
        three_bit[f"decode_us_{lname}"] = round(us, 2)
        three_bit[f"decode_gbs_{lname}"] = round(copies[0].nbytes() / us / 1e3, 1)
        three_bit[f"bytes_{lname}"] = copies[0].nbytes()
        ws3 = torch.empty(B.qeft_workspace_bytes(d3, B.QEFT_OP_FWD, M_ft), dtype=torch.uint8, device=dev)
        for _ in range(2):
            B.qeft_linear_fwd(d3, copies[0], f1["x"], f1["y"], ws=ws3)
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(5):
            B.qeft_linear_fwd(d3, copies[0], f1["x"], f1["y"], ws=ws3)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / 5
        three_bit[f"fwd_M4096_us_{lname}"] = round(us, 1)
        three_bit[f"fwd_M4096_tflops_{lname}"] = round(2.0 * M_ft * 11008 * 4096 / us / 1e6, 1)
        del copies, ws3
    del w3

    progress("decode on the 13B / 70B blocks")
    # ---- decode at M = 1 on the other models' blocks (outside the timed step): one graph per launch over enough
    # distinct copies to exceed the last-level cache; random stored components
    def rand_weight(desc_):
        w_ = B.Weight(desc_)
        w_.qweight.random_(-2**31, 2**31 - 1, generator=gen)
        if desc_.bits == 3 and desc_.layout == B.QEFT_LAYOUT_CANONICAL:
            w_.qweight.bitwise_and_(0x3fffffff)
        w_.scales.copy_((torch.rand(w_.scales.shape, generator=gen, device=dev) * 0.008 + 0.004).half())
        w_.zeros.copy_(torch.randint(0, 2 ** desc_.bits, w_.zeros.shape, generator=gen, device=dev).half())
        w_.weak.copy_((torch.randn(w_.weak.shape, generator=gen, device=dev) * 0.02).half())
        return w_

    decode_other = []
    other_blocks = [] if args.no_other_models else [
        ("Llama-2-13B", 128, 4, B.QEFT_LAYOUT_CANONICAL, [("q/k/v", [(5120, 5120)] * 3), ("o", [(5120, 5120)]), ("gate/up", [(13824, 5120)] * 2), ("down", [(5120, 13824)])]),
        ("Llama-2-13B", 128, 3, B.QEFT_LAYOUT_CANONICAL, [("q/k/v", [(5120, 5120)] * 3), ("o", [(5120, 5120)]), ("gate/up", [(13824, 5120)] * 2), ("down", [(5120, 13824)])]),
        ("Llama-2-13B", 128, 3, B.QEFT_LAYOUT_DENSE3, [("q/k/v", [(5120, 5120)] * 3), ("o", [(5120, 5120)]), ("gate/up", [(13824, 5120)] * 2), ("down", [(5120, 13824)])]),
        ("Llama-2-70B", 256, 4, B.QEFT_LAYOUT_CANONICAL, [("q/k/v", [(8192, 8192), (1024, 8192), (1024, 8192)]), ("o", [(8192, 8192)]), ("gate/up", [(28672, 8192)] * 2), ("down", [(8192, 28672)])]),
    ]
    for model, k_o, bits_o, lay_o, launches_o in other_blocks:
        tot_us, tot_b, per_launch = 0.0, 0, []
        for name, shapes in launches_o:
            ds = [B.make_desc(oc, ic, k_o, bits_o, g, layout=lay_o) for oc, ic in shapes]
            one = sum(B.Weight(d_).nbytes() for d_ in ds)
            n_c = max(2, min(n_blocks * 2, int(1.1e9 // one)))
            copies = [[rand_weight(d_) for d_ in ds] for _ in range(n_c)]
            xo = torch.randn((1, shapes[0][1]), generator=gen, device=dev).half()
            yo = [torch.empty((1, oc), dtype=torch.float16, device=dev) for oc, _ in shapes]
            grp = [B.Group(ds, cw, yo) for cw in copies] if len(shapes) > 1 else None

            def lo(c, ds=ds, copies=copies, xo=xo, yo=yo, grp=grp):
                if grp is None:
                    B.qeft_linear_fwd(ds[0], copies[c][0], xo, yo[0])
                else:
                    B.qeft_linear_fwd_group(None, None, xo, group=grp[c])
            us = graph_period_us(lo, n_c)
            per_launch.append(dict(launch=name, bytes=one, us=round(us, 2), gbs=round(one / us / 1e3, 1)))
            tot_us += us
            tot_b += one
            del copies, grp
        decode_other.append(dict(model=model, bits=bits_o, layout="dense" if lay_o == B.QEFT_LAYOUT_DENSE3 else "canonical", k=k_o,
                                 block_bytes=tot_b, block_us=round(tot_us, 2), gbs=round(tot_b / tot_us / 1e3, 1),
                                 pct_hbm_peak=round(100 * tot_b / tot_us / 1e3 / HBM_PEAK_GBS, 2), launches=per_launch))

    progress("fine-tune on the 13B / 70B shapes")
    # ---- the other models' fine-tune shapes (outside the timed step; context for the 7B figures) ---------
    # forward and input gradient with the optional workspace (launches with few tiles, or with a sparsely filled last
    # round of tiles, split their contraction over it), weak gradient; random stored components, one layer per shape
    other_models = []
    for model, shapes, k_o, m_o in (() if args.no_other_models else (("Llama-2-13B", synth.LLAMA_13B, 128, 4096), ("Llama-2-70B", synth.LLAMA_70B, 256, 2048))):
        for oc, ic in shapes:
            d_o2 = B.make_desc(oc, ic, k_o, bits, g)
            w_o2 = B.Weight(d_o2)
            w_o2.qweight.random_(-2**31, 2**31 - 1, generator=gen)
            w_o2.scales.copy_((torch.rand(w_o2.scales.shape, generator=gen, device=dev) * 0.008 + 0.004).half())
            w_o2.zeros.copy_(torch.randint(0, 16, w_o2.zeros.shape, generator=gen, device=dev).half())
            w_o2.weak.copy_((torch.randn(w_o2.weak.shape, generator=gen, device=dev) * 0.02).half())
            x_o = torch.randn((m_o, ic), generator=gen, device=dev).half()
            dy_o = (torch.randn((m_o, oc), generator=gen, device=dev) * 0.01).half()
            y_o = torch.empty((m_o, oc), dtype=torch.float16, device=dev)
            dx_o = torch.empty((m_o, ic), dtype=torch.float16, device=dev)
            dw_o = torch.zeros((oc, k_o), dtype=torch.float32, device=dev)
            n_ws = max(B.qeft_workspace_bytes(d_o2, op, m_o) for op in (B.QEFT_OP_FWD, B.QEFT_OP_BWD_DX, B.QEFT_OP_WEAK_GRAD))
            ws_o = torch.empty(max(n_ws, 16), dtype=torch.uint8, device=dev)
            calls = (lambda: B.qeft_linear_fwd(d_o2, w_o2, x_o, y_o, ws=ws_o),
                     lambda: B.qeft_linear_bwd_dx(d_o2, w_o2, dy_o, dx_o, ws=ws_o),
                     lambda: B.qeft_weak_grad(d_o2, dy_o, x_o[:, ic - k_o:], dW=dw_o, ws=ws_o),
                     lambda: B.qeft_linear_bwd(d_o2, w_o2, dy_o, x_o[:, ic - k_o:], dX=dx_o, dW=dw_o, ws=ws_o))
            us = [call_us(call) for call in calls]
            fl = 2.0 * m_o * oc * ic
            other_models.append(dict(model=model, shape=f"{oc}x{ic}", k=k_o, M=m_o, fwd_us=round(us[0], 1), fwd_tflops=round(fl / us[0] / 1e6, 1),
                                     dx_us=round(us[1], 1), dx_tflops=round(fl / us[1] / 1e6, 1), dw_us=round(us[2], 1),
                                     bwd_one_call_us=round(us[3], 1),
                                     step_tflops=round((2 * fl + 2.0 * m_o * oc * k_o) / (us[0] + min(us[1] + us[2], us[3])) / 1e6, 1)))
            del w_o2, x_o, dy_o, y_o, dx_o, dw_o, ws_o

    progress("sustained fine-tune leg")
    # ---- sustained: the fine-tune calls of the 7B shapes back to back for a few seconds (the timed step above lasts
    # milliseconds; the chip is power-managed, so a short burst may not show the clock a long run settles at)
    ft_flops_step = sum(4.0 * M_ft * f["shape"][0] * f["shape"][1] + 2.0 * M_ft * f["shape"][0] * k for f in ft)

    def ft_calls():
        for f in ft:
            B.qeft_linear_fwd(f["desc"], f["w"], f["x"], f["y"])
            B.qeft_linear_bwd(f["desc"], f["w"], f["dy"], f["x"][:, f["shape"][1] - k:], dX=f["dx"], dW=f["dw"], ws=f["ws"])

    sustained = None
    if args.sustained_seconds > 0:
        n_sus = max(20, int(args.sustained_seconds / 1.8e-3))
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(n_sus):
            ft_calls()
        e1.record()
        torch.cuda.synchronize()
        sus_ms = e0.elapsed_time(e1)
        sustained = dict(seconds=round(sus_ms * 1e-3, 2), steps=n_sus, finetune_tflops=round(ft_flops_step * n_sus / sus_ms / 1e9, 1))

    # a plain device copy of known size: the reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE
    # (timed as well: what a plain copy reaches on this machine, read + written bytes per second, as context for the HBM fraction)
    cal = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev)
    cal2 = torch.empty_like(cal)
    cal2.copy_(cal)
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(5):
        cal2.copy_(cal)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * cal.numel() * 4 / (e0.elapsed_time(e1) * 1e-3 / 5) / 1e9
    del cal, cal2

    seg = np.array([[m[j].elapsed_time(m[j + 1]) for j in range(len(m) - 1)] for m in records])   # ms
    mean = seg.mean(axis=0)
    decode_ms = mean[0] / graph_blocks
    gemv_gbs = block_bytes / (decode_ms * 1e-3) / 1e9
    kernels = []
    flops_tot, ms_tot = 0.0, 0.0
    bwd_fl, bwd_ms = 0.0, 0.0
    for fi, f in enumerate(ft):
        oc, ic = f["shape"]
        t_fwd, t_bwd = mean[1 + 2 * fi], mean[2 + 2 * fi]
        fl = 2.0 * M_ft * oc * ic
        fl_dw = 2.0 * M_ft * oc * k
        flops_tot += 2 * fl + fl_dw
        ms_tot += t_fwd + t_bwd
        kernels.append(dict(shape=f"{oc}x{ic}", fwd_us=round(t_fwd * 1e3, 1), fwd_tflops=round(fl / t_fwd / 1e9, 1),
                            bwd_us=round(t_bwd * 1e3, 1), bwd_tflops=round((fl + fl_dw) / t_bwd / 1e9, 1),
                            dx_us=round(ft_split[fi][0], 1), dw_us=round(ft_split[fi][1], 1)))
        if max(oc, ic) == 11008:       # the backward of these goes out as the one combined launch
            bwd_fl += fl + fl_dw
            bwd_ms += t_bwd
    ft_tflops = flops_tot / ms_tot / 1e9
    # dominant kernel of the timed region: the backward launch of the two MLP shapes (dX tiles and weak-gradient strips
    # in one grid; the few microseconds of the kernel that sums the strips' token halves are inside the interval)
    dx_tf = bwd_fl / bwd_ms / 1e9

    out = {
        "metric": "M=1 weight GB/s (% HBM peak); M=4096 fwd+bwd TFLOP/s (% MFMA peak)",
        "value": round(gemv_gbs, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms / args.steps, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "Llama-2-7B layer shapes, w4 g128 k=128: decode M=1 over "
                               f"{n_blocks} distinct packed blocks (7 layers in 4 launches each: q/k/v, o, gate/up, down), one graph of {graph_blocks} blocks = one token of the 32-block model + fine-tune M=4096 fwd + bwd (dX + dW_weak in one call) + pack",
                   "block_bytes": block_bytes, "algorithmic_block_bytes": ALGORITHMIC_BLOCK_BYTES, "M_decode": 1, "M_finetune": M_ft},
        "pct_hbm_peak": round(100 * gemv_gbs / HBM_PEAK_GBS, 2),
        "decode_us_per_block": round(decode_ms * 1e3, 2),
        "finetune_tflops": round(ft_tflops, 1),
        "pct_mfma_peak": round(100 * ft_tflops / MFMA_F16_PEAK_TF, 2),
        "pack_us": round(mean[-1] * 1e3, 1),
        "pack_search_us": round(pack_search_us, 1),
        "finetune_kernels": kernels,
        "roofline": {"kernel": "gemm_dx_dw_kernel", "bound": "mfma", "achieved": round(dx_tf, 1), "peak": MFMA_F16_PEAK_TF,
                     "unit": "TFLOP/s", "frac": round(dx_tf / MFMA_F16_PEAK_TF, 4), "traffic": round(TRAFFIC_DX_BYTES),
                     "traffic_source": TRAFFIC_SOURCE},
        "decode_kernels": decode_kernels,
        "decode_M8": decode_m8,
        "decode_other_models": decode_other,
        "sustained": sustained,
        "value_algorithmic_bytes_gbs": round(ALGORITHMIC_BLOCK_BYTES / (decode_ms * 1e-3) / 1e9, 1),
        "irregular_out_proj": {"layer": "4096x4096, weak columns at arbitrary channels (decode: gather inside the matrix-vector kernel; M=4096: a gather pass, then the same GEMM)",
                               "decode_us": round(irr_decode_us, 2),
                               "decode_us_reordered": next(dk["us"] for dk in decode_kernels if dk["launch"] == "o"),
                               "fwd_M4096_us": round(irr_ft_us, 1), "fwd_M4096_us_reordered": kernels[0]["fwd_us"]},
        "three_bit": three_bit,
        "finetune_other_models": other_models,
        "device_copy_gbs": round(copy_gbs, 1),
        "pct_of_device_copy": round(100 * gemv_gbs / copy_gbs, 1),
        "roofline_gemv": {"kernel": "gemv_w4_dot_kernel", "bound": "hbm", "achieved": round(gemv_kernel_gbs, 1),
                          "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gemv_kernel_gbs / HBM_PEAK_GBS, 4),
                          "traffic": round(TRAFFIC_GEMV_BYTES), "traffic_source": TRAFFIC_SOURCE,
                          "note": "stored bytes of the block's 7 layers / sum of its 4 launch periods, each launch "
                                  "replayed from a graph of its own (HIP events; gaps between launches included, "
                                  "host overhead not)"},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(np, synth, k, bits, g)
    print(json.dumps(out))


def cpu_baseline(np, synth, k, bits, g):
    """The oracle as it stands, timed on the host: one 4096 x 4096 layer at M = 1
    (unpack -> dequantize -> float64 product), scaled to the metric's unit; and, as a second leg, its
    forward product at M = 256 on the same layer in GFLOP/s.  `cores` is what the host offers the process
    (os.cpu_count(), capped by OMP_NUM_THREADS when that is set): the float64 product runs on the BLAS's
    threads, the unpack / dequantize loops on one."""
    from oracle import qeft_oracle as qo
    oc, ic = 4096, 4096
    seed = synth.seed_for(2, 0)
    w16 = synth.make_weight(oc, ic, seed)
    x = synth.make_activations(1, ic, k, seed)
    lay = qo.layout(oc, ic, k, bits, g)
    codes, scales, zeros, weak = qo.quantize_rtn(w16, k, bits, g)
    qweight = qo.pack_codes(codes, bits, lay["row_stride_words"])
    nbytes = lay["qweight_bytes"] + lay["scales_bytes"] + lay["zeros_bytes"] + lay["weak_bytes"]
    reps, t_wall = 0, 0.0
    while t_wall < 10.0 and reps < 50:
        w0 = time.perf_counter()
        w64 = qo.dequantize(qo.unpack_codes(qweight, lay["kq"], bits), scales, zeros, weak, g)
        y = qo.round_fp16(qo.linear_fwd(w64, x))
        t_wall += time.perf_counter() - w0
        reps += 1
    x256 = synth.make_activations(256, ic, k, seed + 1)
    g_reps, g_wall = 0, 0.0
    while g_wall < 5.0 and g_reps < 200:
        w0 = time.perf_counter()
        y = qo.linear_fwd(w64, x256)
        g_wall += time.perf_counter() - w0
        g_reps += 1
    # the same product on one thread (the unpack / dequantize part of the decode sample is single-threaded anyway)
    one_gflops = None
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            o_reps, o_wall = 0, 0.0
            while o_wall < 3.0 and o_reps < 40:
                w0 = time.perf_counter()
                y = qo.linear_fwd(w64, x256)
                o_wall += time.perf_counter() - w0
                o_reps += 1
        one_gflops = round(2.0 * 256 * oc * ic * o_reps / o_wall / 1e9, 1)
    except ImportError:
        pass
    cores = os.cpu_count() or 1
    if os.environ.get("OMP_NUM_THREADS", "").isdigit():
        cores = min(cores, int(os.environ["OMP_NUM_THREADS"]))
    return {"value": round(nbytes * reps / t_wall / 1e9, 4), "unit": "GB/s",
            "cores": cores, "kind": "oracle",
            "sample": f"{reps} x (unpack + dequantize + fp64 product) of one 4096x4096 w4 g128 k128 layer at M=1, "
                      f"{t_wall:.1f} s of host time",
            "gemm_gflops": round(2.0 * 256 * oc * ic * g_reps / g_wall / 1e9, 1),
            "gemm_gflops_one_thread": one_gflops,
            "gemm_sample": f"{g_reps} x the oracle's fp64 forward product of the dequantized layer at M=256, {g_wall:.1f} s"}


if __name__ == "__main__":
    main()
