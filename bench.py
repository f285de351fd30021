#!/usr/bin/env python3
"""Benchmark of the quantized-linear hot path on one MI355X.

A step is one pass of the whole RWKV-6-7B-shaped layer stack (32 layers x 8 matrices, each SQ or VQ
by a seeded coin flip) through rwkvq_linear_dispatch:

  * headline (`value`): batch 1, fp16 activations, one independent activation vector per matrix,
    exactly --steps timed steps after --warmup untimed ones; metric = packed weight bytes read per second
    (GB/s) and the fraction of the 8 TB/s HBM peak.  `steady_state` holds the same step timed over a long
    region of its own (run first: the device leaves the clock transient that follows idle there);
  * `decode_batched`: the same matrices at batch 4, 16, 32, 64, and at batch 4 and 16 as the 128 stage-sized launches a
    model would make (`M*_stage_ordered`); `sequential_step`: batch 1 in data-flow order;
  * `config1`, `config2`: the single-matrix configurations, cache-hot, HBM-cold (rotated copies) and grouped;
  * `prefill`: the same matrix recipe at M = 2048 tokens, bf16 activations, bf16 MFMA with binary32
    accumulate; metric = 2*M*N*K FLOP per second and the fraction of the 2.5 PFLOP/s dense bf16 peak;
  * `config5`: the 14B-class stack (48 layers, d = 5120, SQ / 6-bit VQ / 8-bit VQ, bf16 activations) at
    batch 1 and 16 and as a prefill of M = 4096 tokens;
  * `proxy`, `encode`, `mu`: the quantization-time kernels.

All inputs are resident in HBM before a timed region.  Timing uses HIP events on the stream the kernels
are launched on (torch's current stream), one event per step.  The CPU oracle is timed on the host cores
on the decode workload (`cpu_baseline`) and on a sample of the prefill workload as reported baselines.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
DECODE_KERNEL = "rwkvq::decode_kernel<1, 1>"
DECODE16_KERNEL = "rwkvq::decode_kernel<16, 2>"
PREFILL_KERNEL = "rwkvq::prefill_kernel<true, FMT, 8>"   # bf16; one instantiation per weight format
PROXY_KERNEL = "rwkvq::proxy_set_kernel"
DECODE_MATS_PER_LAUNCH = 256
# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each scaled by what the
# same counter reads for a plain 1 GiB copy (FETCH_SIZE x 2.000, WRITE_SIZE x 1.000 on this image).  Counter runs
# are separate runs of this file (commands in the named summaries under profiles/); the figures are theirs, for the
# default workload only, and are not re-measured by the run that prints them.
TRAFFIC = {
    "decode_config3": (2844.3e6, "profiles/decode_hbm_traffic_config3_config5.txt"),
    "decode_config5_M1": (7309.3e6 / 2, "profiles/decode_hbm_traffic_config3_config5.txt"),     # mean of the two launches of a step
    "decode_config5_M16": (7885.2e6 / 2, "profiles/decode_hbm_traffic_config3_config5.txt"),
    "prefill_config4": (8.87e9, "profiles/prefill_and_mix_hbm_traffic.txt"),
    "proxy_8_layers": (3495.6e6, "profiles/proxy_kernel_trace_and_traffic_7b_layers.txt"),
    "mix_per_call": (75.7e6, "profiles/prefill_and_mix_hbm_traffic.txt"),
}


def traffic(key, applies=True):
    """(bytes per launch | None, source) for a roofline record."""
    return (TRAFFIC[key][0] if applies else None), TRAFFIC[key][1]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_stack(config: int, M: int, n_layers, gpu_activations: bool, y_dtype):
    """Upload the stack (native layout) and allocate activations / outputs.  Returns the dispatch
    table and the byte / FLOP counts."""
    import torch
    from paper_2505_03803_amd import binding as B
    from paper_2505_03803_amd import synth

    xdt = synth.STACKS[config][4]
    descs, xs, ys, keep = [], [], [], []
    wbytes = 0
    flops = 0
    xbytes = 0
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1000 + config)
    for mat, x in synth.stack(config, M, n_layers=n_layers, with_activations=not gpu_activations):
        dm = B.upload(mat, native=True)
        wbytes += mat.packed_bytes
        flops += 2 * M * mat.N * mat.K
        if gpu_activations:
            xf = torch.randn((M, mat.K), device="cuda", generator=gen, dtype=torch.float32)
            xd = xf.to(torch.bfloat16 if xdt == "bf16" else torch.float16).view(torch.int16)
            del xf
        else:
            xd = torch.from_numpy(x.view(np.int16)).cuda()
        yd = torch.empty((M, mat.N), dtype=torch.float32 if y_dtype == B.F32 else torch.int16, device="cuda")
        xbytes += xd.numel() * 2 + yd.numel() * yd.element_size()
        descs.append(dm.desc()); xs.append(xd); ys.append(yd); keep.append(dm)
    table = B.DispatchTable(descs, xs, ys)
    return dict(table=table, keep=(keep, xs, ys), wbytes=wbytes, flops=flops, xybytes=xbytes,
                n_mats=len(descs), x_dtype=B.DTYPES[xdt], descs=descs, ys=ys)


def scale_weights(dm, a: float):
    """Deq(W) <- a * Deq(W) for a matrix on the device (SQ: the fp16 scales; VQ: the codebook entries)."""
    import torch
    from paper_2505_03803_amd import binding as B
    if dm.kind == B.SQ:
        dm.scales.view(torch.float16)[0::2] *= a           # native layout: (scale, zero) pairs
    else:
        dm.codebooks.view(torch.float16).mul_(a)


def rms16(t, bf16=False):
    import torch
    return float(t.view(torch.bfloat16 if bf16 else torch.float16).float().pow(2).mean().sqrt())


def unit_gain(stack, M, bf16=False):
    """Rescale every matrix of a resident stack so that N(0, 1) activations give outputs of unit rms.  The
    synthetic weights are not a trained model's and App. A.1 prints no normalisation: left as drawn, the
    values that flow from block to block overflow after two blocks and the legs that chain the stages would be
    timed on NaNs.  Done after the grouped legs, which keep the weights as the recipe draws them."""
    import torch
    from paper_2505_03803_amd import binding as B
    B.rwkvq_linear_dispatch(stack["table"], M, stack["x_dtype"], B.BF16 if bf16 else B.F16)
    torch.cuda.synchronize()
    for dm, y in zip(stack["keep"][0], stack["keep"][2]):
        scale_weights(dm, 1.0 / max(rms16(y, bf16), 1e-6))
    torch.cuda.synchronize()


def sequential_step(dec, n_layers):
    """One token through the stack with the dependencies of an RWKV block between the launches:
    per layer  mix (4 projections) -> {receptance, key, value, gate} -> output -> mix (2) ->
    {channel key, channel receptance} -> channel value, each stage reading the buffer the stage
    before wrote (6 launches per layer, recorded once into a HIP graph and replayed); then with the
    mixes fused into the GEMVs (4 launches), and with the element-wise operators of the block between
    them (7 launches).  The values that flow are not a model's, the launch structure and the bytes
    are.  Reported next to the grouped figure to show what the dependencies cost."""
    import torch
    from paper_2505_03803_amd import binding as B
    from paper_2505_03803_amd import synth
    d = int(dec["descs"][0].K)                                  # hidden size: K of the receptance projection
    rng = np.random.default_rng(4000)
    t16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda()
    h = t16(synth.gen_activations(rng, 1, d, "f16"))            # the hidden state entering a layer
    hprev = t16(synth.gen_activations(rng, 1, d, "f16")[0])
    stages = []
    keep = []
    for layer in range(n_layers):
        D = dec["descs"][8 * layer: 8 * layer + 8]              # r, k, v, g, o, cm_k, cm_v, cm_r
        Y = dec["ys"][8 * layer: 8 * layer + 8]
        mix4 = [torch.empty((1, d), dtype=torch.int16, device="cuda") for _ in range(4)]
        mix2 = [torch.empty((1, d), dtype=torch.int16, device="cuda") for _ in range(2)]
        def mk(P, outs):
            idx = [torch.from_numpy(rng.integers(0, 64, size=d // 2, dtype=np.uint8)).cuda() for _ in range(P)]
            cbs = [t16(synth.gen_codebook(rng, 64)) for _ in range(P)]
            return B.MixTable(idx, cbs, outs)
        src = h if layer == 0 else stages[-1][2]                 # previous layer's channel-value output
        stages.append(("mix", mk(4, mix4), None, src))
        stages.append(("lin", B.DispatchTable(D[0:4], mix4, Y[0:4]), None, None))
        stages.append(("lin", B.DispatchTable([D[4]], [Y[2]], [Y[4]]), None, None))            # output <- value
        stages.append(("mix", mk(2, mix2), None, Y[4]))
        stages.append(("lin", B.DispatchTable([D[5], D[7]], mix2, [Y[5], Y[7]]), None, None))   # channel key, receptance
        stages.append(("lin", B.DispatchTable([D[6]], [Y[5]], [Y[6]]), Y[6], None))             # channel value <- key
        keep.append((mix4, mix2))

    def step():
        for kind, table, _, src in stages:
            if kind == "mix":
                B.rwkvq_token_shift_mix(src, hprev, B.F16, 1, d, table, 6)
            else:
                B.rwkvq_linear_dispatch(table, 1, B.F16, B.F16)

    # the same step with the mixes fused into the GEMVs that consume them: 4 launches per layer
    fused = []
    for layer in range(n_layers):
        D = dec["descs"][8 * layer: 8 * layer + 8]
        Y = dec["ys"][8 * layer: 8 * layer + 8]
        m4, m2 = stages[6 * layer][1], stages[6 * layer + 3][1]
        src4, src2 = stages[6 * layer][3], stages[6 * layer + 3][3]
        fused.append(("mixed", B.MixedDispatchTable(D[0:4], [(src4, hprev, m4.keep[0][p], m4.keep[1][p], 6) for p in range(4)], Y[0:4])))
        fused.append(("lin", B.DispatchTable([D[4]], [Y[2]], [Y[4]])))
        fused.append(("mixed", B.MixedDispatchTable([D[5], D[7]], [(src2, hprev, m2.keep[0][p], m2.keep[1][p], 6) for p in range(2)], [Y[5], Y[7]])))
        fused.append(("lin", B.DispatchTable([D[6]], [Y[5]], [Y[6]])))

    def step_fused():
        for kind, table in fused:
            if kind == "mixed":
                B.rwkvq_linear_dispatch_mixed(table, B.F16, B.F16)
            else:
                B.rwkvq_linear_dispatch(table, 1, B.F16, B.F16)

    # the whole block as App. A.1 chains it: the element-wise operators between the GEMVs as well
    # (wkv recurrence with its gate, squared ReLU, output gate): 7 launches per layer.  The gate
    # projection of the 7B stack (not in the appendix) still runs; nothing consumes its output.
    block = []
    ffn = dec["ys"][5].shape[1]
    for layer in range(n_layers):
        D = dec["descs"][8 * layer: 8 * layer + 8]
        Y = dec["ys"][8 * layer: 8 * layer + 8]
        m4, m2 = stages[6 * layer][1], stages[6 * layer + 3][1]
        src4 = h if layer == 0 else block[-1][1][2]              # the previous block's output
        _, _, _, w, u = synth.gen_block_inputs(rng, 1, d, "f16")
        st = np.zeros((3, d), dtype=np.float32); st[2] = -1e38
        wd, ud, state = torch.from_numpy(w).cuda(), torch.from_numpy(u).cuda(), torch.from_numpy(st).cuda()
        gated, sq, outb = (torch.zeros((1, n), dtype=torch.int16, device="cuda") for n in (d, ffn, d))
        block.append(("mixed", B.MixedDispatchTable(D[0:4], [(src4, hprev, m4.keep[0][p], m4.keep[1][p], 6) for p in range(4)], Y[0:4])))
        block.append(("wkv", (Y[0], Y[1], Y[2], wd, ud, state, gated)))
        block.append(("lin", B.DispatchTable([D[4]], [gated], [Y[4]])))
        block.append(("mixed", B.MixedDispatchTable([D[5], D[7]], [(Y[4], hprev, m2.keep[0][p], m2.keep[1][p], 6) for p in range(2)], [Y[5], Y[7]])))
        block.append(("relu2", (Y[5], sq)))
        block.append(("lin", B.DispatchTable([D[6]], [sq], [Y[6]])))
        block.append(("gate", (Y[7], Y[6], outb)))

    def launch(kind, a):
        if kind == "mixed":
            B.rwkvq_linear_dispatch_mixed(a, B.F16, B.F16)
        elif kind == "lin":
            B.rwkvq_linear_dispatch(a, 1, B.F16, B.F16)
        elif kind == "wkv":
            B.rwkvq_wkv(a[0], a[1], a[2], B.F16, 1, d, a[3], a[4], a[5], a[6])
        elif kind == "relu2":
            B.rwkvq_relu2(a[0], B.F16, ffn, a[1])
        else:
            B.rwkvq_sigmoid_gate(a[0], a[1], B.F16, d, a[2])

    # every block's output back to unit rms (a per-layer factor on W'_v, found block by block on this
    # token): with unit-gain matrices alone the squared ReLU and the gates shrink the values tenfold per
    # block, and after a few blocks the step would run on zeros
    flow = []
    for layer in range(n_layers):
        for kind, a in block[7 * layer: 7 * layer + 7]:
            launch(kind, a)
        torch.cuda.synchronize()
        outb = block[7 * layer + 6][1][2]
        scale_weights(dec["keep"][0][8 * layer + 6], 1.0 / max(rms16(outb), 1e-6))
        for kind, a in block[7 * layer + 5: 7 * layer + 7]:
            launch(kind, a)
        torch.cuda.synchronize()
        flow.append(rms16(outb))
    for layer in range(n_layers):                              # the wkv states back to the empty sums
        st = block[7 * layer + 1][1][5]
        st[:2].zero_(); st[2].fill_(-1e38)

    def step_block():
        for kind, a in block:
            if kind == "mixed":
                B.rwkvq_linear_dispatch_mixed(a, B.F16, B.F16)
            elif kind == "lin":
                B.rwkvq_linear_dispatch(a, 1, B.F16, B.F16)
            elif kind == "wkv":
                B.rwkvq_wkv(a[0], a[1], a[2], B.F16, 1, d, a[3], a[4], a[5], a[6])
            elif kind == "relu2":
                B.rwkvq_relu2(a[0], B.F16, ffn, a[1])
            else:
                B.rwkvq_sigmoid_gate(a[0], a[1], B.F16, d, a[2])

    # the same block with the squared ReLU and the output gate applied by the GEMVs that produce
    # their operands (rwkvq_linear_dispatch_post): 5 launches per layer, the same bits
    block5 = []
    for layer in range(n_layers):
        D = dec["descs"][8 * layer: 8 * layer + 8]
        Y = dec["ys"][8 * layer: 8 * layer + 8]
        b7 = block[7 * layer: 7 * layer + 7]
        m2 = stages[6 * layer + 3][1]
        sq, outb = b7[4][1][1], b7[6][1][2]
        block5.append(b7[0]); block5.append(b7[1]); block5.append(b7[2])
        block5.append(("post", B.PostDispatchTable([D[5], D[7]], None, [(Y[4], hprev, m2.keep[0][p], m2.keep[1][p], 6) for p in range(2)],
                                                   [(B.POST_RELU2, None), (B.POST_NONE, None)], [sq, Y[7]])))
        block5.append(("post", B.PostDispatchTable([D[6]], [sq], None, [(B.POST_SIGMOID_GATE, Y[7])], [outb])))

    def step_block5():
        for kind, a in block5:
            if kind == "mixed":
                B.rwkvq_linear_dispatch_mixed(a, B.F16, B.F16)
            elif kind == "lin":
                B.rwkvq_linear_dispatch(a, 1, B.F16, B.F16)
            elif kind == "wkv":
                B.rwkvq_wkv(a[0], a[1], a[2], B.F16, 1, d, a[3], a[4], a[5], a[6])
            else:
                B.rwkvq_linear_dispatch_post(a, B.F16, B.F16)

    # the same block once more with every token-shift mix taken where its input vector is produced
    # (rwkvq_post_op.n_mix): W_o stores o and the two mixes of channel mixing, W'_v stores the block's
    # output and the four mixes of the next block; the projections then read plain vectors.  One mix
    # pass in front of the first block.  5 launches per layer + 1.
    blockpm = []
    mixbuf = lambda n: [torch.zeros((1, d), dtype=torch.int16, device="cuda") for _ in range(n)]
    in4 = [mixbuf(4) for _ in range(n_layers + 1)]
    m4_0 = stages[0][1]
    blockpm.append(("mix", (h, B.MixTable(m4_0.keep[0], m4_0.keep[1], in4[0]))))
    for layer in range(n_layers):
        D = dec["descs"][8 * layer: 8 * layer + 8]
        Y = dec["ys"][8 * layer: 8 * layer + 8]
        b7 = block[7 * layer: 7 * layer + 7]
        m2 = stages[6 * layer + 3][1]
        m4n = stages[6 * ((layer + 1) % n_layers)][1]         # the next block's four mix weights
        gated, sq, outb = b7[1][1][6], b7[4][1][1], b7[6][1][2]
        in2 = mixbuf(2)
        blockpm.append(("lin", B.DispatchTable(D[0:4], in4[layer], Y[0:4])))
        blockpm.append(b7[1])
        blockpm.append(("post", B.PostDispatchTable([D[4]], [gated], None,
                        [(B.POST_NONE, None, hprev, [(m2.keep[0][p], m2.keep[1][p], 6, in2[p]) for p in range(2)])], [Y[4]])))
        blockpm.append(("post", B.PostDispatchTable([D[5], D[7]], in2, None, [(B.POST_RELU2, None), (B.POST_NONE, None)], [sq, Y[7]])))
        blockpm.append(("post", B.PostDispatchTable([D[6]], [sq], None,
                        [(B.POST_SIGMOID_GATE, Y[7], hprev, [(m4n.keep[0][p], m4n.keep[1][p], 6, in4[layer + 1][p]) for p in range(4)])], [outb])))

    # the bare GEMV chain (no element-wise operators) with the mixes at the producer: 4 launches per layer + 1
    barepm = [blockpm[0]]
    in4b = [mixbuf(4) for _ in range(n_layers + 1)]
    barepm[0] = ("mix", (h, B.MixTable(m4_0.keep[0], m4_0.keep[1], in4b[0])))
    for layer in range(n_layers):
        D = dec["descs"][8 * layer: 8 * layer + 8]
        Y = dec["ys"][8 * layer: 8 * layer + 8]
        m2 = stages[6 * layer + 3][1]
        m4n = stages[6 * ((layer + 1) % n_layers)][1]
        in2 = mixbuf(2)
        barepm.append(("lin", B.DispatchTable(D[0:4], in4b[layer], Y[0:4])))
        barepm.append(("post", B.PostDispatchTable([D[4]], [Y[2]], None,
                       [(B.POST_NONE, None, hprev, [(m2.keep[0][p], m2.keep[1][p], 6, in2[p]) for p in range(2)])], [Y[4]])))
        barepm.append(("lin", B.DispatchTable([D[5], D[7]], in2, [Y[5], Y[7]])))
        barepm.append(("post", B.PostDispatchTable([D[6]], [Y[5]], None,
                       [(B.POST_NONE, None, hprev, [(m4n.keep[0][p], m4n.keep[1][p], 6, in4b[layer + 1][p]) for p in range(4)])], [Y[6]])))

    def step_barepm():
        for kind, a in barepm:
            if kind == "mix":
                B.rwkvq_token_shift_mix(a[0], hprev, B.F16, 1, d, a[1], 6)
            elif kind == "lin":
                B.rwkvq_linear_dispatch(a, 1, B.F16, B.F16)
            else:
                B.rwkvq_linear_dispatch_post(a, B.F16, B.F16)

    # and with r, k, v and the wkv step in one launch (rwkvq_rkv_wkv: the workgroup that computes a row tile
    # of the three projections steps its 16 channels); the gate projection of the 7B stack, which nothing
    # consumes, rides with W_o.  4 launches per layer + 1.
    blockf = [blockpm[0]]
    for layer in range(n_layers):
        D = dec["descs"][8 * layer: 8 * layer + 8]
        Y = dec["ys"][8 * layer: 8 * layer + 8]
        b7 = block[7 * layer: 7 * layer + 7]
        wkv_a = b7[1][1]                                        # (r, k, v, w, u, state, gated)
        post_o = blockpm[1 + 5 * layer + 2][1]
        blockf.append(("rkv", (B.RkvWkvTable(D[0:3], in4[layer][0:3], Y[0:3]), wkv_a[3], wkv_a[4], wkv_a[5], wkv_a[6])))
        m2 = stages[6 * layer + 3][1]
        in2 = [post_o.keep[2][0][3][p][3] for p in range(2)]   # the two mix outputs of the W_o launch above
        blockf.append(("post", B.PostDispatchTable([D[4], D[3]], [wkv_a[6], in4[layer][3]], None,
                       [(B.POST_NONE, None, hprev, [(m2.keep[0][p], m2.keep[1][p], 6, in2[p]) for p in range(2)]),
                        (B.POST_NONE, None)], [Y[4], Y[3]])))
        blockf.append(blockpm[1 + 5 * layer + 3])
        blockf.append(blockpm[1 + 5 * layer + 4])

    def step_blockf():
        for kind, a in blockf:
            if kind == "mix":
                B.rwkvq_token_shift_mix(a[0], hprev, B.F16, 1, d, a[1], 6)
            elif kind == "rkv":
                B.rwkvq_rkv_wkv(a[0], a[1], a[2], a[3], a[4], B.F16, B.F16)
            else:
                B.rwkvq_linear_dispatch_post(a, B.F16, B.F16)

    def step_blockpm():
        for kind, a in blockpm:
            if kind == "mix":
                B.rwkvq_token_shift_mix(a[0], hprev, B.F16, 1, d, a[1], 6)
            elif kind == "lin":
                B.rwkvq_linear_dispatch(a, 1, B.F16, B.F16)
            elif kind == "wkv":
                B.rwkvq_wkv(a[0], a[1], a[2], B.F16, 1, d, a[3], a[4], a[5], a[6])
            else:
                B.rwkvq_linear_dispatch_post(a, B.F16, B.F16)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fn()
        total_ms, _, _ = time_steps(graph.replay, 1000, 300)
        return total_ms / 1000

    ms = timed(step)
    ms_fused = timed(step_fused)
    ms_barepm = timed(step_barepm)
    ms_block7 = timed(step_block)
    ms_block = timed(step_block5)
    ms_blockpm = timed(step_blockpm)
    ms_blockf = timed(step_blockf)

    def one_step_from_empty_state(fn):
        for layer in range(n_layers):
            st = block[7 * layer + 1][1][5]
            st[:2].zero_(); st[2].fill_(-1e38)
        fn()
        torch.cuda.synchronize()
        return block[-1][1][2].clone()
    ref_out = one_step_from_empty_state(step_block5)
    same_bits = bool(torch.equal(ref_out, one_step_from_empty_state(step_blockpm)))
    # here W_o shares its launch with the gate projection, which changes how its rows' columns are split over
    # wavefronts (four instead of eight): the same operations in another order of the binary32 sums
    out_f = one_step_from_empty_state(step_blockf)
    diff_f = float((out_f.view(torch.float16).float() - ref_out.view(torch.float16).float()).abs().max())
    last = block[-1][1][2].view(torch.float16).float()
    final_ok = bool(torch.isfinite(last).all()) and float(last.abs().max()) > 0.0
    eager_ms = time_steps(step, 200, 50)[0] / 200
    return {"ms_per_step": ms_barepm, "tokens_per_s": 1e3 / ms_barepm, "value": dec["wbytes"] / (ms_barepm * 1e-3) / 1e9,
            "unit": "GB/s", "launches_per_step": len(barepm),
            "mixes_in_the_consumers": {"ms_per_step": ms_fused, "launches_per_step": len(fused)},
            "unfused": {"ms_per_step": ms, "launches_per_step": len(stages), "eager_ms_per_step": eager_ms},
            "block": {"ms_per_step": ms_blockf, "tokens_per_s": 1e3 / ms_blockf, "launches_per_step": len(blockf),
                      "max_abs_diff_to_the_other_variants": diff_f,
                      "wkv_a_launch_of_its_own": {"ms_per_step": ms_blockpm, "launches_per_step": len(blockpm),
                                                  "same_output_bits": same_bits},
                      "block_output_rms_min_max": [min(flow), max(flow)], "final_output_finite": final_ok,
                      "mixes_in_the_consumers": {"ms_per_step": ms_block, "launches_per_step": len(block5),
                                                 "same_output_bits": same_bits},
                      "separate_operators": {"ms_per_step": ms_block7, "launches_per_step": len(block)},
                      "note": "with the element-wise operators of the block: r, k, v and the wkv step with its gate in "
                              "one launch, squared ReLU and output gate applied by the GEMVs that produce their operands, "
                              "every token-shift mix taken by the GEMV that produces its input vector (4 launches per "
                              "layer + one mix pass in front); wkv_a_launch_of_its_own = the same with the wkv step as a "
                              "separate launch (5 per layer); mixes_in_the_consumers = the mixes fused into the "
                              "activation loads of the GEMVs that read them instead (5 per layer); separate_operators "
                              "= that, with each operator a launch of its own (7)"},
            "note": "same 256 matrices, data-flow order, in one HIP graph: 4 launches per layer, every token-shift mix "
                    "taken by the GEMV that produces its input vector (+ one mix pass in front); "
                    "mixes_in_the_consumers = the mixes in the activation loads of the GEMVs that read them (4 per "
                    "layer); unfused = 6 launches per layer with separate mix passes; block = with the element-wise "
                    "operators of the block between the stages"}


def batched_decode(dec, stage_ordered=True):
    """The decode stack at batches 4, 16 (streaming kernels, 2..16 rows), 32 (their 17..32-row instance) and
    64 (two passes of it, or the matrix cores: whichever the dispatcher estimates cheaper)."""
    import torch
    from paper_2505_03803_amd import binding as B
    res = {}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    for M in (4, 16, 32, 64):
        xs = [torch.randn((M, int(d.K)), device="cuda", generator=gen).to(torch.float16).view(torch.int16) for d in dec["descs"]]
        ys = [torch.empty((M, int(d.N)), dtype=torch.int16, device="cuda") for d in dec["descs"]]
        table = B.DispatchTable(dec["descs"], xs, ys)
        total, _, _ = time_steps(lambda: B.rwkvq_linear_dispatch(table, M, B.F16, B.F16), 300, 150)
        ms = total / 300
        res[f"M{M}"] = {"ms_per_step": ms, "weight_GBps": dec["wbytes"] / (ms * 1e-3) / 1e9, "tokens_per_s": M * 1e3 / ms}
        del xs, ys, table
    res["note"] = "same 256 matrices, one rwkvq_linear_dispatch call per step; weight_GBps counts the packed weights once per step"
    # The same matrices as the launches a model would make: per layer {r, k, v, g}, then o, then {k', r'}, then v'
    # (4 dispatches per layer, each waiting for the one before; no element-wise operators in between), replayed
    # from one HIP graph.  These are small launches: the streaming kernels take their column-split form.
    n_layers = len(dec["descs"]) // 8
    for M in ((4, 16) if stage_ordered else ()):
        tables = []
        for layer in range(n_layers):
            for ids in ((0, 1, 2, 3), (4,), (5, 7), (6,)):
                ds = [dec["descs"][8 * layer + i] for i in ids]
                xs = [torch.randn((M, int(d.K)), device="cuda", generator=gen).to(torch.float16).view(torch.int16) for d in ds]
                ys = [torch.empty((M, int(d.N)), dtype=torch.int16, device="cuda") for d in ds]
                tables.append((B.DispatchTable(ds, xs, ys), xs, ys))

        def step():
            for t, _, _ in tables:
                B.rwkvq_linear_dispatch(t, M, B.F16, B.F16)

        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        total, _, _ = time_steps(graph.replay, 300, 100)
        ms = total / 300
        res[f"M{M}_stage_ordered"] = {"ms_per_step": ms, "weight_GBps": dec["wbytes"] / (ms * 1e-3) / 1e9, "tokens_per_s": M * 1e3 / ms,
                                      "launches_per_step": len(tables)}
        del tables, graph
    return res


def prefill_block_step(pf, n_layers, M):
    """A chunk of M tokens through the stack in data-flow order with the block's element-wise operators
    (App. A.1): per layer  mix pass (4 projections) -> {r, k, v, g} -> wkv with its gate -> W_o -> mix
    pass (2) -> {k', r'} -> squared ReLU -> W'_v -> gate.  Same matrices as the grouped prefill figure;
    shows what the dependencies and the element-wise passes cost on top of it."""
    import torch
    from paper_2505_03803_amd import binding as B
    from paper_2505_03803_amd import synth
    d = int(pf["descs"][0].K)
    ffn = pf["ys"][5].shape[1]
    rng = np.random.default_rng(4100)
    t16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda()
    buf = lambda n: torch.zeros((M, n), dtype=torch.int16, device="cuda")
    h = t16(synth.gen_activations(rng, M, d, "bf16"))
    hprev = t16(synth.gen_activations(rng, 1, d, "bf16")[0])
    mix4, mix2, gated, sq = [buf(d) for _ in range(4)], [buf(d) for _ in range(2)], buf(d), buf(ffn)
    outs = [buf(d), buf(d)]                                   # block outputs, alternating
    stages = []
    src = h
    for layer in range(n_layers):
        D = pf["descs"][8 * layer: 8 * layer + 8]
        Y = pf["ys"][8 * layer: 8 * layer + 8]
        mk = lambda P, o: B.MixTable([torch.from_numpy(rng.integers(0, 64, size=d // 2, dtype=np.uint8)).cuda() for _ in range(P)],
                                     [t16(synth.gen_codebook(rng, 64)) for _ in range(P)], o)
        _, _, _, w, u = synth.gen_block_inputs(rng, 1, d, "bf16")
        st = np.zeros((3, d), dtype=np.float32); st[2] = -1e38
        out = outs[layer & 1]
        stages += [("mix", (src, mk(4, mix4))), ("lin", B.DispatchTable(D[0:4], mix4, Y[0:4])),
                   ("wkv", (Y[0], Y[1], Y[2], torch.from_numpy(w).cuda(), torch.from_numpy(u).cuda(), torch.from_numpy(st).cuda(), gated)),
                   ("lin", B.DispatchTable([D[4]], [gated], [Y[4]])),
                   ("mix", (Y[4], mk(2, mix2))), ("lin", B.DispatchTable([D[5], D[7]], mix2, [Y[5], Y[7]])),
                   ("relu2", (Y[5], sq)), ("lin", B.DispatchTable([D[6]], [sq], [Y[6]])), ("gate", (Y[7], Y[6], out))]
        src = out

    def launch(kind, a):
        if kind == "mix":
            B.rwkvq_token_shift_mix(a[0], hprev, B.BF16, M, d, a[1], 6)
        elif kind == "lin":
            B.rwkvq_linear_dispatch(a, M, B.BF16, B.BF16)
        elif kind == "wkv":
            B.rwkvq_wkv(a[0], a[1], a[2], B.BF16, M, d, a[3], a[4], a[5], a[6])
        elif kind == "relu2":
            B.rwkvq_relu2(a[0], B.BF16, M * ffn, a[1])
        else:
            B.rwkvq_sigmoid_gate(a[0], a[1], B.BF16, M * d, a[2])

    # every block's output back to unit rms (a per-layer factor on W'_v), as in the token step
    flow = []
    for layer in range(n_layers):
        for kind, a in stages[9 * layer: 9 * layer + 9]:
            launch(kind, a)
        torch.cuda.synchronize()
        out = stages[9 * layer + 8][1][2]
        scale_weights(pf["keep"][0][8 * layer + 6], 1.0 / max(rms16(out, True), 1e-6))
        for kind, a in stages[9 * layer + 7: 9 * layer + 9]:
            launch(kind, a)
        torch.cuda.synchronize()
        flow.append(rms16(out, True))

    def step():
        for kind, a in stages:
            launch(kind, a)

    total, _, _ = time_steps(step, 10, 3)
    last = stages[-1][1][2].view(torch.bfloat16).float()
    final_ok = bool(torch.isfinite(last).all()) and float(last.abs().max()) > 0.0
    ms = total / 10
    return {"ms_per_step": ms, "tokens_per_s": M * 1e3 / ms, "value": pf["flops"] / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
            "calls_per_step": len(stages), "block_output_rms_min_max": [min(flow), max(flow)], "final_output_finite": final_ok,
            "note": "the same matrices in data-flow order, 9 calls per layer: token-shift mix passes, matrix-core GEMMs, "
                    "time-parallel wkv with its gate, squared ReLU, output gate; value counts the GEMM FLOP only"}


class TimedRegion:
    """W untimed steps, then exactly K steps bracketed by synchronize + HIP events on the current stream
    (one event per step).  The steps are enqueued by the constructor; `result()` waits for them and reads
    the events.  Enqueueing a second region before reading the first keeps the device busy between them:
    reading some thousand events takes the host tens of milliseconds, and after an idle gap of that length
    the device runs its next ~100 decode steps through a clock transient."""

    def __init__(self, run, steps: int, warmup: int):
        import torch
        for _ in range(warmup):
            run()
        torch.cuda.synchronize()
        self.steps = steps
        self.ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        self.t0 = time.perf_counter()
        self.ev[0].record()
        for i in range(steps):
            run()
            self.ev[i + 1].record()
        self.res = None

    def result(self):
        """(total ms over the K steps, per-step ms list, host wall ms)"""
        import torch
        if self.res is None:
            self.ev[-1].synchronize()
            wall_ms = (time.perf_counter() - self.t0) * 1e3
            torch.cuda.synchronize()
            ev = self.ev
            self.res = (ev[0].elapsed_time(ev[-1]), [ev[i].elapsed_time(ev[i + 1]) for i in range(self.steps)], wall_ms)
        return self.res


def time_steps(run, steps: int, warmup: int):
    return TimedRegion(run, steps, warmup).result()


def slices_of(per, n=10):
    return [round(float(np.mean(c)), 4) for c in np.array_split(np.asarray(per), n)] if len(per) >= n else None


def hbm_roofline(kernel, bytes_per_step, ms, launches=1, traffic_key=None, traffic_applies=True, note=None):
    """Roofline record of an HBM-bound leg: achieved = algorithmic bytes of one launch / average launch
    duration (HIP events on the launch stream around each step of the timed region, / launches per step)."""
    r = {"kernel": kernel, "bound": "hbm", "achieved": bytes_per_step / launches / (ms / launches * 1e-3) / 1e9,
         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": bytes_per_step / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
         "traffic": None, "algorithmic_bytes_per_launch": bytes_per_step / launches, "avg_launch_ms": ms / launches}
    if traffic_key:
        r["traffic"], r["traffic_source"] = traffic(traffic_key, traffic_applies)
    if note:
        r["note"] = note
    return r


def decode_leg(stack, M, steps, warmup, kernel, traffic_key=None, traffic_applies=True, y_dtype=None, enqueue_only=False):
    """Time `steps` grouped dispatches of a resident stack at batch M after `warmup` untimed ones.  With
    enqueue_only the steps are enqueued and a function that returns the record is handed back."""
    from paper_2505_03803_amd import binding as B
    yd = B.F16 if y_dtype is None else y_dtype
    run = lambda: B.rwkvq_linear_dispatch(stack["table"], M, stack["x_dtype"], yd)
    region = TimedRegion(run, steps, warmup)
    launches = (stack["n_mats"] + DECODE_MATS_PER_LAUNCH - 1) // DECODE_MATS_PER_LAUNCH
    wbytes = stack["wbytes"]

    def record():
        total_ms, per, wall_ms = region.result()
        ms = total_ms / steps
        gbs = wbytes / (ms * 1e-3) / 1e9
        return {"value": gbs, "unit": "GB/s", "steps": steps, "warmup": warmup, "ms_per_step": ms,
                "pct_hbm_peak": 100.0 * gbs / HBM_PEAK_GBS, "tokens_per_s": M * 1e3 / ms,
                "ms_per_step_min": min(per), "ms_per_step_median": float(np.median(per)),
                "ms_per_step_slices": slices_of(per), "wall_ms_per_step": wall_ms / steps,
                "launches_per_step": launches,
                "roofline": hbm_roofline(kernel, wbytes, ms, launches, traffic_key, traffic_applies)}
    return record if enqueue_only else record()


def with_batch(stack, M, y_dtype):
    """The same resident matrices with fresh activations / outputs for batch M (drawn on the GPU)."""
    import torch
    from paper_2505_03803_amd import binding as B
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7000 + M)
    tdt = torch.bfloat16 if stack["x_dtype"] == B.BF16 else torch.float16
    xs = [torch.randn((M, int(d.K)), device="cuda", generator=gen, dtype=torch.float32).to(tdt).view(torch.int16) for d in stack["descs"]]
    ys = [torch.empty((M, int(d.N)), dtype=torch.float32 if y_dtype == B.F32 else torch.int16, device="cuda") for d in stack["descs"]]
    out = dict(stack)
    out.update(table=B.DispatchTable(stack["descs"], xs, ys), keep=(stack["keep"][0], xs, ys), ys=ys,
               flops=sum(2 * M * int(d.N) * int(d.K) for d in stack["descs"]))
    return out


def single_matrix_legs(config, min_copies, steps, warmup):
    """Configurations 1 and 2: ONE matrix, batch 1.  Its working set (0.4 / 6.4 MB) is far below the 256 MB
    memory-side cache, so three figures: cache-hot (the same buffers every call), HBM-cold (rotating through
    `min_copies` copies at distinct addresses, more than twice that cache in all, one call per copy) and
    grouped (all copies in one rwkvq_linear_dispatch: a lone call of 0.05 / 0.8 us of traffic measures launch
    latency, not the kernel).  Only the cold figures say anything about HBM."""
    import torch
    from paper_2505_03803_amd import binding as B
    from paper_2505_03803_amd import synth
    mat, x = (synth.config1 if config == 1 else synth.config2)(1)
    dm0 = B.upload(mat, native=True)
    clone = lambda t: None if t is None else t.clone()
    dms = [dm0] + [B.DeviceMatrix(dm0.kind, dm0.layout, dm0.N, dm0.K, dm0.kbits, clone(dm0.codes), clone(dm0.scales), None,
                                  clone(dm0.codebooks), dm0.packed_bytes) for _ in range(min_copies - 1)]
    xd = [torch.from_numpy(x.view(np.int16)).cuda() for _ in range(min_copies)]
    yd = [torch.empty((1, mat.N), dtype=torch.int16, device="cuda") for _ in range(min_copies)]
    descs = [d.desc() for d in dms]
    singles = [B.DispatchTable([descs[i]], [xd[i]], [yd[i]]) for i in range(min_copies)]
    grouped = B.DispatchTable(descs, xd, yd)
    wb = mat.packed_bytes
    res = {"workload": ("configs[0]: one SQ matrix 1024 x 1024, 3-bit g128" if config == 1 else
                        "configs[1]: one VQ matrix 4096 x 4096, d=2, 6-bit indices, 256 x 256 blocks") + ", batch 1, fp16 activations",
           "weight_bytes": wb, "copies": min_copies, "rotated_set_bytes": wb * min_copies}
    # cache-hot: the same matrix every call
    tot, per, _ = time_steps(lambda: B.rwkvq_linear_dispatch(singles[0], 1, B.F16, B.F16), steps, warmup)
    ms = tot / steps
    res["cache_hot"] = {"ms_per_call": ms, "value": wb / (ms * 1e-3) / 1e9, "unit": "GB/s", "calls": steps,
                        "note": "launch-latency bound; served by the caches, not a statement about HBM"}
    # HBM-cold: one call per copy, rotating
    it = [0]
    def rot():
        B.rwkvq_linear_dispatch(singles[it[0] % min_copies], 1, B.F16, B.F16)
        it[0] += 1
    n_calls = max(steps, min_copies)
    tot, per, _ = time_steps(rot, n_calls, min(warmup, min_copies))
    ms = tot / n_calls
    res["hbm_cold_rotated"] = {"ms_per_call": ms, "value": wb / (ms * 1e-3) / 1e9, "unit": "GB/s", "calls": n_calls,
                               "pct_hbm_peak": 100.0 * wb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                               "note": "one launch per call on cold data: bound by launch latency (%.1f us of traffic at peak)" % (wb / 8e12 * 1e6)}
    # grouped: all copies in one dispatch
    g_steps = max(20, steps // 10)
    tot, per, _ = time_steps(lambda: B.rwkvq_linear_dispatch(grouped, 1, B.F16, B.F16), g_steps, 300)   # ~50 ms of warm-up: past the clock transient
    ms = tot / g_steps
    launches = (min_copies + DECODE_MATS_PER_LAUNCH - 1) // DECODE_MATS_PER_LAUNCH
    res["grouped"] = {"ms_per_step": ms, "value": wb * min_copies / (ms * 1e-3) / 1e9, "unit": "GB/s", "steps": g_steps,
                      "pct_hbm_peak": 100.0 * wb * min_copies / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "launches_per_step": launches,
                      "roofline": hbm_roofline(DECODE_KERNEL, wb * min_copies, ms, launches)}
    return res


def cpu_baseline_prefill(n_rows=256, M=2048, n_layers_total=32):
    """The oracle on a bounded sample of the prefill workload: the 8 matrices of the first layer of the
    configuration-4 stack, the first n_rows of the M token rows (dequantize to binary32, naive binary32 sums)."""
    from oracle import rwkvq_oracle as orc
    from paper_2505_03803_amd import synth
    secs, flop = 0.0, 0
    for mat, x in synth.stack(4, n_rows, n_layers=1):
        xf = orc.widen(x, "bf16")
        t = time.perf_counter()
        orc.linear(mat, xf, "f32")
        secs += time.perf_counter() - t
        flop += 2 * n_rows * mat.N * mat.K
    return {"value": flop / secs / 1e12, "unit": "TFLOP/s", "cores": orc.threads(), "kind": "oracle",
            "sample": f"first layer (8 matrices) of the configuration-4 stack, first {n_rows} of {M} token rows: "
                      f"{flop / 1e9:.1f} GFLOP in {secs:.2f} s of oracle time",
            "extrapolated_s_per_step": secs * (M / n_rows) * n_layers_total,
            "extrapolation": f"linear in rows and layers: x {M // n_rows} rows x {n_layers_total} layers (an extrapolation, not a measurement)"}


def cpu_baseline(n_layers, min_seconds=10.0, max_passes=8):
    """The oracle as it stands on the host cores: decode (M = 1) over the first n_layers layers of
    the same stack (all 32 by default = the whole workload), repeated until about min_seconds of
    oracle time have been measured."""
    from oracle import rwkvq_oracle as orc
    from paper_2505_03803_amd import synth
    nbytes, secs, passes = 0, 0.0, 0
    while secs < min_seconds and passes < max_passes:
        for mat, x in synth.stack(3, 1, n_layers=n_layers):
            xf = orc.widen(x, "f16")
            t = time.perf_counter()
            orc.linear(mat, xf, "f32")
            secs += time.perf_counter() - t
            nbytes += mat.packed_bytes
        passes += 1
    return {"value": nbytes / secs / 1e9, "unit": "GB/s", "cores": orc.threads(), "kind": "oracle",
            "sample": f"decode M=1, {passes} pass(es) over the first {n_layers} of 32 layers of the "
                      f"RWKV-6-7B-shaped stack ({nbytes} packed weight bytes in {secs:.2f} s of oracle time)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200, help="timed steps of the headline decode leg")
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--layers", type=int, default=32, help="layers of the stack (32 = the full workload)")
    ap.add_argument("--prefill-steps", type=int, default=40)
    ap.add_argument("--prefill-warmup", type=int, default=10)
    ap.add_argument("--steady-steps", type=int, default=2000, help="timed steps of the steady-state decode leg")
    ap.add_argument("--steady-warmup", type=int, default=500)
    ap.add_argument("--skip-steady", action="store_true")
    ap.add_argument("--skip-single", action="store_true", help="skip the single-matrix legs (configurations 1 and 2)")
    ap.add_argument("--skip-config5", action="store_true")
    ap.add_argument("--config5-layers", type=int, default=48)
    ap.add_argument("--config5-steps", type=int, default=1000, help="timed batch-1 steps of the configuration-5 leg (batch 16: 0.6 x)")
    ap.add_argument("--skip-prefill", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--skip-proxy", action="store_true", help="skip the proxy and encoder legs")
    ap.add_argument("--skip-encode", action="store_true")
    ap.add_argument("--skip-mu", action="store_true", help="skip the element-wise multiplication leg")
    ap.add_argument("--skip-batched", action="store_true", help="skip the small-batch decode figures")
    ap.add_argument("--skip-sequential", action="store_true", help="skip the legs replayed from a HIP graph: the dependency-ordered token step and the stage-ordered batched steps")
    ap.add_argument("--proxy-layers", type=int, default=8, help="layers of dense bf16 weights the proxy leg scans per call")
    ap.add_argument("--cpu-layers", type=int, default=32)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (--gpus 1); a multi-GPU figure is not "
                 "part of it (the design notes say how the path would shard).")

    import torch
    from paper_2505_03803_amd import binding as B
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    B.lib()                                    # fails loudly if the HIP library is missing

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.int32, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    # ---------------- decode legs: configuration 3
    # Order: the steady-state leg first (its own long warm-up takes the device through the power-management
    # transient that follows idle: step time 0.47 -> 0.69 -> 0.49 ms over the first ~100 steps), then, directly
    # after it, the headline with exactly the --warmup / --steps asked for.
    t = time.time()
    dec = build_stack(3, 1, args.layers, gpu_activations=False, y_dtype=B.F16)
    log(f"decode stack resident: {dec['n_mats']} matrices, {dec['wbytes'] / 1e9:.3f} GB packed, {time.time() - t:.1f} s")
    full = args.layers == 32
    steady = None
    if not args.skip_steady:
        steady = decode_leg(dec, 1, args.steady_steps, args.steady_warmup, DECODE_KERNEL, "decode_config3", full, enqueue_only=True)
    head = decode_leg(dec, 1, args.steps, args.warmup, DECODE_KERNEL, "decode_config3", full)   # enqueued behind the steady leg
    if steady:
        steady = steady()
        steady["note"] = ("the same step as the headline, timed over its own long region; enqueued first, the headline's warm-up and "
                          "timed steps directly behind it on the same stream, so that they are not taken inside the clock "
                          "transient that follows an idle device")
    out = {
        "metric": "dequant-GEMV weight GB/s (% of HBM peak) + prefill TFLOP/s, RWKV-6-7B shapes",
        "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "configs[2]: RWKV-6-7B-shaped decode layer stack, %d layers x 8 matrices, "
                               "d=4096 ffn=14336, batch 1, SQ 3-bit g128 / VQ d=2 6-bit per matrix "
                               "(Bernoulli 0.5, seed 2), fp16 activations" % args.layers,
                   "weight_bytes_per_step": dec["wbytes"], "matrices": dec["n_mats"],
                   "launches_per_step": head["launches_per_step"],
                   "timed_after": "the steady_state leg" if steady else "stack upload (device idle before)"},
        "pct_hbm_peak": head["pct_hbm_peak"], "tokens_per_s": head["tokens_per_s"],
        "ms_per_step_min": head["ms_per_step_min"], "ms_per_step_median": head["ms_per_step_median"],
        # mean of ten equal slices of the timed steps, in order: shows drift
        "ms_per_step_slices": head["ms_per_step_slices"], "wall_ms_per_step": head["wall_ms_per_step"],
        "roofline": head["roofline"],
    }
    if steady:
        out["steady_state"] = steady
    # ---------------- the same matrices at small batches (one grouped call per step)
    if not args.skip_batched:
        out["decode_batched"] = batched_decode(dec, stage_ordered=not args.skip_sequential)   # the graph legs go together
    # ---------------- the same matrices in data-flow order, one HIP graph per token step
    if not args.skip_sequential:
        unit_gain(dec, 1)
        out["sequential_step"] = sequential_step(dec, args.layers)
    del dec
    torch.cuda.empty_cache()

    # ---------------- configurations 1 and 2: one matrix, cache-hot / HBM-cold rotated / grouped
    if not args.skip_single:
        out["config1"] = single_matrix_legs(1, 1600, 2000, 200)      # 1600 x 0.43 MB = 682 MB > 2 x 256 MB
        out["config2"] = single_matrix_legs(2, 104, 1000, 100)       # 104 x 6.36 MB = 661 MB
        torch.cuda.empty_cache()

    # ---------------- prefill leg: configuration 4
    if not args.skip_prefill:
        t = time.time()
        pf = build_stack(4, 2048, args.layers, gpu_activations=True, y_dtype=B.BF16)
        log(f"prefill stack resident: {pf['n_mats']} matrices, {pf['flops'] / 1e12:.2f} TFLOP/step, {time.time() - t:.1f} s")
        runp = lambda: B.rwkvq_linear_dispatch(pf["table"], 2048, pf["x_dtype"], B.BF16)
        ptotal, pper, _ = time_steps(runp, args.prefill_steps, args.prefill_warmup)
        pms = ptotal / args.prefill_steps
        tflops = pf["flops"] / (pms * 1e-3) / 1e12
        out["prefill"] = {"value": tflops, "unit": "TFLOP/s", "ms_per_step": pms, "steps": args.prefill_steps,
                          "warmup": args.prefill_warmup, "ms_per_step_slices": slices_of(pper, 5),
                          "dtype": "bf16", "tokens_per_s": 2048 * 1e3 / pms,
                          "pct_mfma_peak": 100.0 * tflops / MFMA_BF16_PEAK_TFLOPS,
                          "workload": "configs[3]: same stack recipe (seed 3), M=2048 tokens, bf16 "
                                      "activations, %d layers" % args.layers,
                          "flop_per_step": pf["flops"]}
        tr, src = traffic("prefill_config4", full)
        out["roofline_prefill"] = {"kernel": PREFILL_KERNEL, "bound": "mfma", "achieved": tflops,
                                   "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": tflops / MFMA_BF16_PEAK_TFLOPS,
                                   # FETCH_SIZE x 2 + WRITE_SIZE per launch, mean of the four launches of a step
                                   "traffic": tr, "traffic_source": src, "launches_per_step": 4,
                                   "avg_launch_ms": pms / 4}
        if not args.skip_sequential:
            unit_gain(pf, 2048, bf16=True)
            out["prefill"]["block"] = prefill_block_step(pf, args.layers, 2048)
        del pf, runp
        torch.cuda.empty_cache()
        if not args.skip_cpu:
            out["prefill"]["cpu_baseline"] = cpu_baseline_prefill()

    # ---------------- configuration 5: the 14B-class stack (SQ / VQ-6 / VQ-8, bf16 activations)
    if not args.skip_config5:
        t = time.time()
        c5 = build_stack(5, 1, args.config5_layers, gpu_activations=False, y_dtype=B.BF16)
        log(f"configuration 5 resident: {c5['n_mats']} matrices, {c5['wbytes'] / 1e9:.3f} GB packed, {time.time() - t:.1f} s")
        rec = {"workload": "configs[4]: 14B-class stack, %d layers x 8 matrices, d=5120 ffn=17920, SQ 3-bit g128 / VQ d=2 "
                           "6-bit / VQ d=2 8-bit per matrix (seed 4), bf16 activations" % args.config5_layers,
               "weight_bytes_per_step": c5["wbytes"], "matrices": c5["n_mats"]}
        rec["decode_M1"] = decode_leg(c5, 1, args.config5_steps, max(1, args.config5_steps * 3 // 10), DECODE_KERNEL, "decode_config5_M1",
                                      args.config5_layers == 48, y_dtype=B.BF16)
        c16 = with_batch(c5, 16, B.BF16)
        rec["decode_M16"] = decode_leg(c16, 16, max(1, args.config5_steps * 6 // 10), max(1, args.config5_steps * 2 // 10), DECODE16_KERNEL,
                                       "decode_config5_M16", args.config5_layers == 48, y_dtype=B.BF16)
        del c16
        torch.cuda.empty_cache()
        c4k = with_batch(c5, 4096, B.BF16)
        runp = lambda: B.rwkvq_linear_dispatch(c4k["table"], 4096, c4k["x_dtype"], B.BF16)
        ptotal, pper, _ = time_steps(runp, 8, 3)
        pms = ptotal / 8
        tflops = c4k["flops"] / (pms * 1e-3) / 1e12
        launches = sum((n + 63) // 64 for n in np.bincount([0 if int(d.kind) == B.SQ else (1 if int(d.kbits) == 6 else 2) for d in c4k["descs"]], minlength=3) if n)
        rec["prefill_M4096"] = {"value": tflops, "unit": "TFLOP/s", "ms_per_step": pms, "steps": 8, "warmup": 3, "dtype": "bf16",
                                "tokens_per_s": 4096 * 1e3 / pms, "pct_mfma_peak": 100.0 * tflops / MFMA_BF16_PEAK_TFLOPS,
                                "flop_per_step": c4k["flops"], "ms_per_step_slices": slices_of(pper, 4),
                                "roofline": {"kernel": PREFILL_KERNEL, "bound": "mfma", "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS,
                                             "unit": "TFLOP/s", "frac": tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                                             "launches_per_step": int(launches), "avg_launch_ms": pms / launches}}
        out["config5"] = rec
        del c5, c4k, runp
        torch.cuda.empty_cache()

    # ---------------- proxy leg: P_c, P_f, phi of the dense bf16 matrices of some layers
    if not args.skip_proxy:
        from paper_2505_03803_amd import synth
        shapes = [(N, K) for _ in range(args.proxy_layers) for _, N, K in synth.layer_shapes(4096, 14336)]
        gen = torch.Generator(device="cuda")
        gen.manual_seed(2000)
        mats = [(torch.randn(sh, device="cuda", generator=gen) * 0.02).to(torch.bfloat16).view(torch.int16)
                for sh in shapes]
        n = len(mats)
        table = B.ProxyTable(mats, shapes)
        wsp = torch.empty(B.rwkvq_proxy_workspace_bytes(n) // 4, dtype=torch.int32, device="cuda")
        pout = torch.empty(2 * n, dtype=torch.float64, device="cuda")
        pphi = torch.empty(n + 3, dtype=torch.int32, device="cuda")
        runx = lambda: B.rwkvq_proxy(table, B.BF16, 5, 1.5, 50.0, wsp, pout, pphi)
        xcalls = 300
        xtotal, xper, _ = time_steps(runx, xcalls, 100)
        xms = xtotal / xcalls
        xbytes = sum(a * b * 2 for a, b in shapes)
        launches = (n + 63) // 64
        out["proxy"] = {"value": xbytes / (xms * 1e-3) / 1e9, "unit": "GB/s", "ms_per_call": xms, "calls": xcalls,
                        "dtype": "f64", "matrices": n, "dense_weight_bytes_per_call": xbytes,
                        "pct_hbm_peak": 100.0 * xbytes / (xms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "workload": "dense bf16 N(0, 0.02) weights of %d RWKV-6-7B-shaped layers "
                                    "(d=4096, ffn=14336), K = 5 terms" % args.proxy_layers}
        out["roofline_proxy"] = {"kernel": PROXY_KERNEL, "bound": "hbm",
                                 "achieved": xbytes / (xms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": xbytes / (xms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                 # FETCH_SIZE x 2 + WRITE_SIZE of the set kernel for the default 8 layers
                                 # (profiles/proxy_kernel_trace_and_traffic_7b_layers.txt)
                                 "traffic": traffic("proxy_8_layers", args.proxy_layers == 8)[0],
                                 "traffic_source": TRAFFIC["proxy_8_layers"][1],
                                 "algorithmic_bytes_per_launch": xbytes / launches,
                                 "avg_launch_ms": xms / launches,
                                 "note": "achieved = dense weight bytes / time of the whole call (clear + set + "
                                         "final kernels); the set kernel alone is the HBM-bound pass"}
        if not args.skip_cpu:
            # the oracle (sort-based definition) on the first matrices, about ten seconds of host time
            from oracle import proxy_oracle as PO
            secs, nb, k = 0.0, 0, 0
            while secs < 8.0 and k < n:
                host = mats[k].cpu().numpy().view(np.uint16)
                t = time.perf_counter()
                PO.proxies(PO.widen16(host, "bf16"))
                secs += time.perf_counter() - t
                nb += host.size * 2
                k += 1
            out["proxy"]["cpu_baseline"] = {"value": nb / secs / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                            "sample": "first %d of the %d matrices (%d dense bytes in %.2f s)" % (k, n, nb, secs)}
        # ---------------- the proxy for binary32 matrices: a real sort (four radix passes) per matrix
        shapes32 = [(N, K) for _, N, K in synth.layer_shapes(4096, 14336)]
        mats32 = [torch.randn(sh, device="cuda", generator=gen) * 0.02 for sh in shapes32]
        table32 = B.ProxyTable(mats32, shapes32)
        wsp32 = torch.empty((B.rwkvq_proxy_workspace_size(table32, B.F32) + 3) // 4, dtype=torch.int32, device="cuda")
        run32 = lambda: B.rwkvq_proxy(table32, B.F32, 5, 1.5, 50.0, wsp32, pout, pphi)
        t32, _, _ = time_steps(run32, 10, 3)
        ms32 = t32 / 10
        nw32 = sum(a * b for a, b in shapes32)
        alg32 = nw32 * 36                      # per weight: 4 passes x (4 B read + 4 B written) + 4 B for the pass over the sorted keys
        out["proxy_f32"] = {"value": nw32 / (ms32 * 1e-3) / 1e9, "unit": "G weights/s", "ms_per_call": ms32, "calls": 10, "dtype": "f64",
                            "matrices": len(shapes32), "weights_per_call": nw32,
                            "workload": "dense binary32 N(0, 0.02) weights of one RWKV-6-7B-shaped layer (8 matrices), K = 5 terms, "
                                        "sorted by a four-pass radix sort, one matrix after another",
                            "roofline": {"kernel": "rwkvq::sort_scatter_kernel", "bound": "hbm", "achieved": alg32 / (ms32 * 1e-3) / 1e9,
                                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": alg32 / (ms32 * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                         "traffic": None, "algorithmic_bytes_per_call": alg32,
                                         "note": "algorithmic bytes = 36 per weight (4 passes x 8 B + 4 B); the histogram step re-reads "
                                                 "the keys once per pass on top of that; achieved is over the whole call (18 launches per matrix)"}}
        if not args.skip_cpu:
            from oracle import proxy_oracle as PO
            host32 = mats32[0].cpu().numpy()
            t = time.perf_counter()
            PO.proxies(host32.astype(np.float64))
            secs = time.perf_counter() - t
            out["proxy_f32"]["cpu_baseline"] = {"value": host32.size / secs / 1e9, "unit": "G weights/s", "cores": 1, "kind": "oracle",
                                                "sample": "the first matrix (4096 x 4096) in %.2f s" % secs}
        del mats32, table32, wsp32
        torch.cuda.empty_cache()
        # ---------------- encoder leg: the same dense matrices -> SQ codes, and -> 6-bit VQ indices
        if not args.skip_encode:
            Nmax = max(a * b for a, b in shapes)
            codes = torch.empty(Nmax * 3 // 32, dtype=torch.int32, device="cuda")
            sc = torch.empty(Nmax // 128, dtype=torch.int16, device="cuda")
            zr = torch.empty_like(sc)
            idx = torch.empty(Nmax // 2 * 6 // 32, dtype=torch.int32, device="cuda")
            cbs = (torch.randn(Nmax // 65536 * 64 * 2, device="cuda", generator=gen) * 0.02).to(torch.float16).view(torch.int16)

            def run_sq():
                for m, (N_, K_) in zip(mats, shapes):
                    B.rwkvq_sq_encode(m, B.BF16, N_, K_, 3, 128, codes, sc, zr)

            def run_vq():
                for m, (N_, K_) in zip(mats, shapes):
                    B.rwkvq_vq_assign(m, B.BF16, cbs, N_, K_, 2, 6, 256, 256, idx)

            st, _, _ = time_steps(run_sq, 30, 10)
            sms = st / 30
            vt, _, _ = time_steps(run_vq, 10, 3)
            vms = vt / 10
            nw = sum(a * b for a, b in shapes)
            sq_bytes = nw * 2 + nw * 3 // 8 + nw // 128 * 4          # dense in, codes + scale + zero out
            vq_flop = (nw // 2) * 64 * 5                             # 2 sub, 2 mul, 1 add per pair and entry
            out["encode"] = {
                "sq": {"value": sq_bytes / (sms * 1e-3) / 1e9, "unit": "GB/s", "ms_per_step": sms, "dtype": "f32",
                       "bytes_per_step": sq_bytes},
                "vq6": {"value": vq_flop / (vms * 1e-3) / 1e12, "unit": "TFLOP/s", "ms_per_step": vms, "dtype": "f32",
                        "flop_per_step": vq_flop},
                "workload": "the proxy leg's %d dense bf16 matrices: round-to-nearest SQ (3 bit, g128) and "
                            "nearest-entry assignment to 64-entry codebooks" % n}
            out["roofline_sq_encode"] = {"kernel": "rwkvq::sq_encode_kernel", "bound": "hbm",
                                         "achieved": sq_bytes / (sms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": sq_bytes / (sms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                                         "avg_launch_ms": sms / n}
            out["roofline_vq_assign"] = {"kernel": "rwkvq::vq_assign_kernel<6>", "bound": "alu",
                                         "achieved": vq_flop / (vms * 1e-3) / 1e12, "peak": 157.3, "unit": "TFLOP/s",
                                         "frac": vq_flop / (vms * 1e-3) / 1e12 / 157.3, "traffic": None,
                                         "avg_launch_ms": vms / n,
                                         "note": "no step of the distance is a fused multiply-add (each is rounded "
                                                 "separately), so the reachable rate is half the FMA-counted peak"}
            del codes, sc, zr, idx, cbs
        del mats, table, wsp, pout, pphi
        torch.cuda.empty_cache()

    # ---------------- element-wise multiplication leg: token-shift mix with VQ weights, and its calibration
    if not args.skip_mu:
        from paper_2505_03803_amd import synth
        d, M, L = 4096, 2048, args.layers
        rng = np.random.default_rng(3000)
        tdev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
        x = tdev(synth.gen_activations(rng, M, d, "bf16"))
        xprev = tdev(synth.gen_activations(rng, 1, d, "bf16")[0])
        # per layer: five mixes of the time-mixing block and two of the channel-mixing block
        tables, keep = [], []
        outs5 = [torch.empty((M, d), dtype=torch.int16, device="cuda") for _ in range(5)]
        for layer in range(L):
            for P in (5, 2):
                idx = [tdev(rng.integers(0, 64, size=d // 2, dtype=np.uint8)) for _ in range(P)]
                cbs = [tdev(synth.gen_codebook(rng, 64)) for _ in range(P)]
                tables.append(B.MixTable(idx, cbs, outs5[:P]))
        def run_mix():
            for t in tables:
                B.rwkvq_token_shift_mix(x, xprev, B.BF16, M, d, t, 6)
        mt, _, _ = time_steps(run_mix, 30, 10)
        mms = mt / 30
        mix_bytes = L * (6 + 3) * M * d * 2 + L * 7 * (d // 2 + 256)     # x once per call + the outputs; indices, codebooks
        # calibration of one layer-set: representative activation (128 samples) and 7 L codebooks
        cal = tdev(synth.gen_calibration(rng, 128, d, "bf16"))
        xbar = torch.empty(d, dtype=torch.float32, device="cuda")
        run_clip = lambda: B.rwkvq_clip_mean(cal, B.BF16, 128, d, 1.0, xbar)
        ct, _, _ = time_steps(run_clip, 10, 3)
        nt = 7 * L
        mus = [tdev(synth.gen_mu(rng, d, "bf16")) for _ in range(nt)]
        cb0 = [tdev(synth.gen_codebook(rng, 64)) for _ in range(nt)]
        idxo = [torch.empty(d // 2, dtype=torch.uint8, device="cuda") for _ in range(nt)]
        run_cb = lambda: B.rwkvq_mu_codebook(mus, [xbar] * nt, [d] * nt, B.BF16, 6, 10, cb0, idxo)
        kt, _, _ = time_steps(run_cb, 5, 2)
        out["mu"] = {"mix": {"value": mix_bytes / (mms * 1e-3) / 1e9, "unit": "GB/s", "ms_per_step": mms, "dtype": "f32",
                             "bytes_per_step": mix_bytes, "calls_per_step": 2 * L},
                     "clip_mean_ms": ct / 10, "codebook_ms": kt / 5, "codebook_tensors": nt, "codebook_iters": 10,
                     "workload": "%d layers x (5 + 2) token-shift mixes of M=2048 x d=4096 bf16 activations with "
                                 "6-bit VQ mix weights; calibration: 128 samples x 4096, %d weight tensors of 4096" % (L, nt)}
        out["roofline_mix"] = {"kernel": "rwkvq::token_shift_mix_kernel", "bound": "hbm",
                               "achieved": mix_bytes / (mms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                               "frac": mix_bytes / (mms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                               # mean per call (profiles/prefill_and_mix_hbm_traffic.txt)
                               "traffic": traffic("mix_per_call")[0], "traffic_source": TRAFFIC["mix_per_call"][1],
                               "algorithmic_bytes_per_launch": mix_bytes / (2 * L),
                               "avg_launch_ms": mms / (2 * L)}
        if not args.skip_cpu:
            from oracle import mu_oracle as MO
            from oracle import rwkvq_oracle as orc
            xs = orc.widen(x[:256].cpu().numpy().view(np.uint16), "bf16")
            xp = orc.widen(xprev.cpu().numpy().view(np.uint16), "bf16")
            m_hat = rng.uniform(0, 1, d).astype(np.float16).astype(np.float32)
            secs, nb = 0.0, 0
            while secs < 3.0:
                t = time.perf_counter()
                MO.narrow(MO.token_shift_mix(xs, xp, m_hat), "bf16")
                secs += time.perf_counter() - t
                nb += 2 * 256 * d * 2
            out["mu"]["cpu_baseline"] = {"value": nb / secs / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                         "sample": "one projection, 256 of the 2048 rows, repeated for %.1f s" % secs}
        del tables, mus, cb0, idxo, outs5, x, cal
        torch.cuda.empty_cache()

    # ---------------- CPU oracle baseline (reported, not a target)
    if not args.skip_cpu:
        out["cpu_baseline"] = cpu_baseline(args.cpu_layers)

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
