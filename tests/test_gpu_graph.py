"""The linear-layer dispatch, the token-shift mix and a block's token step recorded into a HIP graph
(as a serving loop would) and replayed: every replay, with eager work and synchronisations in between, must give the
eager call's result for the inputs then in the buffers."""
import numpy as np
import pytest

from paper_2505_03803_amd import binding as B
from paper_2505_03803_amd import synth

import gpu_util as G

pytestmark = pytest.mark.gpu


def _bits(t, a):
    import torch
    t.copy_(torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda())


@pytest.mark.parametrize("M,xdt", [(1, "f16"), (16, "bf16"), (48, "bf16")])
def test_dispatch_in_graph(M, xdt):
    torch = G.torch_()
    rng = np.random.default_rng(5)
    mats = [synth.gen_sq(rng, 256, 512), synth.gen_vq(rng, 256, 512, 6), synth.gen_vq(rng, 512, 256, 8),
            synth.gen_sq(rng, 48 if M <= 16 else 256, 256)]
    dms = [B.upload(m, native=True) for m in mats]
    xs = [torch.zeros((M, m.K), dtype=torch.int16, device="cuda") for m in mats]
    ys = [torch.zeros((M, m.N), dtype=torch.float32, device="cuda") for m in mats]
    table = B.DispatchTable([d.desc() for d in dms], xs, ys)
    run = lambda: B.rwkvq_linear_dispatch(table, M, B.DTYPES[xdt], B.F32)

    def fill(seed):
        r = np.random.default_rng(seed)
        for x, m in zip(xs, mats):
            _bits(x, synth.gen_activations(r, M, m.K, xdt))

    fill(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                              # first call outside the capture (one-time set-up)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for seed in (1, 2, 3, 4):
        print(f"graph replay M={M} seed={seed}", flush=True)
        fill(seed)
        for y in ys:
            y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = [y.clone() for y in ys]
        for y in ys:
            y.fill_(-1.0)                                   # eager work between the replays
        run()
        torch.cuda.synchronize()
        for g, y in zip(got, ys):
            assert torch.equal(g, y)


def test_mix_in_graph():
    torch = G.torch_()
    rng = np.random.default_rng(6)
    M, d, P = 4, 256, 3
    idx = [torch.from_numpy(rng.integers(0, 64, size=d // 2, dtype=np.uint8)).cuda() for _ in range(P)]
    cbs = [torch.from_numpy(synth.gen_codebook(rng, 64).view(np.int16)).cuda() for _ in range(P)]
    outs = [torch.zeros((M, d), dtype=torch.int16, device="cuda") for _ in range(P)]
    x = torch.zeros((M, d), dtype=torch.int16, device="cuda")
    xp = torch.zeros(d, dtype=torch.int16, device="cuda")
    table = B.MixTable(idx, cbs, outs)
    run = lambda: B.rwkvq_token_shift_mix(x, xp, B.BF16, M, d, table, 6)
    run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for seed in (1, 2, 3):
        r = np.random.default_rng(seed)
        _bits(x, synth.gen_activations(r, M, d, "bf16"))
        _bits(xp, synth.gen_activations(r, 1, d, "bf16")[0])
        graph.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        for o in outs:
            o.zero_()
        run()
        torch.cuda.synchronize()
        for g, o in zip(got, outs):
            assert torch.equal(g, o)


def test_block_token_step_in_graph():
    """One token through a block - fused mix + GEMV, wkv with its carried state, W_o, fused mix + GEMV
    with the squared ReLU at the store, W'_v with the gate at the store - recorded once and replayed
    for successive tokens: each replay must leave the outputs and the wkv state that the same calls
    give eagerly from the same state and inputs."""
    torch = G.torch_()
    rng = np.random.default_rng(6)
    d, ffn = 512, 1024
    names = ["r", "k", "v", "o", "ck", "cr", "cv"]
    mats = dict(zip(names, [synth.gen_sq(rng, d, d), synth.gen_vq(rng, d, d, 6), synth.gen_vq(rng, d, d, 8),
                            synth.gen_sq(rng, d, d), synth.gen_vq(rng, ffn, d, 6), synth.gen_sq(rng, d, d),
                            synth.gen_vq(rng, d, ffn, 8)]))
    dms = {n: B.upload(m, native=True) for n, m in mats.items()}
    t16 = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()
    mix = {n: (torch.from_numpy(rng.integers(0, 64, size=d // 2, dtype=np.uint8)).cuda(), t16(synth.gen_codebook(rng, 64)))
           for n in ("r", "k", "v", "ck", "cr")}
    _, _, _, w, u = synth.gen_block_inputs(rng, 1, d, "f16")
    wd, ud = torch.from_numpy(w).cuda(), torch.from_numpy(u).cuda()
    buf = lambda n: torch.zeros((1, n), dtype=torch.int16, device="cuda")
    x, xp, o_prev = buf(d), buf(d), buf(d)
    y = {n: buf(mats[n].N) for n in names}
    gated, sq, out = buf(d), buf(ffn), buf(d)
    st0 = np.zeros((3, d), dtype=np.float32); st0[2] = -1e38
    state = torch.from_numpy(st0).cuda()
    t1 = B.MixedDispatchTable([dms[n].desc() for n in ("r", "k", "v")], [(x, xp, *mix[n], 6) for n in ("r", "k", "v")],
                              [y[n] for n in ("r", "k", "v")])
    t2 = B.DispatchTable([dms["o"].desc()], [gated], [y["o"]])
    t3 = B.PostDispatchTable([dms[n].desc() for n in ("ck", "cr")], None, [(y["o"], o_prev, *mix[n], 6) for n in ("ck", "cr")],
                             [(B.POST_RELU2, None), (B.POST_NONE, None)], [sq, y["cr"]])
    t4 = B.PostDispatchTable([dms["cv"].desc()], [sq], None, [(B.POST_SIGMOID_GATE, y["cr"])], [out])

    def run():
        B.rwkvq_linear_dispatch_mixed(t1, B.F16, B.F16)
        B.rwkvq_wkv(y["r"], y["k"], y["v"], B.F16, 1, d, wd, ud, state, gated)
        B.rwkvq_linear_dispatch(t2, 1, B.F16, B.F16)
        B.rwkvq_linear_dispatch_post(t3, B.F16, B.F16)
        B.rwkvq_linear_dispatch_post(t4, B.F16, B.F16)

    toks = synth.gen_activations(rng, 6, d, "f16")
    _bits(x, toks[1][None, :]); _bits(xp, toks[0][None, :])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                              # first call outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    state.copy_(torch.from_numpy(st0).cuda())             # start the sequence again
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    state.copy_(torch.from_numpy(st0).cuda())
    o_prev.zero_()
    for t in range(1, 6):
        print(f"block step graph replay, token {t}", flush=True)
        _bits(x, toks[t][None, :]); _bits(xp, toks[t - 1][None, :])
        before = state.clone()
        out.zero_(); gated.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got_out, got_state, got_o = out.clone(), state.clone(), y["o"].clone()
        state.copy_(before)                                # eager, from the same state and inputs
        out.fill_(-1); gated.fill_(-1)
        run()
        torch.cuda.synchronize()
        assert torch.equal(got_out, out) and torch.equal(got_state, state) and torch.equal(got_o, y["o"])
        assert not torch.equal(state, before)
        o_prev.copy_(y["o"])


def test_fused_block_token_step_in_graph():
    """The same, with r, k, v and the wkv step in one launch and the mixes of channel mixing taken by the
    W_o launch: replayed for successive tokens against the eager calls from the same state."""
    torch = G.torch_()
    rng = np.random.default_rng(7)
    d, ffn = 512, 1024
    names = ["r", "k", "v", "o", "ck", "cr", "cv"]
    mats = dict(zip(names, [synth.gen_vq(rng, d, d, 6), synth.gen_sq(rng, d, d), synth.gen_vq(rng, d, d, 8),
                            synth.gen_sq(rng, d, d), synth.gen_sq(rng, ffn, d), synth.gen_vq(rng, d, d, 6),
                            synth.gen_vq(rng, d, ffn, 6)]))
    dms = {n: B.upload(m, native=True) for n, m in mats.items()}
    t16 = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()
    mix = {n: (torch.from_numpy(rng.integers(0, 64, size=d // 2, dtype=np.uint8)).cuda(), t16(synth.gen_codebook(rng, 64)))
           for n in ("ck", "cr")}
    _, _, _, w, u = synth.gen_block_inputs(rng, 1, d, "f16")
    wd, ud = torch.from_numpy(w).cuda(), torch.from_numpy(u).cuda()
    buf = lambda n: torch.zeros((1, n), dtype=torch.int16, device="cuda")
    x, o_prev = buf(d), buf(d)
    y = {n: buf(mats[n].N) for n in names}
    gated, sq, out, in_ck, in_cr = buf(d), buf(ffn), buf(d), buf(d), buf(d)
    st0 = np.zeros((3, d), dtype=np.float32); st0[2] = -1e38
    state = torch.from_numpy(st0).cuda()
    t1 = B.RkvWkvTable([dms[n].desc() for n in ("r", "k", "v")], [x, x, x], [y[n] for n in ("r", "k", "v")])
    t2 = B.PostDispatchTable([dms["o"].desc()], [gated], None,
                             [(B.POST_NONE, None, o_prev, [(mix["ck"][0], mix["ck"][1], 6, in_ck), (mix["cr"][0], mix["cr"][1], 6, in_cr)])],
                             [y["o"]])
    t3 = B.PostDispatchTable([dms[n].desc() for n in ("ck", "cr")], [in_ck, in_cr], None,
                             [(B.POST_RELU2, None), (B.POST_NONE, None)], [sq, y["cr"]])
    t4 = B.PostDispatchTable([dms["cv"].desc()], [sq], None, [(B.POST_SIGMOID_GATE, y["cr"])], [out])

    def run():
        B.rwkvq_rkv_wkv(t1, wd, ud, state, gated, B.F16, B.F16)
        B.rwkvq_linear_dispatch_post(t2, B.F16, B.F16)
        B.rwkvq_linear_dispatch_post(t3, B.F16, B.F16)
        B.rwkvq_linear_dispatch_post(t4, B.F16, B.F16)

    toks = synth.gen_activations(rng, 6, d, "f16")
    _bits(x, toks[0][None, :])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                              # first call outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    state.copy_(torch.from_numpy(st0).cuda())
    o_prev.zero_()
    for t in range(1, 6):
        print(f"fused block step graph replay, token {t}", flush=True)
        _bits(x, toks[t][None, :])
        before = state.clone()
        out.zero_(); gated.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got_out, got_state, got_o = out.clone(), state.clone(), y["o"].clone()
        state.copy_(before)
        out.fill_(-1); gated.fill_(-1)
        run()
        torch.cuda.synchronize()
        assert torch.equal(got_out, out) and torch.equal(got_state, state) and torch.equal(got_o, y["o"])
        assert not torch.equal(state, before)
        o_prev.copy_(y["o"])
