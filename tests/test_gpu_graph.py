"""The linear-layer dispatch and the token-shift mix recorded into a HIP graph (as a serving loop
would) and replayed: every replay, with eager work and synchronisations in between, must give the
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
