"""GPU parity of the element-wise multiplication path (Sec. 3.2) through the C ABI: representative
activation, weighted-KMeans codebook, token-shift mix.  Bars: every output bit-exact (all decisions
and roundings are fixed by the definition; the binary64 sums of the centroid update are rounded to
fp16 at once, which absorbs their order)."""
import numpy as np
import pytest

from oracle import mu_oracle as MO
from oracle import rwkvq_oracle as orc
from paper_2505_03803_amd import binding as B
from paper_2505_03803_amd import synth

import gpu_util as G

pytestmark = pytest.mark.gpu


def dev(a):
    torch = G.torch_()
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def widen(bits, dt):
    return bits.astype(np.float32) if dt == "f32" else orc.widen(bits, dt)


@pytest.mark.parametrize("Bn,n", [(1, 7), (5, 300), (37, 64), (128, 4096), (129, 1000), (256, 70), (300, 50), (1030, 20)])
@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
def test_clip_mean(Bn, n, dt):
    torch = G.torch_()
    rng = np.random.default_rng(Bn * 1000 + n)
    x = synth.gen_calibration(rng, Bn, n, dt)
    xd = dev(x)
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    for p in (0.0, 1.0, 2.5, 10.0, 50.0):
        print(f"clip_mean B={Bn} n={n} {dt} p={p}", flush=True)
        B.rwkvq_clip_mean(xd, B.DTYPES[dt], Bn, n, p, out)
        torch.cuda.synchronize()
        want = MO.clip_mean(widen(x, dt), p)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32))


def _run_codebook(mus, xbars, cb0s, dt, kbits, iters):
    torch = G.torch_()
    md = [dev(m) for m in mus]
    xd = [dev(x) for x in xbars]
    cd = [dev(c.copy()) for c in cb0s]
    idx = [torch.full((m.size // 2 + 15,), 255, dtype=torch.uint8, device="cuda") for m in mus]
    B.rwkvq_mu_codebook(md, xd, [m.size for m in mus], B.DTYPES[dt], kbits, iters, cd, idx)
    torch.cuda.synchronize()
    return [c.cpu().numpy().view(np.uint16) for c in cd], [i.cpu().numpy() for i in idx]


@pytest.mark.parametrize("kbits", [6, 8])
@pytest.mark.parametrize("iters", [0, 1, 6])
@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_mu_codebook(kbits, iters, dt):
    rng = np.random.default_rng(100 + kbits + iters)
    sizes = [2, 10, 4096, 5 * 4096, 4098]
    E = 1 << kbits
    mus, xbars, cb0s = [], [], []
    for n in sizes:
        m = synth.gen_mu(rng, n, "bf16")
        mus.append(orc.widen(m, "bf16") if dt == "f32" else m)
        xbars.append(MO.clip_mean(orc.widen(synth.gen_calibration(rng, 16, n, "bf16"), "bf16"), 2.0))
        cb0s.append(synth.gen_codebook(rng, E).reshape(E, 2))
    xbars[2][::7] = 0.0                                        # some zero element weights
    print(f"mu_codebook kbits={kbits} iters={iters} {dt}", flush=True)
    cbs, idxs = _run_codebook(mus, xbars, cb0s, dt, kbits, iters)
    for m, x, c0, cb, ix in zip(mus, xbars, cb0s, cbs, idxs):
        mf = m if dt == "f32" else orc.widen(m, "bf16")
        wcb, widx, _ = MO.mu_codebook(mf, x, orc.widen(c0, "f16"), iters)
        assert np.array_equal(cb.reshape(-1), synth.f32_to_f16_bits(wcb).reshape(-1)), m.size
        assert np.array_equal(ix[:m.size // 2], widx.astype(np.uint8)), m.size
        assert np.all(ix[m.size // 2:] == 255)                 # nothing written past the end


def test_mu_codebook_many_tensors():
    """More tensors than one launch holds (64): 70 small tensors."""
    rng = np.random.default_rng(7)
    mus = [synth.gen_mu(rng, 256, "bf16") for _ in range(70)]
    xbars = [rng.standard_normal(256).astype(np.float32) for _ in range(70)]
    cb0s = [synth.gen_codebook(rng, 64).reshape(64, 2) for _ in range(70)]
    cbs, idxs = _run_codebook(mus, xbars, cb0s, "bf16", 6, 3)
    for m, x, c0, cb, ix in zip(mus, xbars, cb0s, cbs, idxs):
        wcb, widx, _ = MO.mu_codebook(orc.widen(m, "bf16"), x, orc.widen(c0, "f16"), 3)
        assert np.array_equal(cb.reshape(-1), synth.f32_to_f16_bits(wcb).reshape(-1))
        assert np.array_equal(ix[:128], widx.astype(np.uint8))


@pytest.mark.parametrize("M,d", [(1, 8), (3, 64), (40, 4096), (1, 4096), (257, 136)])
@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("kbits,P", [(6, 1), (6, 5), (8, 8)])
def test_token_shift_mix(M, d, dt, kbits, P):
    torch = G.torch_()
    rng = np.random.default_rng(M * 10 + d + P)
    E = 1 << kbits
    x = synth.gen_activations(rng, M, d, dt)
    xp = synth.gen_activations(rng, 1, d, dt)[0]
    idx = [rng.integers(0, E, size=d // 2, dtype=np.uint8) for _ in range(P)]
    cbs = [synth.gen_codebook(rng, E).reshape(E, 2) for _ in range(P)]
    outs = [torch.zeros((M, d), dtype=torch.int16, device="cuda") for _ in range(P)]
    table = B.MixTable([dev(i) for i in idx], [dev(c) for c in cbs], outs)
    print(f"mix M={M} d={d} {dt} kbits={kbits} P={P}", flush=True)
    B.rwkvq_token_shift_mix(dev(x), dev(xp), B.DTYPES[dt], M, d, table, kbits)
    torch.cuda.synchronize()
    xf, xpf = orc.widen(x, dt), orc.widen(xp, dt)
    for p in range(P):
        mu_hat = orc.widen(cbs[p], "f16")[idx[p]].reshape(-1)
        want = MO.narrow(MO.token_shift_mix(xf, xpf, mu_hat), dt)
        assert np.array_equal(outs[p].cpu().numpy().view(np.uint16), want), p


def test_calibrate_quantize_mix_gemv_chain():
    """The whole path on one layer's worth of synthetic data: representative activation -> codebook
    and indices of five mix weights -> mixed activations -> the quantized GEMV; every stage of the
    GPU path against the same stage of the oracle (bit-exact up to the GEMV, 2e-3 after)."""
    torch = G.torch_()
    rng = np.random.default_rng(11)
    d, P, Bn = 512, 5, 64
    cal = synth.gen_calibration(rng, Bn, d, "bf16")
    xbar_d = torch.empty(d, dtype=torch.float32, device="cuda")
    B.rwkvq_clip_mean(dev(cal), B.BF16, Bn, d, 1.0, xbar_d)
    torch.cuda.synchronize()
    xbar = MO.clip_mean(orc.widen(cal, "bf16"), 1.0)
    assert np.array_equal(xbar_d.cpu().numpy(), xbar)
    mus = [synth.gen_mu(rng, d, "bf16") for _ in range(P)]
    cb0 = [synth.gen_codebook(rng, 64).reshape(64, 2) for _ in range(P)]
    md, cd = [dev(m) for m in mus], [dev(c.copy()) for c in cb0]
    idd = [torch.empty(d // 2, dtype=torch.uint8, device="cuda") for _ in range(P)]
    B.rwkvq_mu_codebook(md, [xbar_d] * P, [d] * P, B.BF16, 6, 8, cd, idd)
    x = synth.gen_activations(rng, 1, d, "f16")
    xp = synth.gen_activations(rng, 1, d, "f16")[0]
    outs = [torch.empty((1, d), dtype=torch.int16, device="cuda") for _ in range(P)]
    B.rwkvq_token_shift_mix(dev(x), dev(xp), B.F16, 1, d, B.MixTable(idd, cd, outs), 6)
    mats = [synth.gen_sq(rng, 256, d) if p % 2 == 0 else synth.gen_vq(rng, 256, d, 6) for p in range(P)]
    dms = [B.upload(m, native=True) for m in mats]
    ys = [torch.empty((1, 256), dtype=torch.float32, device="cuda") for _ in range(P)]
    B.rwkvq_linear_dispatch(B.DispatchTable([m.desc() for m in dms], outs, ys), 1, B.F16, B.F32)
    torch.cuda.synchronize()
    for p in range(P):
        wcb, widx, _ = MO.mu_codebook(orc.widen(mus[p], "bf16"), xbar, orc.widen(cb0[p], "f16"), 8)
        assert np.array_equal(cd[p].cpu().numpy().view(np.uint16).reshape(-1), synth.f32_to_f16_bits(wcb).reshape(-1))
        assert np.array_equal(idd[p].cpu().numpy(), widx.astype(np.uint8))
        mixed = MO.narrow(MO.token_shift_mix(orc.widen(x, "f16"), orc.widen(xp, "f16"), wcb[widx].reshape(-1)), "f16")
        assert np.array_equal(outs[p].cpu().numpy().view(np.uint16), mixed)
        ref = orc.linear(mats[p], orc.widen(mixed, "f16"), "f64")
        err = np.abs(ys[p].cpu().numpy() - ref).max() / np.abs(ref).max()
        assert err < 2e-3, err


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("kbits", [6, 8])
def test_fused_mix_gemv_equals_chain(dt, kbits):
    """rwkvq_linear_dispatch_mixed against rwkvq_token_shift_mix followed by rwkvq_linear_dispatch on
    the same matrices (bit for bit: same mixed values, same kernel shape), and against the oracle
    chain; shapes that take 4, 8 and 16 wavefronts per row tile, all three weight formats."""
    torch = G.torch_()
    rng = np.random.default_rng(70 + kbits)
    E = 1 << kbits
    for shapes in ([(256, 512), (512, 256), (48, 768)], [(4096, 512)], [(8192, 256), (256, 3584)]):
        mats = []
        for j, (N, K) in enumerate(shapes):
            kind = ("sq", "vq6", "vq8")[(j + kbits) % 3]
            N_ = N if kind == "sq" else max(256, N // 256 * 256)
            mats.append(synth.gen_sq(rng, N_, K) if kind == "sq" else synth.gen_vq(rng, N_, K, 6 if kind == "vq6" else 8))
        dms = [B.upload(m, native=True) for m in mats]
        xs = [synth.gen_activations(rng, 1, m.K, dt) for m in mats]
        xps = [synth.gen_activations(rng, 1, m.K, dt)[0] for m in mats]
        idx = [rng.integers(0, E, size=m.K // 2, dtype=np.uint8) for m in mats]
        cbs = [synth.gen_codebook(rng, E).reshape(E, 2) for m in mats]
        xd, xpd = [dev(x) for x in xs], [dev(x) for x in xps]
        idd, cbd = [dev(i) for i in idx], [dev(c) for c in cbs]
        # chain: one mix call per matrix (their K differ), then one dispatch
        mixed = [torch.empty((1, m.K), dtype=torch.int16, device="cuda") for m in mats]
        for m, x, xp, i, c, o in zip(mats, xd, xpd, idd, cbd, mixed):
            B.rwkvq_token_shift_mix(x, xp, B.DTYPES[dt], 1, m.K, B.MixTable([i], [c], [o]), kbits)
        y_chain = [torch.empty((1, m.N), dtype=torch.float32, device="cuda") for m in mats]
        B.rwkvq_linear_dispatch(B.DispatchTable([d.desc() for d in dms], mixed, y_chain), 1, B.DTYPES[dt], B.F32)
        y_fused = [torch.zeros((1, m.N), dtype=torch.float32, device="cuda") for m in mats]
        table = B.MixedDispatchTable([d.desc() for d in dms],
                                     [(x, xp, i, c, kbits) for x, xp, i, c in zip(xd, xpd, idd, cbd)], y_fused)
        print(f"fused mix {dt} kbits={kbits} shapes={shapes}", flush=True)
        B.rwkvq_linear_dispatch_mixed(table, B.DTYPES[dt], B.F32)
        torch.cuda.synchronize()
        for m, x, xp, i, c, yc, yf in zip(mats, xs, xps, idx, cbs, y_chain, y_fused):
            assert torch.equal(yc, yf), (m.kind, m.N, m.K)
            mu_hat = orc.widen(c, "f16")[i].reshape(-1)
            xm = MO.narrow(MO.token_shift_mix(orc.widen(x, dt), orc.widen(xp, dt), mu_hat), dt)
            ref = orc.linear(m, orc.widen(xm, dt), "f64")
            err = np.abs(yf.cpu().numpy() - ref).max() / np.abs(ref).max()
            assert err <= 2e-5, err
