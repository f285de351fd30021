"""GPU parity of the element-wise operators of the RWKV block (App. A.1) through the C ABI.

Bars.  rwkvq_relu2: bit-exact (the square of a 16-bit value is exact in binary32, so there is one
rounding on either side).  rwkvq_sigmoid_gate and rwkvq_wkv: the kernel works in binary32 and rounds
once to the 16-bit output, the oracle evaluates the printed formulas in binary64, so the bar is half
an output ulp (1 % slack for the binary32 error in front of the rounding) plus, for wkv, 1.5e-4 of the
largest |v|: the state's exponent p is a binary32 number of the size of the keys (|k| < 128 here, so
each of its updates rounds by <= 2^-18); over the 64 tokens of the longest case that shifts the
relative weight of past and current tokens by <= 64 * 2^-18 = 2.4e-4, and a weight shift of delta
moves a convex combination of values in [-vmax, vmax] by <= delta * 2 vmax / 4."""
import numpy as np
import pytest

from oracle import block_oracle as BO
from oracle import mu_oracle as MO
from oracle import rwkvq_oracle as orc
from paper_2505_03803_amd import binding as B
from paper_2505_03803_amd import synth

import gpu_util as G

pytestmark = pytest.mark.gpu

HALF_ULP = {"f16": 2.0 ** -11, "bf16": 2.0 ** -8}       # relative, of the output type (bf16: 8 significant bits)
# absolute floor: half the subnormal spacing of fp16; for bf16 the smallest normal number (the binary32
# sigmoid is 0 below x = -88.7, where exp(-x) overflows, while the exact value is about e^x < 3e-39)
FLOOR = {"f16": 2.0 ** -25, "bf16": 2.0 ** -126}


def dev(a):
    torch = G.torch_()
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def host(t, dt):
    return orc.widen(t.cpu().numpy().view(np.uint16), dt).astype(np.float64)


def fresh_state(d):
    s = np.zeros((3, d), dtype=np.float32)
    s[2] = -1e38
    return dev(s)


def check_close(got, want, dt, scale):
    tol = HALF_ULP[dt] * 1.01 * np.abs(want) + FLOOR[dt] + 1.5e-4 * scale
    bad = np.abs(got - want) > tol
    assert not bad.any(), (int(bad.sum()), float(np.abs(got - want).max()), np.argwhere(bad)[:4])


def oracle_gated_wkv(r, k, v, w, u, dt):
    W = lambda a: orc.widen(a, dt).astype(np.float64)
    return BO.time_mixing_gate(W(r), BO.wkv_direct(W(k), W(v), w, u))


@pytest.mark.parametrize("M,d", [(1, 64), (7, 200), (8, 4096), (33, 777), (64, 2048)])
@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_wkv_chunk(M, d, dt):
    torch = G.torch_()
    rng = np.random.default_rng(9000 + M * 10 + d)
    r, k, v, w, u = synth.gen_block_inputs(rng, M, d, dt)
    print(f"wkv M={M} d={d} {dt}", flush=True)
    out = torch.zeros((M, d), dtype=torch.int16, device="cuda")
    state = fresh_state(d)
    B.rwkvq_wkv(dev(r), dev(k), dev(v), B.DTYPES[dt], M, d, dev(w), dev(u), state, out)
    torch.cuda.synchronize()
    want = oracle_gated_wkv(r, k, v, w, u, dt)
    vmax = float(np.abs(orc.widen(v, dt)).max())
    check_close(host(out, dt), want, dt, vmax)
    assert np.allclose(host(out, dt)[0], BO.time_mixing_gate(orc.widen(r, dt)[0], orc.widen(v, dt)[0]),
                       rtol=2 * HALF_ULP[dt], atol=1e-6)              # wkv_1 = v_1


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_wkv_state_carries_across_calls(dt):
    """Token by token, in two chunks and in one chunk: the same bits (the kernel takes the same
    steps in the same order), and the carried state equals that of the single call."""
    torch = G.torch_()
    M, d = 21, 520
    rng = np.random.default_rng(9100)
    r, k, v, w, u = synth.gen_block_inputs(rng, M, d, dt)
    rd, kd, vd, wd, ud = dev(r), dev(k), dev(v), dev(w), dev(u)
    one = torch.zeros((M, d), dtype=torch.int16, device="cuda")
    s1 = fresh_state(d)
    B.rwkvq_wkv(rd, kd, vd, B.DTYPES[dt], M, d, wd, ud, s1, one)
    two = torch.zeros((M, d), dtype=torch.int16, device="cuda")
    s2 = fresh_state(d)
    B.rwkvq_wkv(rd, kd, vd, B.DTYPES[dt], 13, d, wd, ud, s2, two)
    B.rwkvq_wkv(rd[13:], kd[13:], vd[13:], B.DTYPES[dt], M - 13, d, wd, ud, s2, two[13:])
    tok = torch.zeros((M, d), dtype=torch.int16, device="cuda")
    s3 = fresh_state(d)
    for t in range(M):
        B.rwkvq_wkv(rd[t], kd[t], vd[t], B.DTYPES[dt], 1, d, wd, ud, s3, tok[t])
    torch.cuda.synchronize()
    assert torch.equal(one, two) and torch.equal(one, tok)
    assert torch.equal(s1, s2) and torch.equal(s1, s3)
    check_close(host(one, dt), oracle_gated_wkv(r, k, v, w, u, dt), dt, float(np.abs(orc.widen(v, dt)).max()))


@pytest.mark.parametrize("M,d", [(128, 48), (1000, 200), (2048, 64), (333, 16)])
@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_wkv_long_chunk_time_parallel(M, d, dt):
    """Chunks of 128 tokens and more take the time-parallel kernel (64 pieces, merged).  Against the
    explicit sums, then a second call that continues from the carried state.  The bar on top of half
    an output ulp is 2e-5 of the largest |v| (measured: 5e-7; the exponent's rounding of 2^-18 per token acts
    only over the tokens a channel still remembers, and mostly cancels).  The token-by-token kernel, run on
    the same tokens in pieces of 96, rounds p once per token: a token of age 1 / w is off in weight by
    about 2^-18 / w <= 5.7e-4 for the slowest decay e^-5, which moves a mean of values by <= 2.8e-4 of
    max|v| in the worst case, whatever the length; measured <= 8.6e-5, held to the 1.5e-4 of the short cases.
    The absolute exponent of the carried sums may drift by 2^-18 per token; only differences matter."""
    torch = G.torch_()
    rng = np.random.default_rng(9600 + M + d)
    M2 = 150
    r, k, v, w, u = synth.gen_block_inputs(rng, M + M2, d, dt)
    rd, kd, vd, wd, ud = dev(r), dev(k), dev(v), dev(w), dev(u)
    print(f"wkv time-parallel M={M}+{M2} d={d} {dt}", flush=True)
    out = torch.zeros((M + M2, d), dtype=torch.int16, device="cuda")
    state = fresh_state(d)
    B.rwkvq_wkv(rd, kd, vd, B.DTYPES[dt], M, d, wd, ud, state, out)
    B.rwkvq_wkv(rd[M:], kd[M:], vd[M:], B.DTYPES[dt], M2, d, wd, ud, state, out[M:])
    torch.cuda.synchronize()
    want = oracle_gated_wkv(r, k, v, w, u, dt)
    got = host(out, dt)
    vmax = float(np.abs(orc.widen(v, dt)).max())
    tol = HALF_ULP[dt] * 1.01 * np.abs(want) + FLOOR[dt] + 2e-5 * vmax
    bad = np.abs(got - want) > tol
    excess = float((np.abs(got - want) - HALF_ULP[dt] * np.abs(want)).max() / vmax)
    print(f"  largest error beyond half an ulp: {excess:.2e} of max|v|", flush=True)
    assert not bad.any(), (int(bad.sum()), np.argwhere(bad)[:4])
    # the token-by-token kernel on the same tokens (pieces of 96 < 128)
    seq = torch.zeros((M + M2, d), dtype=torch.int16, device="cuda")
    st2 = fresh_state(d)
    for t0 in range(0, M + M2, 96):                           # 96 rows of any width start 16-byte aligned
        n = min(96, M + M2 - t0)
        B.rwkvq_wkv(rd[t0:], kd[t0:], vd[t0:], B.DTYPES[dt], n, d, wd, ud, st2, seq[t0:])
    torch.cuda.synchronize()
    excess = float((np.abs(host(seq, dt) - want) - HALF_ULP[dt] * np.abs(want)).max() / vmax)
    print(f"  token-by-token kernel on the same tokens: {excess:.2e} of max|v|", flush=True)
    check_close(host(seq, dt), want, dt, vmax)               # its own bar (one rounding of p per token)
    # the carried sums a e^p, b e^p of both kernels against their definition (binary64): the weighted
    # mean a / b and the log of the weight sum log b + p
    T = M + M2
    kf, vf = orc.widen(k, dt).astype(np.float64), orc.widen(v, dt).astype(np.float64)
    e = -(T - 1 - np.arange(T))[:, None] * w.astype(np.float64)[None, :] + kf
    m = e.max(axis=0)
    den = np.exp(e - m).sum(axis=0)
    mean_true, logw_true = (np.exp(e - m) * vf).sum(axis=0) / den, np.log(den) + m
    for name, st, bar in (("time-parallel", state, 2e-5), ("token by token", st2, 1.5e-4)):
        a_, b_, p_ = st.cpu().numpy().astype(np.float64)
        err_mean = float(np.abs(a_ / b_ - mean_true).max() / vmax)
        err_logw = float(np.abs(np.log(b_) + p_ - logw_true).max())
        print(f"  carried state, {name}: mean off by {err_mean:.2e} of max|v|, log weight by {err_logw:.2e}", flush=True)
        # every step rounds the exponent p (|p| < 128) by at most 2^-18, and w is constant: the roundings can add up
        assert err_mean <= bar and err_logw <= T * 2.0 ** -18, name


def test_wkv_extreme_keys_stay_finite():
    """Keys at the ends of the fp16 range (an exponent of +-65504): the running maximum keeps every
    exp() argument non-positive, so nothing overflows and a dominant key returns its own value."""
    torch = G.torch_()
    M, d = 6, 128
    rng = np.random.default_rng(9200)
    r, k, v, w, u = synth.gen_block_inputs(rng, M, d, "f16")
    kf = orc.widen(k, "f16").copy()
    kf[2, :64] = 65504.0
    kf[3, 64:] = -65504.0
    kf[4, :32] = 30000.0
    k = kf.astype(np.float16).view(np.uint16)
    out = torch.zeros((M, d), dtype=torch.int16, device="cuda")
    B.rwkvq_wkv(dev(r), dev(k), dev(v), B.F16, M, d, dev(w), dev(u), fresh_state(d), out)
    torch.cuda.synchronize()
    got = host(out, "f16")
    assert np.isfinite(got).all()
    check_close(got, oracle_gated_wkv(r, k, v, w, u, "f16"), "f16", float(np.abs(orc.widen(v, "f16")).max()))


@pytest.mark.parametrize("n", [1, 8, 2047, 2048, 14336, 100003])
@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_relu2_and_gate(n, dt):
    torch = G.torch_()
    rng = np.random.default_rng(9300 + n)
    x = synth.gen_activations(rng, 1, n, dt)[0]
    y = synth.gen_activations(rng, 1, n, dt)[0]
    xf = orc.widen(x, dt)
    xf[:: 97] *= 30.0                                            # a few large values, also negative ones
    x = MO.narrow(xf, dt)
    xd, yd = dev(x), dev(y)
    out = torch.zeros(n + 8, dtype=torch.int16, device="cuda")  # 8 guard values behind the end
    print(f"relu2/gate n={n} {dt}", flush=True)
    B.rwkvq_relu2(xd, B.DTYPES[dt], n, out)
    torch.cuda.synchronize()
    want = BO.relu_squared(orc.widen(x, dt).astype(np.float64))
    want_bits = MO.narrow(want.astype(np.float32), dt)           # exact in binary32: one rounding in all
    assert np.array_equal(out[:n].cpu().numpy().view(np.uint16), want_bits)
    assert not out[n:].any()
    B.rwkvq_sigmoid_gate(xd, yd, B.DTYPES[dt], n, out)
    torch.cuda.synchronize()
    want = BO.channel_mixing_gate(orc.widen(x, dt).astype(np.float64), orc.widen(y, dt).astype(np.float64))
    check_close(host(out[:n], dt), want, dt, 0.0)
    assert not out[n:].any()
    # in place
    B.rwkvq_sigmoid_gate(xd, yd, B.DTYPES[dt], n, yd)
    torch.cuda.synchronize()
    assert torch.equal(yd, out[:n])


def test_block_tokens_through_quantized_projections():
    """A few tokens through one block as App. A.1 chains it, every projection quantized (SQ, 6- and
    8-bit VQ mixed), batch 1, states carried on the device: fused mix + GEMV -> wkv and gate -> W_o ->
    fused mix + GEMV -> squared ReLU -> W'_v -> gate.  Every stage is checked against the oracle fed
    with the inputs the device held for that stage (stage bar), and the block output against the
    oracle chain running on its own values (the roundings to fp16 between stages then differ now and
    again, so that bar is the loose one)."""
    torch = G.torch_()
    rng = np.random.default_rng(9400)
    d, ffn, T, dt = 512, 1024, 6, "f16"
    mk = {"sq": lambda N, K: synth.gen_sq(rng, N, K), "vq6": lambda N, K: synth.gen_vq(rng, N, K, 6),
          "vq8": lambda N, K: synth.gen_vq(rng, N, K, 8)}
    names = ["r", "k", "v", "o", "ck", "cr", "cv"]
    mats = dict(zip(names, [mk["sq"](d, d), mk["vq6"](d, d), mk["vq8"](d, d), mk["sq"](d, d), mk["vq6"](ffn, d),
                            mk["sq"](d, d), mk["vq8"](d, ffn)]))
    dms = {n: B.upload(m, native=True) for n, m in mats.items()}
    mixes = {n: (rng.integers(0, 64, size=d // 2, dtype=np.uint8), synth.gen_codebook(rng, 64).reshape(64, 2))
             for n in ("r", "k", "v", "ck", "cr")}
    mixd = {n: (dev(i), dev(c)) for n, (i, c) in mixes.items()}
    mu_hat = {n: orc.widen(c, "f16")[i].reshape(-1) for n, (i, c) in mixes.items()}
    _, _, _, w, u = synth.gen_block_inputs(rng, 1, d, dt)
    wd, ud = dev(w), dev(u)
    xs = synth.gen_activations(rng, T + 1, d, dt)                # xs[0] is the token before the first
    buf = lambda n: torch.zeros((1, n), dtype=torch.int16, device="cuda")
    yb = {n: buf(mats[n].N) for n in names}
    gated, sq, out = buf(d), buf(ffn), buf(d)
    o_prev = buf(d)
    state = fresh_state(d)
    W = lambda t: orc.widen(t.cpu().numpy().view(np.uint16).reshape(-1), dt).astype(np.float64)
    lin = lambda n, x: orc.linear(mats[n], x.astype(np.float32)[None, :], "f64")[0]
    rel = lambda got, ref: float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))
    # oracle chain on its own values
    rt = lambda a: orc.widen(MO.narrow(np.asarray(a, dtype=np.float32), dt), dt).astype(np.float64)   # store as fp16
    mixo = lambda n, x, xp: rt(MO.token_shift_mix(x[None, :], xp, mu_hat[n])[0])
    hist_k, hist_v = [], []
    o_prev_ref = np.zeros(d)
    for t in range(1, T + 1):
        print(f"block token {t}", flush=True)
        x, xp = dev(xs[t]), dev(xs[t - 1])
        B.rwkvq_linear_dispatch_mixed(B.MixedDispatchTable(
            [dms[n].desc() for n in ("r", "k", "v")], [(x, xp, *mixd[n], 6) for n in ("r", "k", "v")],
            [yb[n] for n in ("r", "k", "v")]), B.F16, B.F16)
        s_before = state.clone()
        B.rwkvq_wkv(yb["r"], yb["k"], yb["v"], B.F16, 1, d, wd, ud, state, gated)
        B.rwkvq_linear_dispatch(B.DispatchTable([dms["o"].desc()], [gated], [yb["o"]]), 1, B.F16, B.F16)
        B.rwkvq_linear_dispatch_mixed(B.MixedDispatchTable(
            [dms[n].desc() for n in ("ck", "cr")], [(yb["o"], o_prev, *mixd[n], 6) for n in ("ck", "cr")],
            [yb[n] for n in ("ck", "cr")]), B.F16, B.F16)
        B.rwkvq_relu2(yb["ck"], B.F16, ffn, sq)
        B.rwkvq_linear_dispatch(B.DispatchTable([dms["cv"].desc()], [sq], [yb["cv"]]), 1, B.F16, B.F16)
        B.rwkvq_sigmoid_gate(yb["cr"], yb["cv"], B.F16, d, out)
        torch.cuda.synchronize()
        # stage bars, each stage fed with what the device held
        xf, xpf = orc.widen(xs[t], dt), orc.widen(xs[t - 1], dt)
        for n in ("r", "k", "v"):
            assert rel(W(yb[n]), lin(n, mixo(n, xf, xpf))) <= 2e-3, n
        hist_k.append(W(yb["k"])); hist_v.append(W(yb["v"]))
        want = BO.time_mixing_gate(W(yb["r"]), BO.wkv_direct(np.array(hist_k), np.array(hist_v), w, u)[-1])
        check_close(W(gated), want, dt, float(np.abs(np.array(hist_v)).max()))
        assert rel(W(yb["o"]), lin("o", W(gated))) <= 2e-3
        for n in ("ck", "cr"):
            assert rel(W(yb[n]), lin(n, mixo(n, W(yb["o"]).astype(np.float32), W(o_prev).astype(np.float32)))) <= 2e-3, n
        assert np.array_equal(W(sq), rt(BO.relu_squared(W(yb["ck"]))))
        assert rel(W(yb["cv"]), lin("cv", W(sq))) <= 2e-3
        check_close(W(out), BO.channel_mixing_gate(W(yb["cr"]), W(yb["cv"])), dt, 0.0)
        # the oracle's own chain
        if t == 1:
            ref_k, ref_v = [], []
        r_ = rt(lin("r", mixo("r", xf, xpf))); k_ = rt(lin("k", mixo("k", xf, xpf))); v_ = rt(lin("v", mixo("v", xf, xpf)))
        ref_k.append(k_); ref_v.append(v_)
        g_ = rt(BO.time_mixing_gate(r_, BO.wkv_direct(np.array(ref_k), np.array(ref_v), w, u)[-1]))
        o_ = rt(lin("o", g_))
        ck_ = rt(lin("ck", mixo("ck", o_.astype(np.float32), o_prev_ref.astype(np.float32))))
        cr_ = rt(lin("cr", mixo("cr", o_.astype(np.float32), o_prev_ref.astype(np.float32))))
        out_ = rt(BO.channel_mixing_gate(cr_, rt(lin("cv", rt(BO.relu_squared(ck_))))))
        e2e = rel(W(out), out_)
        print(f"  block output vs free-running oracle chain: {e2e:.2e}", flush=True)
        assert e2e <= 2e-3
        o_prev_ref = o_
        o_prev.copy_(yb["o"])
        del s_before


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("shapes", [[(256, 512), (512, 256), (48, 768)], [(4096, 512)], [(8192, 256), (256, 3584)],
                                    [(16384, 256), (16384, 512), (4096, 256)]])
@pytest.mark.parametrize("with_mix", [False, True])
@pytest.mark.parametrize("grid", [1, 2])
def test_post_operator_equals_separate_pass(dt, shapes, with_mix, grid, options):
    """rwkvq_linear_dispatch_post against the same projections followed by rwkvq_relu2 /
    rwkvq_sigmoid_gate: bit for bit (same matrices per call, hence the same kernel shape and order of
    summation; the operator is applied to the rounded output).  The shapes take 4, 8 and 16
    wavefronts per row tile and, the last, the grouped kernel (with the mix in front, which always
    splits the columns, four wavefronts per row tile on 2304 row tiles); matrix j gets operator j mod 3.
    grid: how a workgroup of the split-K kernels finds its matrix and row tile (RWKVQ_OPT_SPLIT_GRID_2D: 1 = from a
    two-dimensional grid, 2 = from the table of first workgroups)."""
    options(B.OPT_SPLIT_GRID_2D, grid)
    torch = G.torch_()
    rng = np.random.default_rng(9500 + len(shapes) + shapes[0][0])
    mats = []
    for j, (N, K) in enumerate(shapes):
        kind = ("sq", "vq6", "vq8")[j % 3]
        N_ = N if kind == "sq" else max(256, N // 256 * 256)
        mats.append(synth.gen_sq(rng, N_, K) if kind == "sq" else synth.gen_vq(rng, N_, K, 6 if kind == "vq6" else 8))
    dms = [B.upload(m, native=True) for m in mats]
    descs = [m.desc() for m in dms]
    xs = [dev(synth.gen_activations(rng, 1, m.K, dt)) for m in mats]
    xps = [dev(synth.gen_activations(rng, 1, m.K, dt)[0]) for m in mats]
    idx = [dev(rng.integers(0, 64, size=m.K // 2, dtype=np.uint8)) for m in mats]
    cbs = [dev(synth.gen_codebook(rng, 64).reshape(64, 2)) for m in mats]
    gates = [dev(synth.gen_activations(rng, 1, m.N, dt)[0]) for m in mats]
    mixes = [(x, xp, i, c, 6) for x, xp, i, c in zip(xs, xps, idx, cbs)] if with_mix else None
    plain = [torch.zeros((1, m.N), dtype=torch.int16, device="cuda") for m in mats]
    if with_mix:
        B.rwkvq_linear_dispatch_mixed(B.MixedDispatchTable(descs, mixes, plain), B.DTYPES[dt], B.DTYPES[dt])
    else:
        B.rwkvq_linear_dispatch(B.DispatchTable(descs, xs, plain), 1, B.DTYPES[dt], B.DTYPES[dt])
    want = []
    for j, (m, y, g) in enumerate(zip(mats, plain, gates)):
        o = torch.zeros_like(y)
        if j % 3 == 0:
            B.rwkvq_relu2(y, B.DTYPES[dt], m.N, o)
        elif j % 3 == 1:
            B.rwkvq_sigmoid_gate(g, y, B.DTYPES[dt], m.N, o)
        else:
            o.copy_(y)
        want.append(o)
    posts = [((B.POST_RELU2, None), (B.POST_SIGMOID_GATE, g), (B.POST_NONE, None))[j % 3] for j, g in enumerate(gates)]
    got = [torch.zeros((1, m.N), dtype=torch.int16, device="cuda") for m in mats]
    print(f"post {dt} mix={with_mix} shapes={shapes}", flush=True)
    B.rwkvq_linear_dispatch_post(B.PostDispatchTable(descs, None if with_mix else xs, mixes, posts, got), B.DTYPES[dt], B.DTYPES[dt])
    torch.cuda.synchronize()
    for j, (w_, g_) in enumerate(zip(want, got)):
        assert torch.equal(w_, g_), (j, mats[j].kind, mats[j].N, mats[j].K)
    # and against the oracle, fed with the plain projection the device stored
    for j, (m, y, g, o) in enumerate(zip(mats, plain, gates, got)):
        yf = host(y, dt).reshape(-1)
        if j % 3 == 0:
            assert np.array_equal(o.cpu().numpy().view(np.uint16).reshape(-1), MO.narrow(BO.relu_squared(yf).astype(np.float32), dt))
        elif j % 3 == 1:
            check_close(host(o, dt).reshape(-1), BO.channel_mixing_gate(host(g, dt), yf), dt, 0.0)


def test_block_chunk_through_quantized_projections():
    """A chunk of 192 tokens through one block (the prefill path: separate mix pass, matrix-core GEMMs,
    time-parallel wkv, element-wise passes), then 3 more tokens one by one (batch-1 path, fused mix,
    operators applied by the GEMVs) continuing from the carried states.  Every stage against the
    oracle fed with what the device held for that stage."""
    torch = G.torch_()
    rng = np.random.default_rng(9700)
    d, ffn, T, T1, dt = 512, 1024, 192, 3, "bf16"
    names = ["r", "k", "v", "o", "ck", "cr", "cv"]
    mats = dict(zip(names, [synth.gen_sq(rng, d, d), synth.gen_vq(rng, d, d, 6), synth.gen_vq(rng, d, d, 8),
                            synth.gen_sq(rng, d, d), synth.gen_vq(rng, ffn, d, 6), synth.gen_sq(rng, d, d),
                            synth.gen_vq(rng, d, ffn, 8)]))
    dms = {n: B.upload(m, native=True) for n, m in mats.items()}
    mixes = {n: (rng.integers(0, 64, size=d // 2, dtype=np.uint8), synth.gen_codebook(rng, 64).reshape(64, 2))
             for n in ("r", "k", "v", "ck", "cr")}
    mixd = {n: (dev(i), dev(c)) for n, (i, c) in mixes.items()}
    mu_hat = {n: orc.widen(c, "f16")[i].reshape(-1) for n, (i, c) in mixes.items()}
    _, _, _, w, u = synth.gen_block_inputs(rng, 1, d, dt)
    wd, ud = dev(w), dev(u)
    xs = synth.gen_activations(rng, T + T1 + 1, d, dt)            # row 0: the token before the chunk
    xd = dev(xs)
    DT = B.DTYPES[dt]
    W = lambda t: orc.widen(t.cpu().numpy().view(np.uint16), dt).astype(np.float64)
    lin = lambda n, x: orc.linear(mats[n], np.asarray(x, dtype=np.float32), "f64", weight_round=dt)
    rel = lambda got, ref: float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))
    narrow = lambda a: orc.widen(MO.narrow(np.asarray(a, dtype=np.float32), dt), dt)
    buf = lambda m, n: torch.zeros((m, n), dtype=torch.int16, device="cuda")
    # ---- the chunk ----
    mixed = {n: buf(T, d) for n in ("r", "k", "v")}
    B.rwkvq_token_shift_mix(xd[1:T + 1], xd[0], DT, T, d, B.MixTable([mixd[n][0] for n in ("r", "k", "v")],
                            [mixd[n][1] for n in ("r", "k", "v")], [mixed[n] for n in ("r", "k", "v")]), 6)
    y = {n: buf(T, mats[n].N) for n in names}
    B.rwkvq_linear_dispatch(B.DispatchTable([dms[n].desc() for n in ("r", "k", "v")], [mixed[n] for n in ("r", "k", "v")],
                                            [y[n] for n in ("r", "k", "v")]), T, DT, DT)
    state = fresh_state(d)
    gated = buf(T, d)
    B.rwkvq_wkv(y["r"], y["k"], y["v"], DT, T, d, wd, ud, state, gated)
    B.rwkvq_linear_dispatch(B.DispatchTable([dms["o"].desc()], [gated], [y["o"]]), T, DT, DT)
    o_before = buf(1, d)                                          # o of the token before the chunk: zeros
    mixed2 = {n: buf(T, d) for n in ("ck", "cr")}
    B.rwkvq_token_shift_mix(y["o"], o_before, DT, T, d, B.MixTable([mixd[n][0] for n in ("ck", "cr")],
                            [mixd[n][1] for n in ("ck", "cr")], [mixed2[n] for n in ("ck", "cr")]), 6)
    B.rwkvq_linear_dispatch(B.DispatchTable([dms[n].desc() for n in ("ck", "cr")], [mixed2[n] for n in ("ck", "cr")],
                                            [y[n] for n in ("ck", "cr")]), T, DT, DT)
    sq = buf(T, ffn)
    B.rwkvq_relu2(y["ck"], DT, T * ffn, sq)
    B.rwkvq_linear_dispatch(B.DispatchTable([dms["cv"].desc()], [sq], [y["cv"]]), T, DT, DT)
    out = buf(T, d)
    B.rwkvq_sigmoid_gate(y["cr"], y["cv"], DT, T * d, out)
    torch.cuda.synchronize()
    print("block chunk: stages", flush=True)
    xf = orc.widen(xs, dt)
    for n in ("r", "k", "v"):
        want_mix = MO.narrow(MO.token_shift_mix(xf[1:T + 1], xf[0], mu_hat[n]), dt)
        assert np.array_equal(mixed[n].cpu().numpy().view(np.uint16), want_mix), n
        assert rel(W(y[n]), lin(n, orc.widen(want_mix, dt))) <= 4e-3, n
    want_g = BO.time_mixing_gate(W(y["r"]), BO.wkv_direct(W(y["k"]), W(y["v"]), w, u))
    vmax = float(np.abs(W(y["v"])).max())
    tol = HALF_ULP[dt] * 1.01 * np.abs(want_g) + FLOOR[dt] + 2e-5 * vmax
    assert not (np.abs(W(gated) - want_g) > tol).any()
    assert rel(W(y["o"]), lin("o", W(gated))) <= 4e-3
    of = W(y["o"]).astype(np.float32)
    for n in ("ck", "cr"):
        want_mix = MO.narrow(MO.token_shift_mix(of, np.zeros(d, np.float32), mu_hat[n]), dt)
        assert np.array_equal(mixed2[n].cpu().numpy().view(np.uint16), want_mix), n
        assert rel(W(y[n]), lin(n, orc.widen(want_mix, dt))) <= 4e-3, n
    assert np.array_equal(sq.cpu().numpy().view(np.uint16), MO.narrow(BO.relu_squared(W(y["ck"])).astype(np.float32), dt))
    assert rel(W(y["cv"]), lin("cv", W(sq))) <= 4e-3
    check_close(W(out), BO.channel_mixing_gate(W(y["cr"]), W(y["cv"])), dt, 0.0)
    # ---- three more tokens, one by one, from the carried states ----
    hist_k, hist_v = list(W(y["k"])), list(W(y["v"]))
    o_prev = y["o"][T - 1:T].clone()
    for t in range(T + 1, T + T1 + 1):
        print(f"block chunk: token {t}", flush=True)
        x, xp = xd[t], xd[t - 1]
        y1 = {n: buf(1, mats[n].N) for n in names}
        g1, s1, out1 = buf(1, d), buf(1, ffn), buf(1, d)
        B.rwkvq_linear_dispatch_mixed(B.MixedDispatchTable([dms[n].desc() for n in ("r", "k", "v")],
                                      [(x, xp, *mixd[n], 6) for n in ("r", "k", "v")], [y1[n] for n in ("r", "k", "v")]), DT, DT)
        B.rwkvq_wkv(y1["r"], y1["k"], y1["v"], DT, 1, d, wd, ud, state, g1)
        B.rwkvq_linear_dispatch(B.DispatchTable([dms["o"].desc()], [g1], [y1["o"]]), 1, DT, DT)
        B.rwkvq_linear_dispatch_post(B.PostDispatchTable([dms[n].desc() for n in ("ck", "cr")], None,
                                     [(y1["o"], o_prev, *mixd[n], 6) for n in ("ck", "cr")],
                                     [(B.POST_RELU2, None), (B.POST_NONE, None)], [s1, y1["cr"]]), DT, DT)
        B.rwkvq_linear_dispatch_post(B.PostDispatchTable([dms["cv"].desc()], [s1], None, [(B.POST_SIGMOID_GATE, y1["cr"])],
                                                         [out1]), DT, DT)
        torch.cuda.synchronize()
        for n in ("r", "k", "v"):
            xm = narrow(MO.token_shift_mix(xf[t][None, :], xf[t - 1], mu_hat[n]))
            assert rel(W(y1[n]), lin(n, xm)) <= 4e-3, n
        hist_k.append(W(y1["k"])[0]); hist_v.append(W(y1["v"])[0])
        want = BO.time_mixing_gate(W(y1["r"])[0], BO.wkv_direct(np.array(hist_k), np.array(hist_v), w, u)[-1])
        check_close(W(g1)[0], want, dt, float(np.abs(np.array(hist_v)).max()))
        assert rel(W(y1["o"]), lin("o", W(g1))) <= 4e-3
        xm = {n: narrow(MO.token_shift_mix(W(y1["o"]).astype(np.float32), W(o_prev)[0].astype(np.float32), mu_hat[n])) for n in ("ck", "cr")}
        assert rel(W(y1["cr"]), lin("cr", xm["cr"])) <= 4e-3
        ck = narrow(lin("ck", xm["ck"]))                          # k' as the GEMV would have stored it
        # the GEMV stored max(k', 0)^2 directly (k' itself is not kept): where the oracle's k' rounds to the
        # neighbouring bf16 value (2^-8 relative) the square differs by twice that
        assert rel(W(s1), BO.relu_squared(ck)) <= 2e-2
        y_cv = lin("cv", W(s1))
        want_out = BO.channel_mixing_gate(W(y1["cr"]), narrow(y_cv))
        assert rel(W(out1), want_out) <= 1e-2
        o_prev = y1["o"]


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("N,K,P,op", [(4096, 512, 4, "gate"), (512, 3584, 2, "none"), (256, 256, 1, "relu2"), (8192, 256, 3, "gate")])
def test_post_mix_equals_projection_then_mix_pass(dt, N, K, P, op):
    """The output of a batch-1 projection also stored as the token-shift mixes of the next stage
    (rwkvq_post_op.n_mix) against the same call without them followed by rwkvq_token_shift_mix on the
    stored output: the same bits in the output and in every mix, for all three operators in front."""
    torch = G.torch_()
    rng = np.random.default_rng(9800 + N + K)
    mat = synth.gen_vq(rng, N, K, 6) if (N // 256) % 2 else synth.gen_sq(rng, N, K)
    dm = B.upload(mat, native=True)
    x = dev(synth.gen_activations(rng, 1, K, dt))
    gate = dev(synth.gen_activations(rng, 1, N, dt)[0])
    zprev = dev(synth.gen_activations(rng, 1, N, dt)[0])
    idx = [dev(rng.integers(0, 64, size=N // 2, dtype=np.uint8)) for _ in range(P)]
    cbs = [dev(synth.gen_codebook(rng, 64).reshape(64, 2)) for _ in range(P)]
    opc = {"none": B.POST_NONE, "relu2": B.POST_RELU2, "gate": B.POST_SIGMOID_GATE}[op]
    g = gate if op == "gate" else None
    buf = lambda: torch.zeros((1, N), dtype=torch.int16, device="cuda")
    z_ref, mix_ref = buf(), [buf() for _ in range(P)]
    B.rwkvq_linear_dispatch_post(B.PostDispatchTable([dm.desc()], [x], None, [(opc, g)], [z_ref]), B.DTYPES[dt], B.DTYPES[dt])
    B.rwkvq_token_shift_mix(z_ref, zprev, B.DTYPES[dt], 1, N, B.MixTable(idx, cbs, mix_ref), 6)
    z, mix = buf(), [buf() for _ in range(P)]
    print(f"post-mix {dt} N={N} K={K} P={P} op={op}", flush=True)
    B.rwkvq_linear_dispatch_post(B.PostDispatchTable([dm.desc()], [x], None,
                                 [(opc, g, zprev, [(idx[p], cbs[p], 6, mix[p]) for p in range(P)])], [z]), B.DTYPES[dt], B.DTYPES[dt])
    torch.cuda.synchronize()
    assert torch.equal(z, z_ref)
    for p in range(P):
        assert torch.equal(mix[p], mix_ref[p]), p
    # and the mix itself against the oracle on the stored output
    zf, zp = orc.widen(z.cpu().numpy().view(np.uint16).reshape(-1), dt), orc.widen(zprev.cpu().numpy().view(np.uint16), dt)
    for p in range(P):
        mu_hat = orc.widen(cbs[p].cpu().numpy().view(np.uint16), "f16").reshape(64, 2)[idx[p].cpu().numpy()].reshape(-1)
        want = MO.narrow(MO.token_shift_mix(zf[None, :], zp, mu_hat), dt)
        assert np.array_equal(mix[p].cpu().numpy().view(np.uint16), want), p


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("d,K,kinds", [(512, 512, ("sq", "vq6", "vq8")), (4096, 4096, ("vq6", "sq", "sq")), (256, 1792, ("vq8", "vq8", "sq"))])
def test_rkv_wkv_equals_dispatch_then_wkv(dt, d, K, kinds):
    """The three projections and the wkv step in one launch against rwkvq_linear_dispatch on the three
    matrices followed by rwkvq_wkv, token after token from the same starting state: the same bits in r, k,
    v, in the gated output and in the carried state whenever the two take their sums in the same order."""
    torch = G.torch_()
    rng = np.random.default_rng(9900 + d + K)
    mats = [synth.gen_sq(rng, d, K) if kd == "sq" else synth.gen_vq(rng, d, K, 6 if kd == "vq6" else 8) for kd in kinds]
    dms = [B.upload(m, native=True) for m in mats]
    descs = [m.desc() for m in dms]
    _, _, _, w, u = synth.gen_block_inputs(rng, 1, d, dt)
    wd, ud = dev(w), dev(u)
    buf = lambda: torch.zeros((1, d), dtype=torch.int16, device="cuda")
    ya, yb = [buf() for _ in range(3)], [buf() for _ in range(3)]
    ga, gb = buf(), buf()
    sa, sb = fresh_state(d), fresh_state(d)
    DT = B.DTYPES[dt]
    for t in range(4):
        xs = [dev(synth.gen_activations(rng, 1, K, dt)) for _ in range(3)]
        print(f"rkv+wkv {dt} d={d} K={K} {kinds} token {t}", flush=True)
        B.rwkvq_linear_dispatch(B.DispatchTable(descs, xs, ya), 1, DT, DT)
        B.rwkvq_wkv(ya[0], ya[1], ya[2], DT, 1, d, wd, ud, sa, ga)
        B.rwkvq_rkv_wkv(B.RkvWkvTable(descs, xs, yb), wd, ud, sb, gb, DT, DT)
        torch.cuda.synchronize()
        # the fused launch always splits a row's columns over four wavefronts; the dispatch of the three
        # matrices does so from 512 row tiles on (or trivially, with at most four column tiles): then the
        # binary32 sums are taken in the same order and every bit agrees; otherwise to rounding
        same_order = 3 * (d // 16) * 4 >= 2048 or K // 256 <= 4
        if same_order:
            for i in range(3):
                assert torch.equal(ya[i], yb[i]), ("rkv"[i], t)
            assert torch.equal(ga, gb), t
            assert torch.equal(sa, sb), t
        else:
            ulp = 2.0 ** -10 if dt == "f16" else 2.0 ** -7
            for i in range(3):
                a_, b_ = host(ya[i], dt), host(yb[i], dt)
                assert np.all(np.abs(a_ - b_) <= ulp * np.maximum(np.abs(a_), 2.0 ** -14)), ("rkv"[i], t)
            a_, b_ = host(ga, dt), host(gb, dt)
            assert np.all(np.abs(a_ - b_) <= 4 * ulp * np.maximum(np.abs(a_), 1e-3)), t
    assert not torch.equal(sb, fresh_state(d))
