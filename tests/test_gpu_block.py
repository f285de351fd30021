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
