"""GPU parity of rwkvq_proxy against the proxy oracle (the sort-based definition in numpy): 16-bit
matrices through the set-of-patterns formulation, binary32 matrices through the radix sort; binary64 on
both sides, different summation orders -> relative 1e-9; the decision bit exact."""
import numpy as np
import pytest

from oracle import proxy_oracle as PO
from paper_2505_03803_amd import synth

pytestmark = pytest.mark.gpu

REL = 1e-9


def run(bits, dtype, terms=5, tau_c=1.5, tau_f=50.0):
    import torch
    from paper_2505_03803_amd import binding as B
    w = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return B.proxy([w], B.DTYPES[dtype], terms, tau_c, tau_f)[0]


def check(bits, dtype, terms=5):
    print(f"proxy {dtype} shape={bits.shape} terms={terms}", flush=True)
    ePc, ePf = PO.proxies(PO.widen16(bits, dtype), terms)
    Pc, Pf, _ = run(bits, dtype, terms)
    assert Pc == pytest.approx(ePc, rel=REL, abs=1e-12), (Pc, ePc)
    assert Pf == pytest.approx(ePf, rel=REL, abs=1e-12), (Pf, ePf)
    return ePc, ePf


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("N,K", [(64, 96), (7, 333), (1, 2), (240, 256), (240, 257), (1024, 1024), (1536, 4100)])
def test_proxy_small(dtype, N, K):
    # 240 x 256 = one full counting chunk exactly, 240 x 257 one chunk and a ragged one,
    # 7 x 333 and 1 x 2 ragged only, the last two span many workgroups
    rng = np.random.default_rng(N * 131 + K)
    check(synth.gen_dense_weights(rng, N, K, dtype), dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_proxy_outliers_and_terms(dtype):
    rng = np.random.default_rng(5)
    bits = synth.gen_dense_weights(rng, 512, 768, dtype, outlier_fraction=1e-3, outlier_scale=30.0)
    for terms in (2, 3, 5, 8):
        check(bits, dtype, terms)


def test_proxy_degenerate_inputs():
    # a constant matrix; two values; both zeros (-0 < +0 as patterns, equal as numbers); every
    # finite fp16 pattern once
    const = np.full((16, 32), 0x3C00, np.uint16)
    assert run(const, "f16")[:2] == (0.0, 0.0)
    two = np.array([[0x3C00] * 31 + [0x4000] * 33], np.uint16)
    check(two, "f16")
    zeros = np.array([[0x0000, 0x8000, 0x0000, 0x8000, 0x3C00, 0xBC00, 0x0001, 0x8001]], np.uint16)
    check(zeros, "f16")
    allfinite = np.array([b for b in range(65536) if (b & 0x7C00) != 0x7C00], np.uint16).reshape(1, -1)
    check(allfinite, "f16")
    allbf = np.array([b for b in range(65536) if (b & 0x7F80) != 0x7F80], np.uint16).reshape(1, -1)
    check(allbf, "bf16", terms=4)


def test_proxy_decision_bit():
    rng = np.random.default_rng(6)
    bits = synth.gen_dense_weights(rng, 256, 512, "bf16")
    ePc, ePf = PO.proxies(PO.widen16(bits, "bf16"))
    for tau_c, tau_f in ((ePc * 2, ePf * 2), (ePc * 2, ePf / 2), (ePc / 2, ePf * 2), (ePc / 2, ePf / 2)):
        assert run(bits, "bf16", 5, tau_c, tau_f)[2] == PO.phi(ePc, ePf, tau_c, tau_f)


def test_proxy_many_matrices_in_one_call():
    """70 matrices of mixed shapes: two launches of the grouped kernels, results per matrix."""
    import torch
    from paper_2505_03803_amd import binding as B
    rng = np.random.default_rng(8)
    shapes = [(64 + 16 * (i % 5), 96 + 8 * (i % 7)) for i in range(69)] + [(1024, 1536)]
    mats = [synth.gen_dense_weights(rng, N, K, "bf16", outlier_fraction=1e-3 * (i % 3)) for i, (N, K) in enumerate(shapes)]
    got = B.proxy([torch.from_numpy(m.view(np.int16)).cuda() for m in mats], B.BF16, 5, 9.0, 1e12)
    for m, (Pc, Pf, flag) in zip(mats, got):
        ePc, ePf = PO.proxies(PO.widen16(m, "bf16"))
        assert Pc == pytest.approx(ePc, rel=REL) and Pf == pytest.approx(ePf, rel=REL)
        assert flag == PO.phi(ePc, ePf, 9.0, 1e12)


@pytest.mark.parametrize("N,K", [(4096, 4096), (4096, 14336)])
def test_proxy_full_size(N, K):
    """The two matrix shapes of the RWKV-6-7B-shaped stack, in the launch shape the benchmark times."""
    rng = np.random.default_rng(7)
    bits = synth.gen_dense_weights(rng, N, K, "bf16", outlier_fraction=1e-4)
    check(bits, "bf16")


# ------------------------------------------------------------------ binary32 matrices: really sorted

def run32(w, terms=5, tau_c=1.5, tau_f=50.0):
    import torch
    from paper_2505_03803_amd import binding as B
    return B.proxy([torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32)).cuda()], B.F32, terms, tau_c, tau_f)[0]


def check32(w, terms=5):
    print(f"proxy f32 shape={w.shape} terms={terms}", flush=True)
    ePc, ePf = PO.proxies(w.astype(np.float64), terms)
    Pc, Pf, _ = run32(w, terms)
    assert Pc == pytest.approx(ePc, rel=REL, abs=1e-12), (Pc, ePc)
    assert Pf == pytest.approx(ePf, rel=REL, abs=1e-12), (Pf, ePf)
    return ePc, ePf


@pytest.mark.parametrize("N,K", [(1, 2), (7, 333), (64, 64), (1, 4096), (1, 4097), (240, 257), (1024, 1024), (1536, 4100)])
def test_proxy_f32_small(N, K):
    # 1 x 4096 = one sort tile exactly, 1 x 4097 a tile and one key, the last two many tiles with a ragged one
    rng = np.random.default_rng(N * 17 + K)
    check32(synth.gen_dense_weights(rng, N, K, "f32", outlier_fraction=1e-3))


def test_proxy_f32_sorted_keys_in_the_workspace():
    """White box: after the call the second key buffer of the workspace holds the sorted keys (the
    order-preserving image of the binary32 patterns).  Compared with numpy's sort of the same keys,
    for values of both signs, both zeros, subnormals and many ties."""
    import torch
    from paper_2505_03803_amd import binding as B
    rng = np.random.default_rng(77)
    n = 3 * 4096 + 123
    w = (rng.standard_normal(n) * rng.choice([1e-30, 1e-3, 1.0, 1e20], size=n)).astype(np.float32)
    w[::7] = w[5]                                   # ties
    w[1::97] = 0.0; w[2::97] = -0.0; w[3::101] = 1e-45      # both zeros, the smallest subnormal
    wd = torch.from_numpy(w.reshape(1, n)).cuda()
    table = B.ProxyTable([wd], [(1, n)])
    size = B.rwkvq_proxy_workspace_size(table, B.F32)
    wsp = torch.zeros(size // 4, dtype=torch.int32, device="cuda")
    out = torch.zeros(2, dtype=torch.float64, device="cuda"); phi = torch.zeros(4, dtype=torch.int32, device="cuda")
    B.rwkvq_proxy(table, B.F32, 5, 1.5, 50.0, wsp, out, phi)
    torch.cuda.synchronize()
    bits = w.view(np.uint32)
    keys = np.where(bits & 0x80000000, ~bits, bits | 0x80000000).astype(np.uint32)
    second = (n * 4 + 255) // 256 * 256 // 4        # the second buffer starts at the next multiple of 256 bytes
    got = wsp[second:second + n].cpu().numpy().view(np.uint32)
    assert np.array_equal(got, np.sort(keys))
    # and the keys order the values: decoding the sorted keys gives numpy's sort of the values
    back = np.where(got & 0x80000000, got & 0x7FFFFFFF, ~got).astype(np.uint32).view(np.float32)
    assert np.array_equal(back, np.sort(w))


def test_proxy_f32_degenerate_and_ties():
    const = np.full((16, 32), 0.375, np.float32)
    assert run32(const)[:2] == (0.0, 0.0)
    two = np.array([[1.0] * 31 + [2.0] * 33], np.float32)
    check32(two)
    zeros = np.array([[0.0, -0.0, 0.0, -0.0, 1.0, -1.0, 1e-45, -1e-45]], np.float32)
    check32(zeros)
    # equally spaced weights: P_c = P_f = 0 (Eq. "absolute_case"), in any arrangement
    W = np.random.default_rng(3).permutation(np.arange(8193, dtype=np.float32) * 0.25 - 100.0).reshape(1, -1)
    Pc, Pf, _ = run32(W)
    assert abs(Pc) < 1e-12 and abs(Pf) < 1e-9
    # the same values as 16-bit and as binary32 matrices: the two formulations agree
    rng = np.random.default_rng(4)
    bits = synth.gen_dense_weights(rng, 300, 500, "bf16", outlier_fraction=1e-3)
    a = run(bits, "bf16")
    b = run32(PO.widen16(bits, "bf16").astype(np.float32))
    assert a[0] == pytest.approx(b[0], rel=REL) and a[1] == pytest.approx(b[1], rel=REL)


def test_proxy_f32_terms_decision_and_several_matrices():
    import torch
    from paper_2505_03803_amd import binding as B
    rng = np.random.default_rng(9)
    w = synth.gen_dense_weights(rng, 200, 300, "f32", outlier_fraction=1e-2, outlier_scale=30.0)
    for terms in (2, 3, 8):
        check32(w, terms)
    ePc, ePf = PO.proxies(w.astype(np.float64))
    for tau_c, tau_f in ((ePc * 2, ePf * 2), (ePc * 2, ePf / 2), (ePc / 2, ePf * 2), (ePc / 2, ePf / 2)):
        assert run32(w, 5, tau_c, tau_f)[2] == PO.phi(ePc, ePf, tau_c, tau_f)
    # matrices of different sizes in one call share the sort buffers, largest in the middle
    shapes = [(64, 100), (513, 1000), (7, 9), (256, 256)]
    mats = [synth.gen_dense_weights(rng, N, K, "f32", outlier_fraction=1e-3 * i) for i, (N, K) in enumerate(shapes)]
    got = B.proxy([torch.from_numpy(m).cuda() for m in mats], B.F32, 5, 0.5, 1e6)
    for m, (Pc, Pf, flag) in zip(mats, got):
        ePc, ePf = PO.proxies(m.astype(np.float64))
        assert Pc == pytest.approx(ePc, rel=REL) and Pf == pytest.approx(ePf, rel=REL)
        assert flag == PO.phi(ePc, ePf, 0.5, 1e6)


@pytest.mark.parametrize("N,K", [(4096, 4096), (4096, 14336)])
def test_proxy_f32_full_size(N, K):
    """The two matrix shapes of the RWKV-6-7B-shaped stack as binary32 (16.8 M and 58.7 M keys)."""
    rng = np.random.default_rng(12)
    check32(synth.gen_dense_weights(rng, N, K, "f32", outlier_fraction=1e-4))
