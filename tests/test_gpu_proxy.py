"""GPU parity of rwkvq_proxy (histogram formulation) against the proxy oracle (sort formulation):
binary64 on both sides, different summation orders -> relative 1e-9; the decision bit exact."""
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
