"""Pins for the oracle's contraction y[m,n] = sum_k w[n,k] x[m,k] (the W. products of App. A.1)."""
from fractions import Fraction

import numpy as np

from oracle import rwkvq_oracle as orc
from paper_2505_03803_amd import synth


def _small(seed=0, N=256, K=256, M=3):
    rng = np.random.default_rng(seed)
    sq = synth.gen_sq(rng, N, K)
    vq = synth.gen_vq(rng, N, K, 6)
    x = orc.widen(synth.gen_activations(rng, M, K, "f16"), "f16")
    return sq, vq, x


def test_f64_matches_numpy_matmul_and_rationals():
    sq, vq, x = _small()
    for m in (sq, vq):
        w = orc.dequant(m)
        y = orc.gemm(w, x, "f64")
        ref = x.astype(np.float64) @ w.astype(np.float64).T
        assert np.allclose(y, ref, rtol=1e-12, atol=1e-13)
        # brute force with exact rationals on a few outputs
        for (mm, n) in ((0, 0), (2, 255), (1, 17)):
            ex = sum(Fraction(float(w[n, k])) * Fraction(float(x[mm, k])) for k in range(256))
            assert abs(y[mm, n] - float(ex)) <= 1e-13 * max(1.0, abs(float(ex)))


def test_operands_are_not_transposed():
    # non-square: W is [N, K], x is [M, K], y is [M, N]
    rng = np.random.default_rng(1)
    w = rng.standard_normal((5, 7)).astype(np.float32)
    x = rng.standard_normal((2, 7)).astype(np.float32)
    y = orc.gemm(w, x, "f64")
    assert y.shape == (2, 5)
    for m in range(2):
        for n in range(5):
            assert abs(y[m, n] - sum(float(w[n, k]) * float(x[m, k]) for k in range(7))) < 1e-12


def test_f32_accumulates_sequentially_in_k():
    # (1e8 + 1) - 1e8 in binary32, k ascending, is 0; any pairwise or reversed order gives 1 or 0
    # differently: [1e8, 1, -1e8] -> 0 ; [1, 1e8, -1e8] -> 0 ; [1e8, -1e8, 1] -> 1
    x = np.ones((1, 3), np.float32)
    assert orc.gemm(np.array([[1e8, 1, -1e8]], np.float32), x, "f32")[0, 0] == 0.0
    assert orc.gemm(np.array([[1e8, -1e8, 1]], np.float32), x, "f32")[0, 0] == 1.0
    assert orc.gemm(np.array([[1e8, 1, -1e8]], np.float32), x, "f64")[0, 0] == 1.0
    # products are rounded to binary32 before the add: (1+2^-12)^2 = 1 + 2^-11 + 2^-24 -> 1 + 2^-11
    a = np.float32(1 + 2.0 ** -12)
    y = orc.gemm(np.array([[a, -1.0]], np.float32), np.array([[a, 1.0]], np.float32), "f32")[0, 0]
    assert y == 2.0 ** -11


def test_one_hot_input_returns_weight_column_exactly():
    sq, vq, _ = _small(2)
    for m in (sq, vq):
        w = orc.dequant(m)
        for k in (0, 127, 128, 255):
            x = np.zeros((1, 256), np.float32)
            x[0, k] = 1.0
            for acc in ("f32", "f64"):
                assert np.array_equal(orc.linear(m, x, acc)[0], w[:, k].astype(np.float64))


def test_ones_input_gives_row_sums_and_linearity():
    sq, vq, x = _small(3)
    for m in (sq, vq):
        w = orc.dequant(m)
        y1 = orc.linear(m, np.ones((1, 256), np.float32), "f64")[0]
        assert np.allclose(y1, w.astype(np.float64).sum(axis=1), rtol=1e-12, atol=1e-12)
        ya = orc.linear(m, x, "f32")
        yb = orc.linear(m, 2 * x, "f32")
        assert np.array_equal(yb, 2 * ya)            # scaling by 2 is exact in binary arithmetic


def test_batched_rows_equal_separate_vectors_and_linear_equals_dequant_plus_gemm():
    sq, vq, x = _small(4)
    for m in (sq, vq):
        y = orc.linear(m, x, "f32")
        for r in range(x.shape[0]):
            assert np.array_equal(orc.linear(m, x[r:r + 1], "f32")[0], y[r])
        assert np.array_equal(orc.gemm(orc.dequant(m), x, "f32"), y)
        for rnd in ("bf16", "f16"):
            assert np.array_equal(orc.gemm(orc.round_weights(orc.dequant(m), rnd), x, "f32"),
                                  orc.linear(m, x, "f32", weight_round=rnd))


def test_constant_codebook_gives_even_odd_sums():
    rng = np.random.default_rng(5)
    vq = synth.gen_vq(rng, 256, 512, 6)
    c0, c1 = np.float16(0.375), np.float16(-1.5)
    cb = np.empty((1, 2, 64, 2), np.float16)
    cb[..., 0], cb[..., 1] = c0, c1
    vq.codebooks = cb.view(np.uint16)
    x = orc.widen(synth.gen_activations(rng, 2, 512, "f16"), "f16")
    y = orc.linear(vq, x, "f64")
    want = float(c0) * x[:, 0::2].astype(np.float64).sum(1) + float(c1) * x[:, 1::2].astype(np.float64).sum(1)
    assert np.allclose(y, want[:, None], rtol=1e-12, atol=1e-12)


def test_f32_sum_is_accurate_on_config1():
    mat, xb = synth.config1()
    x = orc.widen(xb, "f16")
    y32 = orc.linear(mat, x, "f32")
    y64 = orc.linear(mat, x, "f64")
    assert np.abs(y32 - y64).max() / np.abs(y64).max() < 1e-5


def test_config1_is_deterministic_and_shaped():
    a, xa = synth.config1()
    b, xb = synth.config1()
    assert np.array_equal(a.codes, b.codes) and np.array_equal(xa, xb)
    assert a.codes.shape == (1024, 96) and a.scales.shape == (1024, 8) and xa.shape == (1, 1024)
    assert a.packed_bytes == 425984
    s = a.scales.view(np.float16).astype(np.float32)
    z = a.zeros.view(np.float16).astype(np.float32)
    assert 0.0049 < s.min() and s.max() < 0.0201 and 0 <= z.min() and z.max() <= 7
