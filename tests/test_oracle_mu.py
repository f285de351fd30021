"""Pins of the element-wise-multiplication oracle (Sec. 3.2): each function is checked against
something other than itself - a library routine it must reduce to, closed forms, invariants."""
import itertools

import numpy as np
import pytest

from oracle import mu_oracle as MO
from oracle import encode_oracle as EO


# ------------------------------------------------------------------ clip_mean

def test_percentile_matches_numpy():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((37, 50)).astype(np.float32)
    s = np.sort(X, axis=0)
    for q in (0.0, 1.0, 2.5, 10.0, 50.0, 90.0, 99.0, 100.0):
        want = np.percentile(X.astype(np.float64), q, axis=0)      # numpy's default: linear interpolation
        assert np.allclose(MO.percentile_linear(s, q), want, rtol=1e-14, atol=1e-15)


def test_clip_mean_p0_is_plain_mean():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((64, 33)).astype(np.float32)
    assert np.allclose(MO.clip_mean(X, 0.0), X.astype(np.float64).mean(axis=0), rtol=0, atol=2.0 ** -24)


def test_clip_mean_closed_form():
    # samples 0..100 at every position: the 10th / 90th percentiles are 10 and 90; ten samples below
    # clip to 10, ten above to 90, the rest keep their value: mean = (10*10 + sum(10..90) + 10*90)/101 = 50
    X = np.tile(np.arange(101, dtype=np.float32)[:, None], (1, 4))
    got = MO.clip_mean(X, 10.0)
    assert np.array_equal(got, np.full(4, 50.0, np.float32))
    # an asymmetric case by hand: samples {0, 1, 2, 3, 100}, p = 25: P25 = 1, P75 = 3 -> {1,1,2,3,3} -> 2
    X = np.array([[0.0], [1.0], [2.0], [3.0], [100.0]], dtype=np.float32)
    assert MO.clip_mean(X, 25.0)[0] == np.float32(2.0)
    # order of the samples does not matter for the clip bounds
    assert MO.clip_mean(X[::-1].copy(), 25.0)[0] == np.float32(2.0)


def test_clip_mean_outlier_is_bounded():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((128, 8)).astype(np.float32)
    Y = X.copy()
    Y[5, :] = 1e4                                          # one wild sample per position
    plain = Y.astype(np.float64).mean(axis=0)
    clipped = MO.clip_mean(Y, 1.0)
    assert np.all(np.abs(plain) > 50)                      # the plain mean is dragged away
    assert np.all(np.abs(clipped) < 1.0)                   # the clipped one stays near the centre
    hi = np.percentile(Y.astype(np.float64), 99.0, axis=0)
    assert np.all(clipped <= hi)


# ------------------------------------------------------------------ weighted KMeans

def _setup(seed, V=400, E=8):
    rng = np.random.default_rng(seed)
    mu = rng.uniform(0.0, 1.0, size=2 * V).astype(np.float32)
    xbar = rng.standard_normal(2 * V).astype(np.float32)
    cb0 = rng.uniform(0.0, 1.0, size=(E, 2)).astype(np.float16).astype(np.float32)
    return mu, xbar, cb0


def test_equal_weights_is_plain_kmeans():
    """With all weights equal the iteration is Lloyd's algorithm: scipy's kmeans2 from the same
    initial entries (no fp16 rounding of the centroids on either side)."""
    from scipy.cluster.vq import kmeans2
    mu, _, cb0 = _setup(3)
    ones = np.ones_like(mu)
    for iters in (1, 5):
        cb, idx, _ = MO.mu_codebook(mu, ones, cb0, iters, round_fp16=False)
        ref_cb, ref_idx = kmeans2(mu.reshape(-1, 2).astype(np.float64), cb0.astype(np.float64), iter=iters,
                                  minit="matrix", missing="raise")
        assert np.allclose(cb, ref_cb, rtol=1e-6, atol=1e-7)
        # scipy labels against the centroids before its last update; compare against ours one update earlier
        cbm, _, _ = MO.mu_codebook(mu, ones, cb0, iters - 1, round_fp16=False)
        assert np.array_equal(MO.assign(mu.reshape(-1, 2), np.ones((mu.size // 2, 2), np.float32), cbm.astype(np.float32)), ref_idx)


def test_assignment_reduces_to_vq_assign_with_unit_weights():
    mu, _, cb0 = _setup(4, V=256 * 128 // 2 // 64, E=64)    # any V; compare per vector
    mu2 = mu.reshape(-1, 2)
    got = MO.assign(mu2, np.ones_like(mu2), cb0)
    # brute force in binary64 on the same data: identical unless two entries are within rounding
    d = ((mu2[:, None, :].astype(np.float64) - cb0[None, :, :].astype(np.float64)) ** 2).sum(axis=2)
    want = d.argmin(axis=1)
    close = np.sort(d, axis=1)
    unambiguous = (close[:, 1] - close[:, 0]) > 1e-6
    assert np.array_equal(got[unambiguous], want[unambiguous]) and unambiguous.mean() > 0.95


def test_closed_form_two_clusters():
    # vectors near (0,0) and near (8,8); weights chosen by hand, all numbers exact in binary
    mu = np.array([0, 0, 1, 0, 0, 2, 8, 8, 10, 8], dtype=np.float32)          # 5 vectors
    xbar = np.array([1, 1, 2, 1, 1, 1, 1, 2, 1, 2], dtype=np.float32)          # weights = squares: 1,1,4,1,1,1,1,4,1,4
    cb0 = np.array([[1.0, 1.0], [7.0, 7.0]], dtype=np.float32)
    cb, idx, loss = MO.mu_codebook(mu, xbar, cb0, 1)
    assert idx.tolist() == [0, 0, 0, 1, 1]
    # entry 0: x = (1*0 + 4*1 + 1*0)/6 = 2/3, y = (1*0 + 1*0 + 1*2)/3 = 2/3; entry 1: x = (8 + 10)/2 = 9, y = 8
    assert cb[0, 0] == np.float32(np.float16(2.0 / 3.0)) and cb[0, 1] == np.float32(np.float16(2.0 / 3.0))
    assert cb[1, 0] == 9.0 and cb[1, 1] == 8.0
    want_loss = 0.0
    for v, e in zip(range(5), idx):
        for j in range(2):
            want_loss += float(xbar[2 * v + j]) ** 2 * (float(mu[2 * v + j]) - float(cb[e, j])) ** 2
    assert abs(loss - want_loss) < 1e-12


def test_weight_scaling_invariance_and_zero_weight():
    mu, xbar, cb0 = _setup(5)
    a = MO.mu_codebook(mu, xbar, cb0, 4)
    b = MO.mu_codebook(mu, xbar * np.float32(4.0), cb0, 4)                    # weights x 16: every product scales exactly
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # a coordinate with zero weight cannot influence anything: change mu there, nothing moves
    x0 = xbar.copy(); x0[0::2] = 0.0
    mu_b = mu.copy(); mu_b[0::2] += np.float32(0.37)
    c = MO.mu_codebook(mu, x0, cb0, 3)
    d = MO.mu_codebook(mu_b, x0, cb0, 3)
    assert np.array_equal(c[1], d[1]) and np.array_equal(c[0][:, 1], d[0][:, 1])
    assert np.array_equal(c[0][:, 0], cb0[:, 0])                             # zero weight sum: entries keep their value


def test_heavy_element_pins_its_entry():
    mu, xbar, cb0 = _setup(6, V=200, E=4)
    xbar = np.abs(xbar) * np.float32(0.01) + np.float32(0.01)
    xbar[10] = np.float32(1e4)                                               # element 10 = coordinate 0 of vector 5
    cb, idx, _ = MO.mu_codebook(mu, xbar, cb0, 6)
    e = idx[5]
    assert abs(float(cb[e, 0]) - float(mu[10])) <= 2.0 ** -11 * abs(float(mu[10])) + 1e-7


def test_loss_does_not_increase_without_rounding():
    mu, xbar, cb0 = _setup(7, V=600, E=16)
    prev = None
    for it in range(0, 7):
        _, _, loss = MO.mu_codebook(mu, xbar, cb0, it, round_fp16=False)
        if prev is not None:
            assert loss <= prev * (1 + 1e-9)
        prev = loss


def test_tiny_brute_force_fixed_point():
    """Six vectors, two entries: the partition Lloyd's iteration settles on is a fixed point, and no
    single reassignment lowers the weighted loss (checked by exhaustive search over partitions that
    differ in one vector)."""
    mu, xbar, cb0 = _setup(8, V=6, E=2)
    cb, idx, loss = MO.mu_codebook(mu, xbar, cb0, 20, round_fp16=False)
    mu2 = mu.reshape(-1, 2); w2 = MO.element_weights(xbar).reshape(-1, 2)
    again = MO.update(mu2, w2, idx, cb, round_fp16=False)
    assert np.allclose(again, cb, rtol=1e-12)
    for v in range(6):
        alt = idx.copy(); alt[v] ^= 1
        if len(set(alt.tolist())) < 2:
            continue
        assert MO.weighted_loss(mu2, w2, cb, alt) >= loss - 1e-12


# ------------------------------------------------------------------ token-shift mix

def test_mix_special_cases():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((5, 16)).astype(np.float32)
    xp = rng.standard_normal(16).astype(np.float32)
    shifted = np.concatenate([xp[None], x[:-1]])
    assert np.array_equal(MO.token_shift_mix(x, xp, np.ones(16, np.float32)), x)
    assert np.array_equal(MO.token_shift_mix(x, xp, np.zeros(16, np.float32)), shifted)
    xi = rng.integers(-8, 8, size=(5, 16)).astype(np.float32)
    xpi = rng.integers(-8, 8, size=16).astype(np.float32)
    half = MO.token_shift_mix(xi, xpi, np.full(16, 0.5, np.float32))
    assert np.array_equal(half, (xi + np.concatenate([xpi[None], xi[:-1]])) / 2)
    # hand value: mu = 0.25, x_t = 3, x_{t-1} = -5 -> 0.75 + (-3.75) = -3
    assert MO.token_shift_mix(np.array([[3.0]], np.float32), np.array([-5.0], np.float32), np.array([0.25], np.float32))[0, 0] == -3.0


def test_mix_matches_float64_within_rounding():
    rng = np.random.default_rng(10)
    x = rng.standard_normal((7, 64)).astype(np.float32)
    xp = rng.standard_normal(64).astype(np.float32)
    m = rng.uniform(0, 1, 64).astype(np.float16).astype(np.float32)
    got = MO.token_shift_mix(x, xp, m).astype(np.float64)
    sh = np.concatenate([xp[None], x[:-1]]).astype(np.float64)
    want = m.astype(np.float64) * x.astype(np.float64) + (1.0 - m.astype(np.float64)) * sh
    assert np.all(np.abs(got - want) <= 3 * 2.0 ** -24 * (np.abs(m * x) + np.abs((1 - m) * sh) + np.abs(want)) + 1e-12)


def test_narrow_matches_numpy_and_bits():
    a = np.array([1.0, 1.0009765625, 65504.0, -0.1, 3.140625], np.float32)
    assert np.array_equal(MO.narrow(a, "f16"), a.astype(np.float16).view(np.uint16))
    # bf16: 1.00390625 = 0x3F808000 is a tie -> even (0x3F80); 1.01171875 = 0x3F818000 -> 0x3F82
    b = np.array([1.00390625, 1.01171875], np.float32)
    assert MO.narrow(b, "bf16").tolist() == [0x3F80, 0x3F82]
