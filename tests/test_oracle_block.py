"""Pins of the block oracle (App. A.1): closed forms and invariants of Eq. "time mixing wkv" and of
the two gates."""
import numpy as np

from oracle import block_oracle as BO


def test_first_token_is_v():
    rng = np.random.default_rng(0)
    k = rng.standard_normal((1, 9)); v = rng.standard_normal((1, 9))
    out = BO.wkv_direct(k, v, rng.uniform(0.1, 1, 9), rng.standard_normal(9))
    assert np.allclose(out[0], v[0], rtol=1e-15)          # the sums over i < 1 are empty


def test_no_decay_no_bonus_equal_keys_is_the_running_mean():
    rng = np.random.default_rng(1)
    v = rng.standard_normal((7, 5))
    out = BO.wkv_direct(np.zeros((7, 5)), v, np.zeros(5), np.zeros(5))
    want = np.cumsum(v, axis=0) / np.arange(1, 8)[:, None]
    assert np.allclose(out, want, rtol=1e-14)


def test_two_tokens_by_hand():
    # d = 1: k = (0, ln 3), v = (2, 10), w = ln 2, u = ln 5
    # t = 2: past term exp(-(2-1-1) w + k_1) = 1, current exp(u + k_2) = 15 -> (2 + 150) / 16 = 9.5
    out = BO.wkv_direct(np.array([[0.0], [np.log(3.0)]]), np.array([[2.0], [10.0]]), np.array([np.log(2.0)]), np.array([np.log(5.0)]))
    assert abs(out[1, 0] - 9.5) < 1e-13
    # t = 3 with k_3 = 0, v_3 = -4: past exp(-w + 0) = 1/2 (i = 1), exp(0 + ln 3) = 3 (i = 2); current 5
    out = BO.wkv_direct(np.array([[0.0], [np.log(3.0)], [0.0]]), np.array([[2.0], [10.0], [-4.0]]), np.array([np.log(2.0)]), np.array([np.log(5.0)]))
    assert abs(out[2, 0] - (0.5 * 2 + 3 * 10 + 5 * -4) / 8.5) < 1e-13


def test_convex_combination_and_shift_invariance():
    rng = np.random.default_rng(2)
    k = rng.standard_normal((12, 6)) * 3; v = rng.standard_normal((12, 6))
    w = rng.uniform(0.05, 2, 6); u = rng.standard_normal(6)
    out = BO.wkv_direct(k, v, w, u)
    lo = np.minimum.accumulate(v, axis=0); hi = np.maximum.accumulate(v, axis=0)
    assert np.all(out >= lo - 1e-12) and np.all(out <= hi + 1e-12)
    # adding a constant to every key multiplies numerator and denominator alike
    assert np.allclose(BO.wkv_direct(k + 7.5, v, w, u), out, rtol=1e-12)
    # huge keys do not overflow, and a dominant current key returns (almost) the current value
    kk = k.copy(); kk[5] += 800.0
    big = BO.wkv_direct(kk, v, w, u)
    assert np.all(np.isfinite(big)) and np.allclose(big[5], v[5], rtol=1e-9)


def test_strong_decay_forgets_the_past():
    rng = np.random.default_rng(3)
    k = np.zeros((6, 4)); v = rng.standard_normal((6, 4))
    out = BO.wkv_direct(k, v, np.full(4, 60.0), np.zeros(4))
    # only i = t - 1 (undecayed) and the current token survive, with equal weight
    assert np.allclose(out[1:], (v[:-1] + v[1:]) / 2, rtol=1e-12)


def test_gates_and_relu_squared():
    assert BO.sigmoid(np.array([0.0]))[0] == 0.5
    x = np.array([-3.0, -0.5, 0.0, 0.25, 2.0])
    assert np.allclose(BO.sigmoid(x) + BO.sigmoid(-x), 1.0, rtol=1e-15)
    assert np.allclose(BO.sigmoid(np.array([np.log(3.0)])), 0.75, rtol=1e-15)
    assert np.array_equal(BO.relu_squared(x), np.array([0.0, 0.0, 0.0, 0.0625, 4.0]))
    assert np.allclose(BO.time_mixing_gate(np.array([0.0, np.log(3.0)]), np.array([4.0, -8.0])), [2.0, -6.0])
    assert np.allclose(BO.channel_mixing_gate(np.array([np.log(3.0)]), np.array([2.0])), [1.5])
