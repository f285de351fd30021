"""CPU oracle of the element-wise operators of the RWKV block as App. A.1 prints it (Eq. "time
mixing wkv", Eq. "time mixing o", Eq. "channel mixing o"), in binary64, each function the
printed formula written out.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU baseline may import this;
the GPU library never does, and this module imports nothing from the GPU package.

wkv_direct evaluates Eq. "time mixing wkv" for every t from all earlier k_i, v_i (the explicit sums,
O(T^2)); the only liberty is that numerator and denominator are divided by the same factor
exp(max exponent) before they are summed, which changes nothing mathematically and keeps the
exponentials finite.  The GPU path carries the sums as a running state instead (three numbers per
channel); that the two agree is what the parity test checks.

Readings (the appendix is the RWKV-4 form and leaves the following open; also in the design notes):
  * w is the per-channel decay with the sign of the printed exponent, -(t - 1 - i) w: positive w
    forgets; u is the per-channel bonus of the current token;
  * sigma is the logistic function 1 / (1 + exp(-x));
  * the blocks are chained as printed, without the normalisations and residual additions of the
    released models (the appendix prints none): the output o_t of time mixing is the input of
    channel mixing, whose output o'_t is the block's output;
  * intermediate vectors are stored in the activation type (fp16 / bf16) between kernels.
"""
from __future__ import annotations

import numpy as np


def sigmoid(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    return 1.0 / (1.0 + np.exp(-x))


def wkv_direct(k: np.ndarray, v: np.ndarray, w: np.ndarray, u: np.ndarray) -> np.ndarray:
    """k, v: [T][d]; w, u: [d].  wkv_t for t = 1..T (row t-1), Eq. "time mixing wkv"."""
    k = np.asarray(k, dtype=np.float64); v = np.asarray(v, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64); u = np.asarray(u, dtype=np.float64)
    T, d = k.shape
    out = np.empty((T, d), dtype=np.float64)
    for t in range(1, T + 1):                           # 1-based as printed
        # exponents of the terms i = 1 .. t-1 and of the current token
        i = np.arange(1, t)
        e_past = -(t - 1 - i)[:, None] * w[None, :] + k[:t - 1]          # [t-1][d]
        e_now = u + k[t - 1]                                              # [d]
        m = np.maximum(e_past.max(axis=0), e_now) if t > 1 else e_now
        num = (np.exp(e_past - m) * v[:t - 1]).sum(axis=0) + np.exp(e_now - m) * v[t - 1]
        den = np.exp(e_past - m).sum(axis=0) + np.exp(e_now - m)
        out[t - 1] = num / den
    return out


def time_mixing_gate(r: np.ndarray, wkv: np.ndarray) -> np.ndarray:
    """sigma(r_t) (.) wkv_t: the input of W_o in Eq. "time mixing o"."""
    return sigmoid(r) * np.asarray(wkv, dtype=np.float64)


def relu_squared(kp: np.ndarray) -> np.ndarray:
    """max(k'_t, 0)^2: the input of W'_v in Eq. "channel mixing o"."""
    kp = np.asarray(kp, dtype=np.float64)
    return np.maximum(kp, 0.0) ** 2


def channel_mixing_gate(rp: np.ndarray, y: np.ndarray) -> np.ndarray:
    """sigma(r'_t) (.) y with y = W'_v max(k'_t, 0)^2: Eq. "channel mixing o"."""
    return sigmoid(rp) * np.asarray(y, dtype=np.float64)
