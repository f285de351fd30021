"""CPU oracle of the element-wise multiplication path of Sec. 3.2 ("Codebook Optimization for
Element-wise Multiplication") and of the token-shift mix that consumes its result (Eq. "time
mixing r/k/v", Eq. "channel mixing r/k").

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU baseline may import this;
the GPU library never does, and this module imports nothing from the GPU package.

Three steps, in the order the section gives them:

1. clip_mean: the representative X of a calibration batch.  X must have the shape of the weight,
   so the batch is integrated per position: the samples of a position are limited to the range
   between their p-th and (100 - p)-th percentile and then averaged.
2. mu_codebook: weighted KMeans (Lloyd iterations) of the weight's d-vectors under the loss of
   Eq. "quantization loss of mul", sum_ij X_ij^2 (mu_ij - c_ij)^2: the weight of an element is the
   square of the representative activation at its position.
3. token_shift_mix: mu_hat * x_t + (1 - mu_hat) * x_{t-1} with mu_hat the de-quantized weight.

Readings (the paper is silent or ambiguous; also listed in the design notes):
  * the weight mu [m][n] is cut, row-major, into vectors of d = 2 consecutive elements (the VQ
    vector dimension of Eq. "VQ"; the section's "hidden dimension" is read as that d);
  * percentiles are taken per position over the samples of the batch, symmetric (p and 100 - p),
    with linear interpolation between order statistics: rank r = (B - 1) q / 100,
    value = v[floor r] + (r - floor r) (v[floor r + 1] - v[floor r]) in binary64; p is a parameter
    (the paper does not print it);
  * the mean is a binary64 sum over the samples in their order, divided by B, rounded to binary32;
    the element weight is that binary32 value squared in binary32;
  * Lloyd iterations start from a codebook the caller supplies (the draw of the initial entries is
    an input, not part of the method) and run a fixed number of times;
  * assignment: argmin_e fl( fl(fl(w0) * fl(fl(t0)^2)) + fl(fl(w1) * fl(fl(t1)^2)) ) with
    t = mu - c_e, all binary32, one rounding per operation; equal costs resolve to the lowest index;
  * update: entry e, coordinate j becomes sum w_ij mu_ij / sum w_ij over the vectors assigned to
    e, both sums in binary64; the quotient is rounded to fp16 at once (the stored precision of a
    codebook), so every iteration works with a storable codebook; an entry whose weight sum in a
    coordinate is zero keeps its value there;
  * after the last update one more assignment yields the indices that go with the final codebook;
  * mix, in binary32 with one rounding per operation: fl( fl(m * x_t) + fl( fl(1 - m) * x_prev ) ),
    then rounded once to the activation type; row 0 of a chunk takes x_{t-1} from the carried state.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def percentile_linear(v_sorted: np.ndarray, q: float) -> np.ndarray:
    """q-th percentile (0..100) of each column of v_sorted [B][n] (ascending along axis 0)."""
    B = v_sorted.shape[0]
    r = (B - 1) * (q / 100.0)
    k = int(np.floor(r))
    f = r - k
    lo = v_sorted[k].astype(np.float64)
    hi = v_sorted[min(k + 1, B - 1)].astype(np.float64)
    return lo + f * (hi - lo)


def clip_mean(X: np.ndarray, p: float) -> np.ndarray:
    """X: [B][n] calibration activations (already widened exactly to float32).  Returns the
    representative [n] float32: per position, samples clipped to [P_p, P_{100-p}] and averaged."""
    X = np.asarray(X, dtype=F32)
    B, n = X.shape
    s = np.sort(X, axis=0)
    lo = percentile_linear(s, p)
    hi = percentile_linear(s, 100.0 - p)
    acc = np.zeros(n, dtype=np.float64)
    for b in range(B):                                   # sequential binary64 sum, sample order
        acc += np.minimum(np.maximum(X[b].astype(np.float64), lo), hi)
    return (acc / B).astype(F32)


def element_weights(xbar: np.ndarray) -> np.ndarray:
    """X^2 of Eq. "quantization loss of mul" in binary32."""
    xbar = np.asarray(xbar, dtype=F32)
    return xbar * xbar


def f16_round(a: np.ndarray) -> np.ndarray:
    return np.asarray(a, dtype=np.float64).astype(np.float16)


def assign(mu2: np.ndarray, w2: np.ndarray, cb: np.ndarray) -> np.ndarray:
    """mu2, w2: [V][2] float32 vectors and element weights; cb: [E][2] float32.  Index of the
    cheapest entry per vector (lowest index on ties)."""
    mu2 = np.asarray(mu2, dtype=F32); w2 = np.asarray(w2, dtype=F32); cb = np.asarray(cb, dtype=F32)
    best = np.zeros(mu2.shape[0], dtype=np.int64)
    bestc = np.full(mu2.shape[0], np.inf, dtype=F32)
    for e in range(cb.shape[0]):
        t0 = mu2[:, 0] - cb[e, 0]
        t1 = mu2[:, 1] - cb[e, 1]
        c = w2[:, 0] * (t0 * t0) + w2[:, 1] * (t1 * t1)   # float32 ufuncs: one rounding each
        better = c < bestc
        best[better] = e
        bestc[better] = c[better]
    return best


def update(mu2: np.ndarray, w2: np.ndarray, idx: np.ndarray, cb: np.ndarray, round_fp16: bool = True) -> np.ndarray:
    """One centroid update; returns the new codebook [E][2] (float32 values, fp16-representable
    when round_fp16)."""
    E = cb.shape[0]
    num = np.zeros((E, 2), dtype=np.float64)
    den = np.zeros((E, 2), dtype=np.float64)
    wm = w2.astype(np.float64) * mu2.astype(np.float64)
    np.add.at(num, idx, wm)
    np.add.at(den, idx, w2.astype(np.float64))
    new = cb.astype(np.float64).copy()
    ok = den > 0
    new[ok] = num[ok] / den[ok]
    if round_fp16:
        return f16_round(new).astype(F32)
    return new                                           # binary64: plain weighted KMeans (used by the pins)


def mu_codebook(mu: np.ndarray, xbar: np.ndarray, cb0: np.ndarray, iters: int, round_fp16: bool = True):
    """mu: [n] float32 (row-major flattening of the weight), xbar: [n] float32 representative,
    cb0: [E][2] initial codebook (float32 values of fp16 entries).  Returns (codebook [E][2]
    float32, indices [n/2] int64, weighted loss as binary64)."""
    mu2 = np.asarray(mu, dtype=F32).reshape(-1, 2)
    w2 = element_weights(xbar).reshape(-1, 2)
    cb = np.array(cb0, dtype=F32 if round_fp16 else np.float64)
    for _ in range(iters):
        idx = assign(mu2, w2, cb.astype(F32))
        cb = update(mu2, w2, idx, cb, round_fp16)
    idx = assign(mu2, w2, cb.astype(F32))
    return cb, idx, weighted_loss(mu2, w2, cb, idx)


def weighted_loss(mu2, w2, cb, idx) -> float:
    d = mu2.astype(np.float64) - np.asarray(cb, dtype=np.float64)[idx]
    return float((w2.astype(np.float64) * d * d).sum())


def narrow(a: np.ndarray, dtype: str) -> np.ndarray:
    """float32 -> fp16 / bf16 bit patterns, round to nearest even (finite inputs)."""
    a = np.ascontiguousarray(a, dtype=F32)
    if dtype == "f16":
        return a.astype(np.float16).view(np.uint16)
    u = a.view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def token_shift_mix(x: np.ndarray, x_prev: np.ndarray, mu_hat: np.ndarray) -> np.ndarray:
    """x: [M][d] float32 activations of a chunk, x_prev: [d] the token before the chunk,
    mu_hat: [d] de-quantized weight.  Returns [M][d] float32 (before the final narrowing)."""
    x = np.asarray(x, dtype=F32); mu_hat = np.asarray(mu_hat, dtype=F32)
    shifted = np.concatenate([np.asarray(x_prev, dtype=F32)[None, :], x[:-1]], axis=0)
    a = mu_hat[None, :] * x
    b = (F32(1.0) - mu_hat)[None, :] * shifted
    return a + b
