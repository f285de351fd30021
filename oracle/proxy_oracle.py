"""CPU oracle of the coarse-to-fine proxy (Sec. 3.1, "Coarse-grained Proxy" and "Fine-grained
Proxy") that decides, per weight matrix, between SQ and VQ.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU baseline may import this;
the GPU library never does, and this module imports nothing from the GPU package.

The oracle is the paper's definition written out, step by step, in binary64:

    W' = sort(flatten(W))                          ascending
    G  = W'[1:] - W'[:-1]                          Eq. "interval";  n = oc*ic - 1 intervals
    G' = G / sum(G)                                Eq. "interval_norm"
    H(G') = - sum_i G'_i ln G'_i                   Eq. "ie", natural logarithm (the base Step 2
                                                   of the fine-grained proxy fixes), 0 ln 0 := 0
    P_c = H(uniform) - H(G') = ln n - H(G')        Eq. "coarse_proxy" with Eq. "absolute_case"
    delta = G' - 1/n                               Eq. "delta"
    M_k = (1/n) sum_i delta_i^k                    Eq. "taylor_refomulation" (k-th central moment)
    v_k = n^k / (k (k-1))
    P_f = sum_{k=2}^{K} v_k |M_k|                  Eq. "fine_proxy"
    phi = 1 (SQ) iff P_c < tau_c and P_f < tau_f   Eq. "multi_scale_proxy"; otherwise 0 (VQ)

Readings where the paper is silent (also listed in the design notes):
  * K: a hyper-parameter; a remark left in the source speaks of the first four terms, k = 2..5,
    which is the default here.
  * ties in W give intervals of length zero: 0 ln 0 := 0 (the limit), and delta_i = -1/n for them.
  * a constant matrix has sum(G) = 0 and no distribution to speak of: both proxies are reported
    as 0 (nothing argues against the uniform quantizer).
  * inputs are finite.
"""
from __future__ import annotations

import numpy as np

DEFAULT_TERMS = 5          # K of Eq. "fine_proxy": k = 2 .. 5


def intervals(W: np.ndarray) -> np.ndarray:
    """G of Eq. "interval" for the weights W (any shape), binary64."""
    w = np.sort(np.asarray(W, dtype=np.float64).ravel())
    return w[1:] - w[:-1]


def coarse(G: np.ndarray) -> float:
    """P_c of Eq. "coarse_proxy" from the intervals G."""
    n = G.size
    total = G.sum()
    if n == 0 or total == 0.0:
        return 0.0
    Gp = G / total
    pos = Gp[Gp > 0.0]
    H = -np.sum(pos * np.log(pos))
    return float(np.log(n) - H)


def fine(G: np.ndarray, terms: int = DEFAULT_TERMS) -> float:
    """P_f of Eq. "fine_proxy" from the intervals G, K = terms."""
    n = G.size
    total = G.sum()
    if n == 0 or total == 0.0:
        return 0.0
    delta = G / total - 1.0 / n
    Pf = 0.0
    for k in range(2, terms + 1):
        Mk = np.sum(delta ** k) / n
        vk = float(n) ** k / (k * (k - 1))
        Pf += vk * abs(Mk)
    return float(Pf)


def proxies(W: np.ndarray, terms: int = DEFAULT_TERMS):
    """(P_c, P_f) of a weight matrix."""
    G = intervals(W)
    return coarse(G), fine(G, terms)


def phi(Pc: float, Pf: float, tau_c: float, tau_f: float) -> int:
    """Eq. "multi_scale_proxy": 1 = SQ, 0 = VQ."""
    return 1 if (Pc < tau_c and Pf < tau_f) else 0


def widen16(bits: np.ndarray, dtype: str) -> np.ndarray:
    """fp16 / bf16 bit patterns -> float64 values (exact)."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError(dtype)
