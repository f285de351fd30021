"""Seeded synthetic workloads for the quantized-linear path.

This module only draws random bytes and floats and lays them out in the
interchange ("canonical") format; it contains none of the method's arithmetic
(no unpacking, no dequantization, no contraction), so both the CPU oracle's
tests and the HIP path's tests may take their inputs from it.

Canonical format of one weight matrix W of shape [N, K] (N = output channels,
K = input channels, y = x W^T):

* scalar-quantized (SQ, Eq. "SQ" of Sec. 2.2): ``codes`` is uint32
  [N, 3K/32]; row n is a little-endian bit string holding K 3-bit codes, code k
  at bits [3k, 3k+3).  ``scales`` and ``zeros`` are fp16 bit patterns (uint16)
  of shape [N, K/128]: one pair per group of 128 consecutive input channels.
* vector-quantized (VQ, Eq. "VQ" of Sec. 2.2, vector dimension d = 2):
  ``codes`` is uint32 [N, (K/2)*kbits/32]; row n holds K/2 indices of kbits
  bits each, index j (covering columns 2j, 2j+1) at bits [kbits*j, kbits*(j+1)).
  ``codebooks`` is fp16 bits (uint16) of shape [N/256, K/256, 2^kbits, 2]: one
  codebook per 256 x 256 block of W.

Because every 3-, 6- and 8-bit pattern is a valid code, uniformly random words
are uniformly random codes: no packing routine is needed here.

Random streams: weights of a configuration come from
``default_rng(SeedSequence([seed, 0]))`` in matrix order (per matrix: kind
flag, [index width], codes, scales, zeros | codebooks); activations for batch
size M come from ``default_rng(SeedSequence([seed, 1, M]))`` in matrix order,
so the same matrices can be paired with several batch sizes.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, Optional, Tuple

import numpy as np

SQ_BITS = 3
SQ_GROUP = 128
VQ_DIM = 2
VQ_BLOCK = 256

# name, N-as-multiple, K-as-multiple of (d, ffn): the RWKV-6 per-layer list.
_LAYER = (
    ("tm_receptance", "d", "d"),
    ("tm_key", "d", "d"),
    ("tm_value", "d", "d"),
    ("tm_gate", "d", "d"),
    ("tm_output", "d", "d"),
    ("cm_key", "ffn", "d"),
    ("cm_value", "d", "ffn"),
    ("cm_receptance", "d", "d"),
)


@dataclass
class QMatrix:
    name: str
    kind: str            # "sq" or "vq"
    N: int
    K: int
    kbits: int           # VQ index width (6 or 8); 0 for SQ
    codes: np.ndarray    # uint32 [N, words_per_row]
    scales: Optional[np.ndarray] = None     # uint16 [N, K/128]  (SQ)
    zeros: Optional[np.ndarray] = None      # uint16 [N, K/128]  (SQ)
    codebooks: Optional[np.ndarray] = None  # uint16 [N/256, K/256, 2^kbits, 2]  (VQ)

    @property
    def packed_bytes(self) -> int:
        """Bytes of everything that stands for W in memory."""
        b = self.codes.nbytes
        for a in (self.scales, self.zeros, self.codebooks):
            if a is not None:
                b += a.nbytes
        return b


def f32_to_f16_bits(a: np.ndarray) -> np.ndarray:
    return np.asarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Nearest-even narrowing of finite float32 values to bfloat16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def gen_sq(rng: np.random.Generator, N: int, K: int, name: str = "sq") -> QMatrix:
    assert K % SQ_GROUP == 0 and (K * SQ_BITS) % 32 == 0
    codes = rng.integers(0, 1 << 32, size=(N, K * SQ_BITS // 32), dtype=np.uint32)
    scales = f32_to_f16_bits(rng.uniform(0.005, 0.02, size=(N, K // SQ_GROUP)))
    zeros = f32_to_f16_bits(rng.uniform(0.0, 7.0, size=(N, K // SQ_GROUP)))
    return QMatrix(name, "sq", N, K, 0, codes, scales=scales, zeros=zeros)


def gen_vq(rng: np.random.Generator, N: int, K: int, kbits: int, name: str = "vq") -> QMatrix:
    assert N % VQ_BLOCK == 0 and K % VQ_BLOCK == 0 and kbits in (6, 8)
    codes = rng.integers(0, 1 << 32, size=(N, (K // VQ_DIM) * kbits // 32), dtype=np.uint32)
    cb = rng.normal(0.0, 0.02, size=(N // VQ_BLOCK, K // VQ_BLOCK, 1 << kbits, VQ_DIM))
    return QMatrix(name, "vq", N, K, kbits, codes, codebooks=f32_to_f16_bits(cb))


def gen_activations(rng: np.random.Generator, M: int, K: int, dtype: str) -> np.ndarray:
    """[M, K] standard-normal activations as fp16 or bf16 bit patterns (uint16)."""
    a = rng.standard_normal(size=(M, K), dtype=np.float32)
    if dtype == "f16":
        return f32_to_f16_bits(a)
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    raise ValueError(dtype)


def _rngs(seed: int, M: int) -> Tuple[np.random.Generator, np.random.Generator]:
    return (np.random.default_rng(np.random.SeedSequence([seed, 0])),
            np.random.default_rng(np.random.SeedSequence([seed, 1, M])))


def config1(M: int = 1) -> Tuple[QMatrix, np.ndarray]:
    """Single SQ matrix 1024 x 1024, fp16 activations, seed 0."""
    wr, ar = _rngs(0, M)
    return gen_sq(wr, 1024, 1024, "c1_sq"), gen_activations(ar, M, 1024, "f16")


def config2(M: int = 1) -> Tuple[QMatrix, np.ndarray]:
    """Single VQ matrix 4096 x 4096, 6-bit indices, fp16 activations, seed 1."""
    wr, ar = _rngs(1, M)
    return gen_vq(wr, 4096, 4096, 6, "c2_vq"), gen_activations(ar, M, 4096, "f16")


STACKS = {
    # config: (seed, d, ffn, layers, activation dtype, 8-bit-index VQ variants allowed)
    3: (2, 4096, 14336, 32, "f16", False),
    4: (3, 4096, 14336, 32, "bf16", False),
    5: (4, 5120, 17920, 48, "bf16", True),
}
STACK_M = {3: (1,), 4: (2048,), 5: (1, 16, 4096)}


def layer_shapes(d: int, ffn: int):
    dims = {"d": d, "ffn": ffn}
    return [(nm, dims[n], dims[k]) for nm, n, k in _LAYER]


def stack(config: int, M: int, n_layers: Optional[int] = None,
          with_activations: bool = True) -> Iterator[Tuple[QMatrix, Optional[np.ndarray]]]:
    """Yield (matrix, activations) for the layer stack of configuration 3, 4 or 5.

    Matrices come layer by layer in the fixed per-layer order; ``n_layers``
    truncates the stack (the first layers are identical to the full stack's).
    Each matrix is SQ or VQ with probability 1/2; in configuration 5 a VQ matrix
    has 6- or 8-bit indices with probability 1/2 each.
    """
    seed, d, ffn, layers, dt, k8 = STACKS[config]
    wr, ar = _rngs(seed, M)
    for layer in range(layers if n_layers is None else min(n_layers, layers)):
        for nm, N, K in layer_shapes(d, ffn):
            name = f"L{layer}.{nm}"
            is_sq = bool(wr.random() < 0.5)
            if is_sq:
                mat = gen_sq(wr, N, K, name)
            else:
                kbits = 6
                if k8:
                    kbits = 6 if wr.random() < 0.5 else 8
                mat = gen_vq(wr, N, K, kbits, name)
            x = gen_activations(ar, M, K, dt) if with_activations else None
            yield mat, x


def gen_dense_weights(rng: np.random.Generator, N: int, K: int, dtype: str = "bf16", sigma: float = 0.02,
                      outlier_fraction: float = 0.0, outlier_scale: float = 20.0) -> np.ndarray:
    """A dense weight matrix as the proxy of Sec. 3.1 sees it: [N][K] fp16 / bf16 bit patterns (or, for
    dtype "f32", binary32 values: a master copy of the weights, with few equal values) of N(0, sigma) values, a fraction of them multiplied by outlier_scale (the stored precision of
    RWKV checkpoints is 16 bits; trained matrices are near-Gaussian with a few large entries)."""
    w = rng.standard_normal((N, K), dtype=np.float32) * np.float32(sigma)
    if outlier_fraction > 0.0:
        mask = rng.random((N, K)) < outlier_fraction
        w = np.where(mask, w * np.float32(outlier_scale), w).astype(np.float32)
    if dtype == "f32":
        return w
    return f32_to_f16_bits(w) if dtype == "f16" else f32_to_bf16_bits(w)


def gen_mu(rng: np.random.Generator, n: int, dtype: str = "bf16") -> np.ndarray:
    """A token-shift mix weight as RWKV checkpoints hold it: n values in (0, 1), 16-bit storage
    (fp16 / bf16 bit patterns).  Trained mix weights fill the unit interval unevenly; a Beta(2, 3)
    draw stands in for them."""
    v = rng.beta(2.0, 3.0, size=n).astype(np.float32)
    return f32_to_f16_bits(v) if dtype == "f16" else f32_to_bf16_bits(v)


def gen_calibration(rng: np.random.Generator, n_samples: int, n: int, dtype: str = "bf16",
                    outlier_fraction: float = 0.01, outlier_scale: float = 30.0) -> np.ndarray:
    """[n_samples][n] calibration activations for the element-wise multiplication (Sec. 3.2 and
    its ablation: near-normal per channel, a per-channel offset and scale, a small fraction of
    samples far out) as fp16 / bf16 bit patterns or float32 (dtype "f32")."""
    loc = rng.normal(0.0, 0.5, size=n).astype(np.float32)
    scale = rng.uniform(0.5, 2.0, size=n).astype(np.float32)
    x = rng.standard_normal((n_samples, n), dtype=np.float32) * scale[None, :] + loc[None, :]
    mask = rng.random((n_samples, n)) < outlier_fraction
    x = np.where(mask, x * np.float32(outlier_scale), x).astype(np.float32)
    if dtype == "f32":
        return x
    return f32_to_f16_bits(x) if dtype == "f16" else f32_to_bf16_bits(x)


def gen_codebook(rng: np.random.Generator, entries: int, lo: float = 0.0, hi: float = 1.0) -> np.ndarray:
    """[entries][2] fp16 bit patterns drawn uniformly from [lo, hi): an initial codebook."""
    return f32_to_f16_bits(rng.uniform(lo, hi, size=(entries, 2)).astype(np.float32))


def gen_block_inputs(rng: np.random.Generator, M: int, d: int, dtype: str):
    """Inputs of the element-wise operators of an RWKV block (App. A.1) for a chunk of M tokens:
    receptance, key, value [M][d] as 16-bit patterns (keys with a wider spread and a few large
    entries, since they sit in an exponent), decay w [d] > 0 spread over e^-5 .. e^1 as in a trained
    RWKV-4 (log-uniform), bonus u [d] ~ N(0, 0.5)."""
    narrow = f32_to_f16_bits if dtype == "f16" else f32_to_bf16_bits
    r = rng.standard_normal(size=(M, d), dtype=np.float32) * 2.0
    k = rng.standard_normal(size=(M, d), dtype=np.float32) * 3.0
    k[rng.random(size=(M, d)) < 0.01] *= 8.0
    v = rng.standard_normal(size=(M, d), dtype=np.float32)
    w = np.exp(rng.uniform(-5.0, 1.0, size=d)).astype(np.float32)
    u = (rng.standard_normal(size=d) * 0.5).astype(np.float32)
    return narrow(r), narrow(k), narrow(v), w, u
