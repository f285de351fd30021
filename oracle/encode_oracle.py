"""CPU oracle of the two encoders of Sec. 2.2: round-to-nearest scalar quantization (Eq. "SQ") and
nearest-codebook-entry vector quantization (Eq. "VQ").  They turn a dense weight matrix into the
codes / indices the linear-layer path reads, in the canonical layout (per-row little-endian bit
strings).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU baseline may import this;
the GPU library never does, and this module imports nothing from the GPU package.

Every floating-point step is a single binary32 operation rounded to nearest even, in the order
written here (numpy float32 arrays: one IEEE operation per ufunc, no fused multiply-add).

SQ, per row and per group of `group` consecutive input channels (Eq. "SQ", b bits):
    s  = (max - min) / (2^b - 1)          binary32 subtract and divide, then rounded to fp16 (stored)
    z  = (-min) / s                       with the stored s, binary32 divide, rounded to fp16 (stored)
    q  = clamp( rne( w / s + z ), 0, 2^b - 1 )    with the stored s and z: divide, add, round
The dequantized value is (q - z) s, the inverse the run-time path evaluates.
Readings (the paper is silent or ambiguous; also listed in the design notes):
  * the scale is printed as (max - min)/2^b - 1; read as /(2^b - 1);
  * the zero point is real-valued (no rounding is shown) and the equation adds it outside the
    rounding, which would make the code a non-integer; it is added inside, so that q is the index of
    the nearest point of the grid {(q - z) s} that the dequantization spans;
  * rounding to nearest resolves ties to even;
  * s and z are stored as fp16 and the codes are chosen against the stored values;
  * a constant group (max = min), or one whose range is below the resolution of an fp16 scale,
    takes s = 1, z = -min (the codes then round w - min, i.e. are 0);
  * inputs are finite and a group's scale and zero point must fit fp16.

VQ (Eq. "VQ", d = 2): the vector (w[n][2j], w[n][2j+1]) is replaced by
    argmin_e  fl( fl((v0 - c_e0)^2) + fl((v1 - c_e1)^2) )
over the 2^k entries c_e of the codebook of the 256 x 256 block that holds it; the squared
Euclidean distance has the same minimiser as the norm of the equation; equal distances resolve to
the lowest index (paper silent).
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def pack_fields(vals: np.ndarray, width: int) -> np.ndarray:
    """[N][F] integers -> [N][F*width/32] uint32, field i of a row at bits [width*i, width*i+width)
    of the row's little-endian bit string."""
    N, F = vals.shape
    assert (F * width) % 32 == 0
    bits = ((vals[:, :, None].astype(np.uint32) >> np.arange(width, dtype=np.uint32)) & 1).astype(np.uint8)
    bits = bits.reshape(N, F * width)
    words = bits.reshape(N, -1, 32).astype(np.uint32)
    return (words << np.arange(32, dtype=np.uint32)).sum(axis=2, dtype=np.uint64).astype(np.uint32)


def sq_encode(W: np.ndarray, bits: int = 3, group: int = 128):
    """W: [N][K] float32 (already widened exactly from its storage type).
    Returns (q [N][K] uint8, scales [N][K/group] fp16 bit patterns, zeros likewise)."""
    W = np.asarray(W, dtype=F32)
    N, K = W.shape
    assert K % group == 0
    G = K // group
    Wg = W.reshape(N, G, group)
    lo = Wg.min(axis=2)
    hi = Wg.max(axis=2)
    levels = F32(2 ** bits - 1)
    with np.errstate(divide="ignore", invalid="ignore"):
        s32 = ((hi - lo) / levels).astype(F32)
    # constant group, or a range so small that the fp16 scale would be zero
    const = (hi == lo) | (s32.astype(np.float16) == 0)
    s32 = np.where(const, F32(1.0), s32).astype(F32)
    s16 = s32.astype(np.float16)
    s = s16.astype(F32)
    with np.errstate(divide="ignore", invalid="ignore"):
        z32 = (-lo) / s
    z16 = z32.astype(np.float16)
    z = z16.astype(F32)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = Wg / s[:, :, None]
    t = (t + z[:, :, None]).astype(F32)
    q = np.clip(np.rint(t), 0, 2 ** bits - 1).astype(np.uint8)
    return q.reshape(N, K), s16.view(np.uint16), z16.view(np.uint16)


def sq_encode_packed(W: np.ndarray, bits: int = 3, group: int = 128):
    q, s, z = sq_encode(W, bits, group)
    return pack_fields(q, bits), s, z


def vq_assign(W: np.ndarray, codebooks: np.ndarray, kbits: int, block: int = 256) -> np.ndarray:
    """W: [N][K] float32; codebooks: [N/block][K/block][2^kbits][2] fp16 bit patterns.
    Returns idx [N][K/2] (uint16)."""
    W = np.asarray(W, dtype=F32)
    N, K = W.shape
    cb = np.asarray(codebooks, dtype=np.uint16).view(np.float16).astype(F32).reshape(N // block, K // block, 2 ** kbits, 2)
    idx = np.empty((N, K // 2), np.uint16)
    for bi in range(N // block):
        for bj in range(K // block):
            v = W[bi * block:(bi + 1) * block, bj * block:(bj + 1) * block].reshape(block, block // 2, 2)
            c = cb[bi, bj]
            d0 = (v[:, :, None, 0] - c[None, None, :, 0]).astype(F32)
            d1 = (v[:, :, None, 1] - c[None, None, :, 1]).astype(F32)
            dist = ((d0 * d0).astype(F32) + (d1 * d1).astype(F32)).astype(F32)
            idx[bi * block:(bi + 1) * block, bj * (block // 2):(bj + 1) * (block // 2)] = dist.argmin(axis=2)
    return idx


def vq_assign_packed(W: np.ndarray, codebooks: np.ndarray, kbits: int, block: int = 256) -> np.ndarray:
    return pack_fields(vq_assign(W, codebooks, kbits, block), kbits)
