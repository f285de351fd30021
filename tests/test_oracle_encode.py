"""Pins of the encoder oracle (oracle/encode_oracle.py): round trips through the independently
pinned decoder oracle, the error bound of round-to-nearest, end points, exhaustive search on tiny
inputs, tie handling and the bit packing."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import encode_oracle as E
from oracle import rwkvq_oracle as orc
from paper_2505_03803_amd import synth


def f16(x):
    return np.asarray(x, np.float16).astype(np.float32)


def test_pack_fields_matches_the_decoder_bit_layout():
    rng = np.random.default_rng(0)
    for width, F in ((3, 256), (6, 128), (8, 64)):
        vals = rng.integers(0, 2 ** width, size=(5, F), dtype=np.uint32)
        words = E.pack_fields(vals, width)
        assert np.array_equal(orc.unpack(words, width, F), vals)     # the decoder's own field reader
    # field 10 of a 3-bit string straddles words 0 and 1 (bits 30-32)
    vals = np.zeros((1, 32), np.uint32); vals[0, 10] = 0b101
    assert E.pack_fields(vals, 3)[0].tolist() == [0x40000000, 0x00000001, 0]


def test_sq_grid_exact_weights_round_trip():
    # weights that lie exactly on a grid {(q - z) s} with s, z exact in fp16 come back bit for bit
    rng = np.random.default_rng(1)
    N, K = 8, 512
    q = rng.integers(0, 8, size=(N, K)).astype(np.float32)
    q[:, ::128] = 0; q[:, 1::128] = 7                   # every group spans the whole range
    s = np.float32(0.015625)                              # 2^-6
    for zval in (0.0, 3.0, 3.5, 7.0):
        W = ((q - np.float32(zval)) * s).astype(np.float32)
        q2, s16, z16 = E.sq_encode(W)
        assert np.array_equal(q2, q.astype(np.uint8))
        assert np.all(s16.view(np.float16) == np.float16(s)) and np.all(z16.view(np.float16) == np.float16(zval))
        mat = synth.QMatrix("t", "sq", N, K, 0, E.pack_fields(q2, 3), s16, z16, None)
        assert np.array_equal(orc.dequant(mat), W)


def test_sq_error_bound_end_points_and_monotonicity():
    rng = np.random.default_rng(2)
    N, K = 16, 1024
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    q, s16, z16 = E.sq_encode(W)
    mat = synth.QMatrix("t", "sq", N, K, 0, E.pack_fields(q, 3), s16, z16, None)
    What = orc.dequant(mat)                                # the decoder oracle, pinned separately
    s = np.repeat(s16.view(np.float16).astype(np.float64), 128, axis=1)
    # round to nearest: at most half a step, plus what fp16 storage of s and z moves the grid
    assert np.all(np.abs(W.astype(np.float64) - What) <= 0.5 * s * (1 + 2 ** -9) + 7 * s * 2 ** -11)
    Wg, qg = W.reshape(N, K // 128, 128), q.reshape(N, K // 128, 128)
    assert np.all(np.take_along_axis(qg, Wg.argmin(axis=2)[..., None], 2) == 0)     # min -> code 0
    assert np.all(np.take_along_axis(qg, Wg.argmax(axis=2)[..., None], 2) == 7)     # max -> code 7
    order = np.argsort(Wg, axis=2)
    assert np.all(np.diff(np.take_along_axis(qg.astype(int), order, 2), axis=2) >= 0)   # monotone


def test_sq_codes_are_the_nearest_grid_point_exact_arithmetic():
    # one group, exact rational arithmetic of the same formula on the stored s and z
    rng = np.random.default_rng(3)
    W = (rng.standard_normal((1, 128)) * 0.3).astype(np.float32)
    q, s16, z16 = E.sq_encode(W)
    s = Fraction(float(s16.view(np.float16)[0, 0])); z = Fraction(float(z16.view(np.float16)[0, 0]))
    for k in range(128):
        w = Fraction(float(W[0, k]))
        best = min(range(8), key=lambda c: abs((Fraction(c) - z) * s - w))
        dist_best = abs((Fraction(best) - z) * s - w)
        dist_got = abs((Fraction(int(q[0, k])) - z) * s - w)
        # the code taken is a nearest grid point up to the binary32 rounding of w/s + z
        assert dist_got <= dist_best + s * Fraction(1, 2 ** 20)


def test_sq_constant_group_and_scale_definition():
    W = np.full((2, 128), 0.375, np.float32)
    q, s16, z16 = E.sq_encode(W)
    assert not q.any() and np.all(s16.view(np.float16) == 1.0) and np.all(z16.view(np.float16) == -0.375)
    mat = synth.QMatrix("t", "sq", 2, 128, 0, E.pack_fields(q, 3), s16, z16, None)
    assert np.array_equal(orc.dequant(mat), W)
    # (max - min) / (2^b - 1): a group spanning [-1, 2.5] has s = 0.5, z = 2
    W = np.linspace(-1.0, 2.5, 128, dtype=np.float32)[None, :]
    _, s16, z16 = E.sq_encode(W)
    assert s16.view(np.float16)[0, 0] == 0.5 and z16.view(np.float16)[0, 0] == 2.0


def subresolution_groups():
    """Groups whose range is positive but too small for an fp16 scale: (max - min)/7 rounds to the
    fp16 zero exactly when it is at most 2^-25 (the tie 2^-25 itself goes to the even neighbour 0).
    Hand values, every number a power of two or a small multiple:
      row 0: 2^-8 and 2^-8 + 2^-30 alternating        -> s = 1, z = -2^-8, all codes 0
      row 1: 0 and 7 * 2^-25 alternating (the tie)      -> s = 1, z = 0, all codes 0
      row 2: 0 and 7 * 2^-25 * (1 + 2^-20): just above  -> s = 2^-24 (smallest fp16 subnormal), z = 0,
             codes 0 and rne(3.5 (1 + 2^-20)) = 4
      row 3: -3 * 2^-30 and 0                            -> s = 1, z = 3 * 2^-30 -> fp16 0, all codes 0"""
    W = np.zeros((4, 128), np.float32)
    W[0] = 2.0 ** -8; W[0, 1::2] = 2.0 ** -8 + 2.0 ** -30
    W[1, 1::2] = 7 * 2.0 ** -25
    W[2, 1::2] = np.float32(7 * 2.0 ** -25) * np.float32(1 + 2.0 ** -20)
    W[3, 0::2] = -3 * 2.0 ** -30
    want_s = np.array([1.0, 1.0, 2.0 ** -24, 1.0], np.float16)
    want_z = np.array([-(2.0 ** -8), -0.0, -0.0, 0.0], np.float16)      # z = -min / s: a minimum of +0 gives -0
    want_q = np.zeros((4, 128), np.uint8); want_q[2, 1::2] = 4
    return W, want_s, want_z, want_q


def test_sq_range_below_the_resolution_of_an_fp16_scale():
    W, want_s, want_z, want_q = subresolution_groups()
    assert W[0, 1] != W[0, 0] and W[2, 1] > W[1, 1]          # the inputs really differ in binary32
    q, s16, z16 = E.sq_encode(W)
    assert np.array_equal(s16[:, 0], want_s.view(np.uint16))
    assert np.array_equal(z16[:, 0], want_z.view(np.uint16))
    assert np.array_equal(q, want_q)
    # what the decoder returns: the group's minimum for rows 0, 1, 3 (error at most the range), and
    # for row 2 the grid {0, 4 * 2^-24}: the error stays within half a step of the stored scale
    mat = synth.QMatrix("t", "sq", 4, 128, 0, E.pack_fields(q, 3), s16, z16, None)
    What = orc.dequant(mat).astype(np.float64)
    assert np.all(What[0] == 2.0 ** -8) and np.all(What[1] == 0.0) and np.all(What[3] == 0.0)
    assert np.all(np.abs(What - W) <= np.array([2.0 ** -30, 7 * 2.0 ** -25, 2.0 ** -25, 3 * 2.0 ** -30])[:, None] * (1 + 1e-6))


def brute_force_assign(v, cb):
    best, bestd = 0, None
    for e in range(cb.shape[0]):
        d = (Fraction(float(v[0])) - Fraction(float(cb[e, 0]))) ** 2 + (Fraction(float(v[1])) - Fraction(float(cb[e, 1]))) ** 2
        if bestd is None or d < bestd:
            best, bestd = e, d
    return best


@pytest.mark.parametrize("kbits", [6, 8])
def test_vq_assign_equals_exhaustive_search(kbits):
    rng = np.random.default_rng(4 + kbits)
    N = K = 256
    cb16 = (rng.standard_normal((1, 1, 2 ** kbits, 2)) * 0.02).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    idx = E.vq_assign(W, cb16.view(np.uint16), kbits)
    cb = cb16.astype(np.float32)[0, 0]
    for (n, j) in [(0, 0), (3, 17), (255, 127), (100, 64), (17, 5), (200, 90)]:
        assert idx[n, j] == brute_force_assign(W[n, 2 * j:2 * j + 2], cb)
    # every vector: no entry is closer (binary64 check of all 2^k distances)
    v = W.reshape(N, K // 2, 2).astype(np.float64)
    d = ((v[:, :, None, :] - cb.astype(np.float64)[None, None]) ** 2).sum(axis=3)
    chosen = np.take_along_axis(d, idx[..., None].astype(np.int64), 2)[..., 0]
    assert np.all(chosen <= d.min(axis=2) * (1 + 1e-6) + 1e-12)


def test_vq_codebook_vectors_round_trip_and_ties_go_to_the_lowest_index():
    rng = np.random.default_rng(9)
    cb16 = (rng.standard_normal((1, 2, 64, 2)) * 0.02).astype(np.float16)
    cb16[0, 1, 40] = cb16[0, 1, 7]                       # duplicate entry in the second block
    pick = rng.integers(0, 64, size=(256, 256))          # [n][pair] over both column blocks
    W = np.empty((256, 512), np.float32)
    for bj in range(2):
        c = cb16[0, bj].astype(np.float32)
        W[:, 256 * bj:256 * bj + 256] = c[pick[:, 128 * bj:128 * bj + 128]].reshape(256, 256)
    idx = E.vq_assign(W, cb16.view(np.uint16), 6)
    want = pick.copy()
    want[:, 128:][want[:, 128:] == 40] = 7               # the duplicate resolves to the lower index
    # other accidental duplicates of random fp16 entries would also resolve downwards
    assert np.all(idx <= want)
    mat = synth.QMatrix("t", "vq", 256, 512, 6, E.pack_fields(idx, 6), None, None, cb16.view(np.uint16))
    assert np.array_equal(orc.dequant(mat), W)           # decoded through the decoder oracle
    assert np.all(idx[:, 128:][pick[:, 128:] == 40] == 7)
