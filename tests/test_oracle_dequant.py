"""Pins for the oracle's SQ and VQ dequantization (Sec. 2.2, Eqs. "SQ" and "VQ")."""
import os
from fractions import Fraction

import numpy as np
import pytest

import exact
from oracle import rwkvq_oracle as orc
from test_oracle_bits import bigint_pack


def f16b(v):
    return np.asarray(v, dtype=np.float32).astype(np.float16).view(np.uint16)


def pack_rows(vals, width):
    return np.stack([bigint_pack(r, width) for r in vals])


# ---------------------------------------------------------------- SQ

def test_sq_unit_scale_zero_offset_returns_codes():
    rng = np.random.default_rng(0)
    q = rng.integers(0, 8, size=(4, 256))
    w = orc.sq_dequant(pack_rows(q, 3), f16b(np.ones((4, 2))), f16b(np.zeros((4, 2))), 256)
    assert np.array_equal(w, q.astype(np.float32))


def test_sq_closed_form_half_steps():
    # s = 0.5, z = 3.5: codes 0..7 -> -1.75, -1.25, ..., 1.75 (all exact)
    q = np.tile(np.arange(8), 16)[None, :]
    w = orc.sq_dequant(pack_rows(q, 3), f16b([[0.5]]), f16b([[3.5]]), 128)
    expect = np.tile(np.array([-1.75, -1.25, -0.75, -0.25, 0.25, 0.75, 1.25, 1.75], np.float32), 16)
    assert np.array_equal(w[0], expect)


def test_sq_inverts_the_forward_quantizer_on_grid_points():
    # Eq. "SQ": Q(x) = clamp(round(x/s) + z, 0, 7).  For x on the grid s*(q - z) with an integer
    # z the forward map returns q, so Deq(Q(x)) = x: check the oracle reproduces such x exactly.
    s, z = 0.25, 3.0
    q = np.tile(np.arange(8), 16)[None, :]
    x = s * (q - z)
    assert np.array_equal(np.clip(np.rint(x / s) + z, 0, 7), q)
    w = orc.sq_dequant(pack_rows(q, 3), f16b([[s]]), f16b([[z]]), 128)
    assert np.array_equal(w, x.astype(np.float32))


def test_sq_power_of_two_scaling_is_exact():
    rng = np.random.default_rng(1)
    q = rng.integers(0, 8, size=(8, 256))
    s = rng.uniform(0.005, 0.02, size=(8, 2)).astype(np.float16)
    z = f16b(rng.uniform(0, 7, size=(8, 2)))
    w1 = orc.sq_dequant(pack_rows(q, 3), s.view(np.uint16), z, 256)
    w2 = orc.sq_dequant(pack_rows(q, 3), (s * np.float16(2)).view(np.uint16), z, 256)
    assert np.array_equal(w2, w1 * np.float32(2))


def test_sq_groups_run_along_input_channels():
    # all codes 1, z = 0, a different scale per (row, group): w[n, k] = s[n, k // 128]
    N, K = 3, 512
    q = np.ones((N, K), dtype=np.int64)
    s = (np.arange(N * 4).reshape(N, 4) + 1).astype(np.float32) / 64
    w = orc.sq_dequant(pack_rows(q, 3), f16b(s), f16b(np.zeros((N, 4))), K)
    assert np.array_equal(w, np.repeat(s, 128, axis=1))
    # and the zero point likewise: codes 0, s = 1 -> w = -z[n, k // 128]
    z = (np.arange(N * 4).reshape(N, 4)).astype(np.float32) / 4
    w = orc.sq_dequant(pack_rows(np.zeros((N, K), np.int64), 3), f16b(np.ones((N, 4))), f16b(z), K)
    assert np.array_equal(w, -np.repeat(z, 128, axis=1))


def test_sq_rounding_order_cases(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "sq_rounding_cases.txt"))
            if not l.startswith("#")]
    assert len(rows) == 10 and sum(r[0] == "order" for r in rows) == 6
    for tag, q, zb, sb, a, b, c, d in rows:
        q, zb, sb = int(q), int(zb, 16), int(sb, 16)
        codes = np.zeros((1, 128), np.int64)
        codes[0, 77] = q
        w = orc.sq_dequant(pack_rows(codes, 3), np.array([[sb]], np.uint16),
                           np.array([[zb]], np.uint16), 128)
        assert int(w.view(np.uint32)[0, 77]) == int(a, 16)
        if tag == "order":
            assert int(a, 16) != int(d, 16)


def test_sq_random_against_exact_rationals():
    rng = np.random.default_rng(5)
    q = rng.integers(0, 8, size=(2, 128))
    s = f16b(rng.uniform(0.005, 0.02, size=(2, 1)))
    z = f16b(rng.uniform(0, 7, size=(2, 1)))
    w = orc.sq_dequant(pack_rows(q, 3), s, z, 128).view(np.uint32)
    for n in range(2):
        sv, zv = exact.f16_value(int(s[n, 0])), exact.f16_value(int(z[n, 0]))
        for k in range(128):
            want = exact.f32_bits(exact.f32_round(Fraction(int(q[n, k])) - zv) * sv)
            assert int(w[n, k]) == want


def test_sq_random_against_wide_arithmetic():
    # q - z rounded to binary32, times s: both steps done in binary64 (where they are exact
    # before the rounding) and narrowed once each - a different route to the same two roundings.
    from paper_2505_03803_amd import synth
    m = synth.gen_sq(np.random.default_rng(7), 64, 1024)
    q = orc.unpack(m.codes, 3, 1024).astype(np.float64)
    s = np.repeat(m.scales.view(np.float16).astype(np.float64), 128, axis=1)
    z = np.repeat(m.zeros.view(np.float16).astype(np.float64), 128, axis=1)
    want = ((q - z).astype(np.float32).astype(np.float64) * s).astype(np.float32)
    got = orc.sq_dequant(m.codes, m.scales, m.zeros, 1024)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


# ---------------------------------------------------------------- VQ

def _vq_case(seed, N=512, K=512, kbits=6):
    rng = np.random.default_rng(seed)
    idx = rng.integers(0, 1 << kbits, size=(N, K // 2))
    cb = rng.standard_normal((N // 256, K // 256, 1 << kbits, 2)).astype(np.float16)
    return idx, cb


@pytest.mark.parametrize("kbits", [6, 8])
def test_vq_reproduces_indexed_codebook_entry_exactly(kbits):
    idx, cb = _vq_case(kbits, kbits=kbits)
    w = orc.vq_dequant(pack_rows(idx, kbits), cb.view(np.uint16), 512, kbits)
    n = np.arange(512)[:, None]
    j = np.arange(256)[None, :]
    want = cb[n // 256, (2 * j) // 256, idx]              # [N, K/2, 2]
    assert np.array_equal(w.reshape(512, 256, 2).view(np.uint32),
                          want.astype(np.float32).view(np.uint32))


def test_vq_vector_is_two_consecutive_input_channels():
    # Sec. 2.2: W (m, n) -> (m*n/d, d) row-major: vector j of row n covers columns 2j, 2j+1.
    cb = np.zeros((1, 1, 64, 2), np.float16)
    cb[0, 0, :, 0] = np.arange(64)           # first element = index
    cb[0, 0, :, 1] = -np.arange(64)          # second element = -index
    idx = (np.arange(256 * 128).reshape(256, 128) * 7) % 64
    w = orc.vq_dequant(pack_rows(idx, 6), cb.view(np.uint16), 256, 6)
    assert np.array_equal(w[:, 0::2], idx.astype(np.float32))
    assert np.array_equal(w[:, 1::2], -idx.astype(np.float32))


def test_vq_block_mapping_at_block_edges():
    # every 256 x 256 block has a constant codebook equal to (block_row*10 + block_col):
    # rows/cols 255 and 256 must fall in different blocks.
    N, K = 768, 1024
    cb = np.zeros((3, 4, 64, 2), np.float16)
    for br in range(3):
        for bc in range(4):
            cb[br, bc] = br * 10 + bc
    idx = np.random.default_rng(0).integers(0, 64, size=(N, K // 2))
    w = orc.vq_dequant(pack_rows(idx, 6), cb.view(np.uint16), K, 6)
    n = np.arange(N)[:, None]
    k = np.arange(K)[None, :]
    assert np.array_equal(w, ((n // 256) * 10 + k // 256).astype(np.float32))
    assert w[255, 255] == 0 and w[256, 255] == 10 and w[255, 256] == 1 and w[256, 256] == 11


def test_vq_generalises_sq():
    # a 64-entry codebook listing the 8 x 8 grid (s(q0-z), s(q1-z)), index q0 + 8 q1, with s, z
    # chosen so entries are exact in fp16, must dequantize to the same bits as SQ with codes q.
    rng = np.random.default_rng(11)
    N = K = 256
    q = rng.integers(0, 8, size=(N, K))
    s, z = 0.0625, 2.5
    grid = np.array([[s * (q0 - z), s * (q1 - z)] for q1 in range(8) for q0 in range(8)], np.float16)
    assert np.array_equal(grid.astype(np.float64)[:, 0], [s * (i % 8 - z) for i in range(64)])
    idx = q[:, 0::2] + 8 * q[:, 1::2]
    w_vq = orc.vq_dequant(pack_rows(idx, 6), grid.reshape(1, 1, 64, 2).view(np.uint16), K, 6)
    w_sq = orc.sq_dequant(pack_rows(q, 3), f16b(np.full((N, 2), s)), f16b(np.full((N, 2), z)), K)
    assert np.array_equal(w_vq.view(np.uint32), w_sq.view(np.uint32))
    # and for 3-bit fields the two bit strings are the same words
    assert np.array_equal(pack_rows(idx, 6), pack_rows(q, 3))


def test_vq_values_come_from_the_codebook_only():
    from paper_2505_03803_amd import synth
    m = synth.gen_vq(np.random.default_rng(3), 256, 512, 8)
    w = orc.vq_dequant(m.codes, m.codebooks, 512, 8)
    for bc in range(2):
        vals = set(m.codebooks[0, bc].view(np.float16).astype(np.float32).ravel().tolist())
        assert set(w[:, bc * 256:(bc + 1) * 256].ravel().tolist()) <= vals
