"""Pins for the oracle's bit-string reader (canonical layout; code range of Sec. 2.2 Eq. "SQ",
k-bit indices of Eq. "VQ")."""
import os

import numpy as np
import pytest

from oracle import rwkvq_oracle as orc


def _golden(golden_dir):
    out = {}
    for line in open(os.path.join(golden_dir, "bitstrings.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, *words = line.split()
        out[name] = np.array([int(w, 16) for w in words], dtype=np.uint32)[None, :]
    return out


def bigint_pack(values, width):
    """Independent packer: one Python integer as the bit string, cut into 32-bit words."""
    s = 0
    for i, v in enumerate(values):
        s |= int(v) << (width * i)
    nwords = (len(values) * width + 31) // 32
    return np.array([(s >> (32 * w)) & 0xFFFFFFFF for w in range(nwords)], dtype=np.uint32)


def test_hand_packed_sq_codes(golden_dir):
    g = _golden(golden_dir)
    got = orc.unpack(g["sq3_kmod8"], 3, 32)
    assert got.tolist() == [[k % 8 for k in range(32)]]


def test_hand_packed_vq_indices(golden_dir):
    g = _golden(golden_dir)
    got = orc.unpack(g["vq6_iota16"], 6, 16)
    assert got.tolist() == [list(range(16))]


def test_straddling_fields(golden_dir):
    g = _golden(golden_dir)
    sq = orc.unpack(g["sq3_code10_is5"], 3, 32)[0]
    assert sq[10] == 5 and sq.sum() == 5
    vq = orc.unpack(g["vq6_index5_is45"], 6, 16)[0]
    assert vq[5] == 45 and vq.sum() == 45


def test_golden_words_match_bigint_packer(golden_dir):
    g = _golden(golden_dir)
    assert bigint_pack([k % 8 for k in range(32)], 3).tolist() == g["sq3_kmod8"][0].tolist()
    assert bigint_pack(list(range(16)), 6).tolist() == g["vq6_iota16"][0].tolist()


@pytest.mark.parametrize("width,count", [(3, 128), (6, 128), (8, 64), (3, 1024), (6, 512)])
def test_roundtrip_random(width, count):
    rng = np.random.default_rng(width * 1000 + count)
    vals = rng.integers(0, 1 << width, size=(5, count))
    words = np.stack([bigint_pack(v, width) for v in vals])
    assert np.array_equal(orc.unpack(words, width, count), vals.astype(np.uint16))


def test_single_field_isolated():
    # exactly one field set to all ones, everything else zero: each field, including the
    # straddling ones, must come back alone.
    for width, count in ((3, 32), (6, 16)):
        for i in range(count):
            vals = [0] * count
            vals[i] = (1 << width) - 1
            got = orc.unpack(bigint_pack(vals, width)[None, :], width, count)[0]
            assert got.tolist() == vals


def test_eight_bit_fields_are_bytes():
    rng = np.random.default_rng(8)
    words = rng.integers(0, 1 << 32, size=(3, 16), dtype=np.uint32)
    got = orc.unpack(words, 8, 64)
    assert np.array_equal(got, words.view(np.uint8).reshape(3, 64).astype(np.uint16))


def test_rows_are_independent_bit_strings():
    # row r starts at its own word 0: a second row must not continue the first row's bit phase
    rng = np.random.default_rng(3)
    vals = rng.integers(0, 8, size=(4, 32))
    words = np.stack([bigint_pack(v, 3) for v in vals])
    assert words.shape == (4, 3)
    assert np.array_equal(orc.unpack(words, 3, 32), vals.astype(np.uint16))
