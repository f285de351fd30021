"""Pins for the oracle's own number-format conversions against numpy / torch / exact rationals."""
from fractions import Fraction

import numpy as np
import torch

import exact
from oracle import rwkvq_oracle as orc


def test_half_to_float_exhaustive():
    L = orc.lib()
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([L.rwkvq_oracle_half_to_float(int(b)) for b in bits], dtype=np.float32)
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite].view(np.uint32), ref[finite].view(np.uint32))
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(got[np.isinf(ref)], ref[np.isinf(ref)])


def _interesting_floats(rng, n):
    u = rng.integers(0, 1 << 32, size=n, dtype=np.uint32)
    f = u.view(np.float32)
    f = f[np.isfinite(f)]
    # concentrate on the fp16 range, its subnormals, ties and the overflow edge
    extra = np.concatenate([
        rng.standard_normal(n).astype(np.float32),
        (rng.standard_normal(n) * 1e-5).astype(np.float32),
        (rng.standard_normal(n) * 6e-8).astype(np.float32),
        (rng.standard_normal(n) * 3e4).astype(np.float32),
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 65536.0, 2.0 ** -24, 2.0 ** -25,
                  2.0 ** -25 * 1.0000001, 2.0 ** -26, 2.0 ** -14, 2.0 ** -14 * (1 - 2.0 ** -11),
                  1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -20],
                 dtype=np.float32)])
    return np.concatenate([f, extra, -extra])


def test_float_to_half_matches_numpy():
    L = orc.lib()
    f = _interesting_floats(np.random.default_rng(1), 20000)
    ref = f.astype(np.float16).view(np.uint16)
    got = np.array([L.rwkvq_oracle_float_to_half(float(v)) for v in f], dtype=np.uint16)
    assert np.array_equal(got, ref)


def test_float_to_bf16_matches_torch_and_rationals():
    L = orc.lib()
    f = _interesting_floats(np.random.default_rng(2), 20000)
    ref = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([L.rwkvq_oracle_float_to_bf16(float(v)) for v in f], dtype=np.uint16)
    assert np.array_equal(got, ref)
    for v in f[:300]:
        if v != 0 and abs(v) > 1e-30 and abs(v) < 1e30:
            assert int(L.rwkvq_oracle_float_to_bf16(float(v))) == exact.bf16_bits(Fraction(float(v)))


def test_round_weights_is_value_preserving_for_representable():
    w = np.array([0.5, -1.75, 3.0, 0.0078125], dtype=np.float32)
    assert np.array_equal(orc.round_weights(w, "bf16"), w)
    assert np.array_equal(orc.round_weights(w, "f16"), w)
    # 1 + 2^-8 is a tie in bf16 (8 significand bits, ulp 2^-7 at 1.0): goes to the even neighbour 1.0
    assert orc.round_weights(np.array([1.0 + 2.0 ** -8], np.float32), "bf16")[0] == np.float32(1.0)
    assert orc.round_weights(np.array([1.0 + 3 * 2.0 ** -8], np.float32), "bf16")[0] == np.float32(1.0 + 2.0 ** -6)


def test_widen_bf16_exhaustive_against_torch_and_rationals():
    """rwkvq_oracle.widen(bits, "bf16") for every one of the 65536 patterns: equal to torch's
    bfloat16 -> float32 (bit for bit on the finite ones), and on a sample equal to the value the
    format defines, (-1)^s 2^(e-127) (1 + m/128) or the subnormal m 2^-133, as an exact rational."""
    bits = np.arange(65536, dtype=np.uint16)
    got = orc.widen(bits, "bf16")
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite].view(np.uint32), ref[finite].view(np.uint32))
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(got[np.isinf(ref)], ref[np.isinf(ref)])
    for b in list(range(0, 65536, 257)) + [0x0001, 0x007F, 0x0080, 0x3F80, 0x3F81, 0x7F7F, 0x8000, 0xBF80, 0xFF7F, 0x477F, 0x4780]:
        s, e, m = b >> 15, (b >> 7) & 0xFF, b & 0x7F
        if e == 0xFF:
            continue
        v = Fraction(m, 128) * Fraction(2) ** -126 if e == 0 else (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)
        assert Fraction(float(got[b])) == (-v if s else v), hex(b)
    # and it round-trips through the oracle's own narrowing
    L = orc.lib()
    for b in (0x3F80, 0x3F81, 0x0001, 0x477F, 0xC2F7):
        assert int(L.rwkvq_oracle_float_to_bf16(float(got[b]))) == b


def test_widen_f16_matches_the_c_routine_and_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    got = orc.widen(bits, "f16")
    ref = bits.view(np.float16).astype(np.float32)
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite].view(np.uint32), ref[finite].view(np.uint32))
