"""Writes tests/golden/sq_rounding_cases.txt: (q, z, s) triples, found by exact rational search,
for which different evaluation orders of the SQ inverse  w = (q - z) s  (Sec. 2.2, Eq. "SQ")
give different binary32 bit patterns.  Expected bits are computed here with Python integers
only (tests/exact.py); no oracle and no GPU code is involved.

Orders compared (fl = round to nearest even in binary32):
  A  fl(fl(q - z) * s)                subtract, then multiply   <- the reading taken
  B  fl(fl(q*s) - fl(z*s))            distribute, three roundings
  C  fl(q*s - fl(z*s))                fused multiply-add with a rounded z*s
  D  fl((q - z) * s)                  a single rounding of the exact value
Run:  python tests/golden/make_sq_rounding_case.py
"""
import os
import random
import sys
from fractions import Fraction

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from exact import f16_bits, f16_value, f32_bits, f32_round  # noqa: E402


def orders(q, zb, sb):
    z, s, qf = f16_value(zb), f16_value(sb), Fraction(q)
    a = f32_bits(f32_round(qf - z) * s)
    b = f32_bits(f32_round(qf * s) - f32_round(z * s))
    c = f32_bits(qf * s - f32_round(z * s))
    d = f32_bits((qf - z) * s)
    return a, b, c, d


def main():
    rnd = random.Random(20250503)
    rows = []
    # (1) ordinary magnitudes: z in (0, 7), s in (0.005, 0.02).  q*s and z*s have at most 22
    # significant bits and q - z at most 24, so every order is the single correctly rounded value.
    for _ in range(4):
        q = rnd.randrange(8)
        zb = f16_bits(Fraction(rnd.uniform(0.0, 7.0)))
        sb = f16_bits(Fraction(rnd.uniform(0.005, 0.02)))
        a, b, c, d = orders(q, zb, sb)
        assert a == b == c == d
        rows.append(("same", q, zb, sb, a, b, c, d))
    # (2) tiny zero point: q - z is not exact in binary32, so A (two roundings) can differ from
    # D (one rounding); these rows decide the evaluation order.
    for _ in range(200000):
        if len([r for r in rows if r[0] == "order"]) >= 6:
            break
        q = rnd.randrange(1, 8)
        zb = rnd.randrange(1, 0x0800)            # fp16 zero point below 2^-13
        sb = f16_bits(Fraction(rnd.uniform(0.005, 0.02)))
        a, b, c, d = orders(q, zb, sb)
        if a != d:
            rows.append(("order", q, zb, sb, a, b, c, d))
    assert len(rows) == 10
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "sq_rounding_cases.txt")
    with open(out, "w") as f:
        f.write("# SQ inverse w = (q - z) s, Sec. 2.2 Eq. \"SQ\": binary32 bit patterns under four\n"
                "# evaluation orders (see make_sq_rounding_case.py, which wrote this file with exact\n"
                "# rational arithmetic).  Column A is the reading the oracle must reproduce.\n"
                "# tag q z_fp16_bits s_fp16_bits A B C D\n")
        for tag, q, zb, sb, a, b, c, d in rows:
            f.write(f"{tag} {q} 0x{zb:04X} 0x{sb:04X} 0x{a:08X} 0x{b:08X} 0x{c:08X} 0x{d:08X}\n")
    print(open(out).read())


if __name__ == "__main__":
    main()
