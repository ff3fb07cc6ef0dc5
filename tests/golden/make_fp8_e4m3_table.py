"""Writes fp8_e4m3_values.txt: the value of each of the 256 code points of the 8-bit floating-point format
E4M3 (the "OCP 8-bit Floating Point Specification (OFP8)", Sec. 5: 1 sign bit, 4 exponent bits with bias 7,
3 mantissa bits; exponent field 0 holds the subnormals m/8 * 2^-6; there are no infinities; S.1111.111 is
NaN, so the largest finite value is 1.75 * 2^8 = 448).  Exact rational arithmetic, no floating point and no
code of the repository: the table is the yardstick for the oracle's decoder.

Usage: python tests/golden/make_fp8_e4m3_table.py   (rewrites the file next to it)
"""
import os
from fractions import Fraction


def value(code):
    s, e, m = code >> 7, (code >> 3) & 15, code & 7
    if e == 15 and m == 7:
        return None
    mag = Fraction(m, 8) * Fraction(1, 64) if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)
    return -mag if s else mag


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "fp8_e4m3_values.txt")
    with open(out, "w") as f:
        f.write("# code (hex)  value as an exact fraction  (E4M3 of the OCP OFP8 specification, Sec. 5; written by\n"
                "# make_fp8_e4m3_table.py with rational arithmetic)\n")
        for c in range(256):
            v = value(c)
            f.write(f"{c:02x} {'nan' if v is None else f'{v.numerator}/{v.denominator}'}\n")


if __name__ == "__main__":
    main()
