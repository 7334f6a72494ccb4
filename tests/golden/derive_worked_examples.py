"""Derives the worked examples in rtn_worked_examples.txt with exact rational arithmetic.

Independent of both the CPU oracle and the HIP library: it imports neither.  Every value
can be re-derived by hand from Eq. 1 and Eq. 2 of Section 2.2 (RTN): round the decimal
inputs to fp16, take max|w|, divide by D, round once to fp16 (the stored scale), divide
every weight by the stored scale, round half to even, clamp to [-2^(b-1), 2^(b-1)-1].

Run:  python tests/golden/derive_worked_examples.py  > tests/golden/rtn_worked_examples.txt
      python tests/golden/derive_worked_examples.py asym  > tests/golden/rtn_asym_worked_examples.txt

The second form derives examples of the asymmetric variant (the remark after Eq. 1: an integer zero point is subtracted
from the result of Int()) under this library's reading: range [alpha, beta] = [min(min w, 0), max(max w, 0)];
S = fp16((beta - alpha) / (2^b - 1)), the exact quotient rounded once; Z = clamp(rne(alpha / S), -(2^b - 1), 0) + 2^(b-1);
q = clamp(rne(w / S) - Z); all-zero scale: Z = 2^(b-1), q = -2^(b-1).
"""
from fractions import Fraction as F
import struct


def half_bits_to_fraction(h: int) -> F:
    s, e, m = h >> 15, (h >> 10) & 0x1F, h & 0x3FF
    v = F(m, 1 << 24) if e == 0 else F((1 << 10) | m, 1 << 10) * (F(2) ** (e - 15))
    return -v if s else v


_POS_HALVES = [(half_bits_to_fraction(h), h) for h in range(0x0000, 0x7C00)]


def round_to_half_bits(x: F) -> int:
    """Round-to-nearest-even of a rational onto the finite fp16 grid (binary search)."""
    sign = 0x8000 if x < 0 else 0
    x = abs(x)
    lo, hi = 0, len(_POS_HALVES) - 1
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if _POS_HALVES[mid][0] <= x:
            lo = mid
        else:
            hi = mid
    a, b = _POS_HALVES[lo], _POS_HALVES[hi]
    if x - a[0] < b[0] - x:
        return sign | a[1]
    if x - a[0] > b[0] - x:
        return sign | b[1]
    return sign | (a[1] if a[1] % 2 == 0 else b[1])


def decimal_to_half_bits(text: str) -> int:
    return round_to_half_bits(F(text))


def rne_int(x: F) -> int:
    fl = x.numerator // x.denominator
    r = x - fl
    if r > F(1, 2):
        return fl + 1
    if r < F(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def example(name, decimals, bits, divisor: F):
    wb = [decimal_to_half_bits(d) for d in decimals]
    w = [half_bits_to_fraction(h) for h in wb]
    amax = max(abs(v) for v in w)
    sb = round_to_half_bits(amax / divisor)
    s = half_bits_to_fraction(sb)
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    q = [0 if s == 0 else max(lo, min(hi, rne_int(v / s))) for v in w]
    print(f"{name} bits={bits} divisor={divisor} w={','.join(decimals)} "
          f"scale_bits=0x{sb:04X} q={','.join(str(v) for v in q)}")


def example_asym(name, decimals, bits):
    wb = [decimal_to_half_bits(d) for d in decimals]
    w = [half_bits_to_fraction(h) for h in wb]
    levels = (1 << bits) - 1
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    alpha, beta = min(min(w), F(0)), max(max(w), F(0))
    sb = round_to_half_bits((beta - alpha) / levels)
    s = half_bits_to_fraction(sb)
    t = 0 if s == 0 else max(-levels, min(0, rne_int(alpha / s)))
    z = t - lo
    q = [max(lo, min(hi, (0 if s == 0 else rne_int(v / s)) - z)) for v in w]
    print(f"{name} bits={bits} w={','.join(decimals)} scale_bits=0x{sb:04X} zero={z} q={','.join(str(v) for v in q)}")


def main_asym():
    print("# Worked examples of the asymmetric variant (Section 2.2, the remark after Eq. 1), derived by")
    print("# derive_worked_examples.py asym with exact rationals; weight = S * (q + zero).")
    base = ["0.7", "-0.35", "0.05", "0.1", "-0.25", "0.45", "0", "-0.7"]
    example_asym("plain4", base, 4)
    example_asym("plain8", base, 8)
    example_asym("positive4", ["0.1", "0.2", "0.35", "0.8", "0.05", "0.6", "0.75", "0.4"], 4)
    example_asym("negative8", ["-0.1", "-0.2", "-0.35", "-0.8", "-0.05", "-0.6", "-0.75", "-0.4"], 8)
    example_asym("grid4", [repr((k - 3) / 128) for k in range(16)], 4)      # multiples of 2^-7: exact decimals
    example_asym("ties_odd_zero4", ["-3", "12", "0.5", "1.5", "2.5", "-0.5", "-1.5", "-2.5"], 4)
    example_asym("shifted8", ["1.0", "1.001", "1.01", "1.05", "0.99", "1.1", "0.95", "1.02"], 8)
    example_asym("zeros4", ["0", "-0", "0", "0"], 4)
    example_asym("tiny4", ["0.00000005960464477539", "0.00000011920928955078", "-0.00000023841857910156", "0"], 4)
    example_asym("wide_range8", ["60000", "-60000", "1", "-1", "30000.5", "0.25", "-12345", "7"], 8)
    # ranges whose width needs more than 24 bits: a difference or quotient first rounded to fp32 gives another scale
    example_asym("single_rounding4", ["1.6328125", "-0.000030457973480224609375", "0.5", "0"], 4)
    example_asym("single_rounding8", ["3.23046875", "-0.000026762485504150390625", "1.25", "0"], 8)


if __name__ == "__main__":
    import sys
    if len(sys.argv) > 1 and sys.argv[1] == "asym":
        main_asym()
        sys.exit(0)
    print("# Worked examples of Eq. 1 / Eq. 2 (Section 2.2), derived by derive_worked_examples.py")
    print("# with exact rationals.  divisor 7 / 127 = 2^(b-1)-1 (graded rule); 15/2 / 255/2 = Eq. 2.")
    base = ["0.7", "-0.35", "0.05", "0.1", "-0.25", "0.45", "0", "-0.7"]
    example("plain4", base, 4, F(7))
    example("plain4_eq2", base, 4, F(15, 2))
    example("plain8", base, 8, F(127))
    example("plain8_eq2", base, 8, F(255, 2))
    example("ties4", ["7", "0.5", "1.5", "2.5", "-0.5", "-1.5", "-2.5", "3.5"], 4, F(7))
    example("clamp4_eq2", ["-1.5", "1.5", "0.3", "0.1"], 4, F(15, 2))
    example("ties8", ["127", "0.5", "1.5", "-2.5", "63.5", "-64.5", "126.5", "-127"], 8, F(127))
    example("zeros4", ["0", "-0", "0", "0"], 4, F(7))
    example("tiny4", ["0.00000005960464477539", "0.00000011920928955078", "-0.00000023841857910156", "0"], 4, F(7))
