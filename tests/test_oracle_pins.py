"""Pins of the CPU oracle against things other than itself.

Sources of truth used here: worked examples derived with exact rationals
(tests/golden/rtn_worked_examples.txt; Eq. 1 and Eq. 2 of Section 2.2), an exact-rational
re-statement of round-half-to-even division, invariants and closed forms that follow from
Eq. 1-2, special cases that reduce to integer matrix products, a pure-Python triple loop,
hand-computed byte positions of the packed layout, and the average-precision figures the
paper states in Sections 1 and 4.3.
"""
import os
from fractions import Fraction as F

import numpy as np
import pytest

from oracle import rtn_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "rtn_worked_examples.txt")


def _frac(h) -> F:
    return F(float(np.float16(h)))


def _rne(x: F) -> int:
    fl = x.numerator // x.denominator
    r = x - fl
    if r != F(1, 2):
        return fl + (1 if r > F(1, 2) else 0)
    return fl if fl % 2 == 0 else fl + 1


def _golden_cases():
    out = []
    with open(GOLDEN) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, *kv = line.split()
            d = dict(item.split("=", 1) for item in kv)
            out.append((name, int(d["bits"]), d["divisor"], d["w"].split(","),
                        int(d["scale_bits"], 16), [int(v) for v in d["q"].split(",")]))
    return out


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c[0])
def test_worked_examples(case):
    name, bits, divisor, w, scale_bits, q = case
    rule = "qmax" if "/" not in divisor else "eq2"
    W = np.array([[float(v) for v in w]], dtype=np.float16)
    codes, scales = O.rtn_quantize(W, bits, W.shape[1], rule)
    assert int(scales.view(np.uint16)[0, 0]) == scale_bits
    assert codes[0].tolist() == q


def test_eq2_identity():
    # Eq. 2: 2 max / (2^b - 1) == max / (2^(b-1) - 0.5)
    for b in (4, 8):
        assert F(2) / F(2 ** b - 1) == F(1) / (F(2 ** (b - 1)) - F(1, 2))
        assert O.scale_divisor(b, "eq2") == 2 ** (b - 1) - 0.5
        assert O.scale_divisor(b, "qmax") == 2 ** (b - 1) - 1
    assert O.qrange(4) == (-8, 7) and O.qrange(8) == (-128, 127)   # Section 2.2


@pytest.mark.parametrize("bits,rule", [(4, "qmax"), (8, "qmax"), (4, "eq2"), (8, "eq2")])
def test_scale_is_single_rounding_of_exact_quotient_all_fp16(bits, rule):
    """Stored scale == RNE_fp16(exact amax / D) with exact rationals, on all 2048 smallest fp16 values and every 7th
    above them (the exhaustive check of all 31 743 values, in integer arithmetic, is in tests/test_exhaustive_pins.py)."""
    D = F(O.scale_divisor(bits, rule))
    halves = np.arange(1, 0x7C00, dtype=np.uint16).view(np.float16)
    got = O.rtn_scale(halves, bits, rule).view(np.uint16)
    grid = [F(float(h)) for h in np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16)]
    # exact check: the chosen grid point must be a nearest one, and on a tie the even one
    step = 7  # every 7th value (co-prime with the periods of 1/7, 1/127) plus all the small ones
    idx = list(range(0, 2048)) + list(range(2048, len(halves), step))
    for i in idx:
        x = F(float(halves[i])) / D
        j = int(got[i])
        d = abs(grid[j] - x)
        if j + 1 < len(grid):
            assert d <= abs(grid[j + 1] - x)
            if d == abs(grid[j + 1] - x):
                assert j % 2 == 0
        if j > 0:
            assert d <= abs(grid[j - 1] - x)
            if d == abs(grid[j - 1] - x):
                assert j % 2 == 0


@pytest.mark.parametrize("bits,rule", [(4, "qmax"), (8, "qmax"), (4, "eq2"), (8, "eq2")])
def test_codes_match_exact_rational_rounding(bits, rule):
    rng = np.random.default_rng(7 + bits)
    lo, hi = O.qrange(bits)
    g = 32
    W = (rng.standard_normal((6, 2 * g)) * 0.02).astype(np.float16)
    # plant exact ties: row 0 is multiples of half a step of a power-of-two scale
    qmax = hi
    W[0, :g] = ((np.arange(g) % 13) - 6) * 0.5 * 2.0 ** -6   # -3 .. 3 in steps of 0.5, in units of s
    W[0, 0] = qmax * 2.0 ** -6            # amax = qmax * s  ->  s = 2^-6 exactly (qmax rule)
    W[1, :g] = 0
    W[2, g:] = np.float16(6e-8)           # subnormal group
    codes, scales = O.rtn_quantize(W, bits, g, rule)
    for n in range(W.shape[0]):
        for j in range(2):
            s = _frac(scales[n, j])
            for k in range(g):
                w = _frac(W[n, j * g + k])
                want = 0 if s == 0 else max(lo, min(hi, _rne(w / s)))
                assert int(codes[n, j * g + k]) == want, (n, j, k)
    assert (codes[1, :g] == 0).all() and scales[1, 0] == 0
    # the planted ties really are ties and went to even
    if rule == "qmax":
        assert float(scales[0, 0]) == 2.0 ** -6
        assert codes[0, 7:12].tolist() == [0, 1, 2, 2, 2]      # 0.5 1.0 1.5 2.0 2.5 -> ties to even
        assert codes[0, 1:6].tolist() == [-2, -2, -2, -1, 0]     # -2.5 -2.0 -1.5 -1.0 -0.5


@pytest.mark.parametrize("bits", [4, 8])
def test_reconstruction_error_bound(bits):
    rng = np.random.default_rng(1)
    W = (rng.standard_normal((64, 512)) * 0.02).astype(np.float16)
    for g in (128, 512):
        codes, scales = O.rtn_quantize(W, bits, g, "qmax")
        deq = O.rtn_dequantize(codes, scales, g)
        s = np.repeat(scales.astype(np.float64), g, axis=1)
        assert np.all(np.abs(W.astype(np.float64) - deq) <= s / 2 + 1e-300)
        # Eq. 2 rule: the clamped +amax element may exceed s/2, by at most the scale's own rounding
        codes, scales = O.rtn_quantize(W, bits, g, "eq2")
        deq = O.rtn_dequantize(codes, scales, g)
        s = np.repeat(scales.astype(np.float64), g, axis=1)
        D = O.scale_divisor(bits, "eq2")
        assert np.all(np.abs(W.astype(np.float64) - deq) <= s * (0.5 + D * 2.0 ** -11))


@pytest.mark.parametrize("bits", [4, 8])
def test_on_grid_weights_round_trip_exactly(bits):
    rng = np.random.default_rng(2)
    lo, hi = O.qrange(bits)
    g = 128
    q = rng.integers(-hi, hi + 1, size=(32, 2 * g))
    q[:, 0] = hi
    q[:, g] = -hi                               # every group attains qmax
    e = rng.integers(-14, 4, size=(32, 2))      # power-of-two scales, fp16-normal, q*s in range
    s = 2.0 ** e
    W = (q.reshape(32, 2, g) * s[:, :, None]).reshape(32, 2 * g).astype(np.float16)
    codes, scales = O.rtn_quantize(W, bits, g, "qmax")
    assert np.array_equal(codes, q.astype(np.int8))
    assert np.array_equal(scales.astype(np.float64), s)
    assert np.array_equal(O.rtn_dequantize(codes, scales, g), W.astype(np.float64))


@pytest.mark.parametrize("bits", [4, 8])
def test_closed_forms(bits):
    rng = np.random.default_rng(3)
    lo, hi = O.qrange(bits)
    W = (rng.standard_normal((48, 256)) * 0.05).astype(np.float16)
    codes, scales = O.rtn_quantize(W, bits, 128, "qmax")
    normal = scales.astype(np.float64) >= 2.0 ** -14
    # the group maximum maps to +-qmax when the scale is a normal fp16
    assert np.all(np.abs(codes).reshape(48, 2, 128).max(axis=2)[normal] == hi)
    assert codes.min() >= -hi                    # -2^(b-1) is never produced under the qmax rule
    # odd symmetry
    c2, s2 = O.rtn_quantize(-W, bits, 128, "qmax")
    assert np.array_equal(c2, -codes) and np.array_equal(s2, scales)
    # scaling by a power of two moves only the scale
    c3, s3 = O.rtn_quantize((W.astype(np.float32) * 8).astype(np.float16), bits, 128, "qmax")
    assert np.array_equal(c3, codes) and np.array_equal(s3.astype(np.float64), scales.astype(np.float64) * 8)
    # per-channel equals group-wise when all groups of a row share one amax
    W2 = W.copy()
    W2[:, 0] = W2[:, 128] = np.float16(0.9)
    cg, sg = O.rtn_quantize(W2, bits, 128, "qmax")
    cc, sc = O.rtn_quantize(W2, bits, 256, "qmax")
    assert np.array_equal(cg, cc) and np.all(sg == sc)
    # Eq. 2 rule is asymmetric at +-amax by construction (clamp at +2^(b-1) only)
    We = np.array([[-1.5, 1.5, 0.3, 0.1]], dtype=np.float16)
    ce, _ = O.rtn_quantize(We, bits, 4, "eq2")
    assert ce[0, 0] == lo and ce[0, 1] == hi


def test_group_direction_is_along_K():
    # one large value in row 0, columns 0..127: only that row/group's scale may change
    W = np.full((4, 256), 0.01, dtype=np.float16)
    W[0, 5] = 1.0
    _, s = O.rtn_quantize(W, 4, 128, "qmax")
    assert s.shape == (4, 2)
    assert s[0, 0] > s[0, 1] and s[0, 1] == s[1, 0] == s[3, 1]


def test_linear_integer_special_case_and_shapes():
    rng = np.random.default_rng(4)
    M, N, K, g = 3, 16, 256, 128                 # N != K != M catches transposed operands
    q = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    A = rng.integers(-4, 5, size=(M, K)).astype(np.float16)
    ones = np.ones((N, K // g), dtype=np.float16)
    C = O.rtn_linear(A, q, ones, g)
    assert C.shape == (M, N)
    assert np.array_equal(C, (A.astype(np.int64) @ q.astype(np.int64).T).astype(np.float64))
    # scales enter per (row, group): doubling one group's scale adds that group's partial sum once more
    s = ones.copy()
    s[5, 1] = 2
    C2 = O.rtn_linear(A, q, s, g)
    extra = A[:, g:].astype(np.int64) @ q[5, g:].astype(np.int64)
    assert np.array_equal(C2[:, 5] - C[:, 5], extra.astype(np.float64))
    assert np.array_equal(np.delete(C2, 5, axis=1), np.delete(C, 5, axis=1))


def test_linear_one_hot_and_bruteforce():
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((8, 8)) * 0.02).astype(np.float16)
    A = rng.standard_normal((8, 8)).astype(np.float16)
    for bits in (4, 8):
        for g in (4, 8):
            codes, scales = O.rtn_quantize(W, bits, g)
            C = O.rtn_linear(A, codes, scales, g)
            B = O.rtn_linear_bruteforce(A, codes, scales, g)
            assert np.max(np.abs(C - B)) <= 1e-12
            eye = np.eye(8, dtype=np.float16)
            C1 = O.rtn_linear(eye, codes, scales, g)
            assert np.array_equal(C1, O.rtn_dequantize(codes, scales, g).T)
    # row_block must not change the result
    codes, scales = O.rtn_quantize(W, 4, 8)
    assert np.array_equal(O.rtn_linear(A, codes, scales, 8, row_block=3), O.rtn_linear(A, codes, scales, 8))


def test_pack_layout_hand_positions():
    # 4-bit, one tile (16 x 128): a single 7 at (row 3, col 45), everything else -8 (stored 0).
    c = np.full((16, 128), -8, dtype=np.int8)
    c[3, 45] = 7
    img = O.pack_gfx950(c, 4)
    assert img.size == 1024
    # col 45 = 32*1 + 8*1 + 5 -> word t=1, quarter kq=1, element e=5 -> nibble 6 -> byte 3 low nibble
    # chunk = kq*16 + row = 19 ; byte = 19*16 + 4*1 + 3 = 311
    assert img[311] == 0x0F and img.sum() == 0x0F
    # element e=1 goes to nibble 4 (byte 2 low), e=2 to nibble 1 (byte 0 high)
    c[:] = -8
    c[0, 1] = -7       # stored 1
    c[0, 2] = -6       # stored 2
    img = O.pack_gfx950(c, 4)
    assert img[2] == 0x01 and img[0] == 0x20 and img.sum() == 0x21
    # second k-tile / second n-tile offsets: tiles are row-tile-major, 1024 bytes each
    c2 = np.full((32, 256), -8, dtype=np.int8)
    c2[16, 128] = -7   # n-tile 1, k-tile 1, chunk 0, word 0, nibble 0
    img = O.pack_gfx950(c2, 4)
    assert img[(1 * 2 + 1) * 1024] == 0x01 and img.sum() == 1
    # 8-bit, tile 16 x 64: (row 2, col 41): t=1, kq=1, e=1 -> chunk 18, byte 9, stored q+128
    c8 = np.full((16, 64), -128, dtype=np.int8)
    c8[2, 41] = 5
    img = O.pack_gfx950(c8, 8)
    assert img.size == 1024 and img[18 * 16 + 9] == 133 and img.sum() == 133


@pytest.mark.parametrize("bits", [4, 8])
def test_pack_unpack_round_trip(bits):
    rng = np.random.default_rng(6)
    lo, hi = O.qrange(bits)
    c = rng.integers(lo, hi + 1, size=(32, 256)).astype(np.int8)
    img = O.pack_gfx950(c, bits)
    assert img.size == 32 * 256 * bits // 8
    assert np.array_equal(O.unpack_gfx950(img, 32, 256, bits), c)


def test_selective_precision_accounting():
    # Section 4.3: a quarter / a half of the layers fully at 8 bit -> 5 / 6 bits on average
    p8b = [4096 * 6144, 4096 * 4096, 4096 * 28672, 14336 * 4096]
    assert O.effective_bits(32, p8b, "first", 8) == 5.0
    assert O.effective_bits(32, p8b, "first", 16) == 6.0
    assert O.effective_bits(32, p8b, "middle", 8) == 5.0 and O.effective_bits(32, p8b, "last", 8) == 5.0
    # ... and lower than that once module 2 stays at 4 bit (modules 1+3+4)
    assert 4.0 < O.effective_bits(32, p8b, "first", 8, (1, 3, 4)) < 5.0
    # one whole layer at 8 bit: 4 + 4/n  (4.125 for 32 layers, 4.05 for 80)
    p70 = [8192 * 10240, 8192 * 8192, 8192 * 57344, 28672 * 8192]
    assert O.effective_bits(32, p8b, "first", 1) == 4.125
    assert abs(O.effective_bits(80, p70, "first", 1) - 4.05) < 1e-12
    # Sections 1 and 6: the 70B variant with modules 1+3+4 of the first layer at 8 bit
    # costs "less than 0.05" extra bits per weight
    extra = O.effective_bits(80, p70, "first", 1, (1, 3, 4)) - 4.0
    assert 0.0 < extra < 0.05
    assert abs(extra - 4 * F(96256, 104448) / 80) < 1e-12
    # selection geometry
    assert O.selected_layers(10, "first", 3) == [0, 1, 2]
    assert O.selected_layers(10, "last", 3) == [7, 8, 9]
    assert O.selected_layers(10, "middle", 4) == [3, 4, 5, 6]
    assert O.plan_bits(0, 80, 2, "first", 1, (1, 3, 4)) == 4
    assert O.plan_bits(0, 80, 4, "first", 1, (1, 3, 4)) == 8
    assert O.plan_bits(1, 80, 4, "first", 1, (1, 3, 4)) == 4


# --------------------------------------------------------------------------------------
# Asymmetric variant (Section 2.2's remark; reading R8 in the oracle's header)
# --------------------------------------------------------------------------------------
GOLDEN_ASYM = os.path.join(os.path.dirname(__file__), "golden", "rtn_asym_worked_examples.txt")


def _golden_asym_cases():
    out = []
    with open(GOLDEN_ASYM) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, *kv = line.split()
            d = dict(item.split("=", 1) for item in kv)
            out.append((name, int(d["bits"]), d["w"].split(","), int(d["scale_bits"], 16), int(d["zero"]),
                        [int(v) for v in d["q"].split(",")]))
    return out


@pytest.mark.parametrize("case", _golden_asym_cases(), ids=lambda c: c[0])
def test_asym_worked_examples(case):
    """Examples derived with exact rationals by tests/golden/derive_worked_examples.py (imports neither side)."""
    name, bits, w, scale_bits, zero, q = case
    W = np.array([[float(v) for v in w]], dtype=np.float16)
    codes, scales, zeros = O.rtn_quantize_asym(W, bits, W.shape[1])
    assert int(scales.view(np.uint16)[0, 0]) == scale_bits
    assert int(zeros[0, 0]) == zero
    assert codes[0].tolist() == q

def _round_binary(x: F, precision: int, min_quantum_exp: int) -> F:
    """Round-half-even of a non-negative rational to a binary format with `precision` significand bits and smallest
    quantum 2^min_quantum_exp (IEEE rounding restated with exact rationals; no overflow handling)."""
    if x == 0:
        return F(0)
    e = x.numerator.bit_length() - x.denominator.bit_length()          # floor(log2 x) or one more
    if F(2) ** e > x:
        e -= 1
    qe = max(e - precision + 1, min_quantum_exp)
    quantum = F(2) ** qe
    return _rne(x / quantum) * quantum


@pytest.mark.parametrize("bits", [4, 8])
def test_asym_matches_exact_rationals(bits):
    rng = np.random.default_rng(100 + bits)
    lo, hi = O.qrange(bits)
    levels = (1 << bits) - 1
    g = 32
    W = (rng.standard_normal((8, 2 * g)) * 0.02).astype(np.float16)
    W[0, :g] += np.float16(0.05)                       # mostly positive group
    W[1, :g] = np.abs(W[1, :g])                        # all non-negative: alpha = 0
    W[2, :g] = -np.abs(W[2, :g])                       # all non-positive: beta = 0
    W[3, :g] = 0                                       # all zero
    W[4, :g] = np.float16(3e-7) * (np.arange(g) % 5 - 1)     # subnormal scale
    W[5, :g] = np.float16(0.37)                        # constant group (range is [0, 0.37])
    # planted ties with an odd shift: range [-3, 12] in units of s = 2^-5, halves in between
    W[6, :g] = (np.arange(g) % 31 * 0.5 - 3.0) * 2.0 ** -5
    W[6, 0], W[6, 1] = -3.0 * 2.0 ** -5, 12.0 * 2.0 ** -5
    W[7, :g] = np.float16(1.0) + np.float16(2.0 ** -10) * np.arange(g)     # far from zero, narrow spread
    W[7, g] = np.float16(-2.0 ** -20) * np.float16(1.0 + 2.0 ** -10)     # beta - alpha does not fit fp32
    W[7, g + 1] = np.float16(1.0)
    # a (beta, alpha) pair on which an fp32 intermediate (difference and quotient rounded to 24 bits first) would give
    # a different fp16 scale than the single rounding of the exact quotient: a lower-precision shortcut fails here
    hb, ha = {4: (16008, 33279), 8: (17014, 33217)}[bits]
    W[5, g:] = 0
    W[5, g] = np.array([hb], dtype=np.uint16).view(np.float16)[0]
    W[5, g + 1] = np.array([ha], dtype=np.uint16).view(np.float16)[0]
    codes, scales, zeros = O.rtn_quantize_asym(W, bits, g)
    exact = (F(float(W[5, g])) - F(float(W[5, g + 1]))) / levels
    via_fp32 = _round_binary(_round_binary(_round_binary(F(float(W[5, g])) - F(float(W[5, g + 1])), 24, -149) / levels, 24, -149), 11, -24)
    assert via_fp32 != _round_binary(exact, 11, -24)                  # the planted pair does tell the two apart
    for n in range(W.shape[0]):
        for j in range(2):
            grp = [_frac(v) for v in W[n, j * g:(j + 1) * g]]
            alpha, beta = min(min(grp), F(0)), max(max(grp), F(0))
            s = _round_binary((beta - alpha) / levels, 11, -24)        # the exact quotient, rounded once
            assert _frac(scales[n, j]) == s, (n, j)
            t = 0 if s == 0 else max(-levels, min(0, _rne(alpha / s)))
            assert int(zeros[n, j]) == t - lo, (n, j)
            for k in range(g):
                r = 0 if s == 0 else _rne(grp[k] / s)
                assert int(codes[n, j * g + k]) == max(lo, min(hi, r - (t - lo))), (n, j, k)
    # the planted ties are ties, the shift is odd, and they went to even BEFORE the shift
    if bits == 4:
        assert float(scales[6, 0]) == 2.0 ** -5 and int(zeros[6, 0]) == -3 + 8
        # k = 7, 9, 11: w / s = 0.5, 1.5, 2.5 -> 0, 2, 2 -> minus Z = 5
        assert [int(codes[6, k]) for k in (7, 9, 11)] == [0 - 5, 2 - 5, 2 - 5]
    assert scales[3, 0] == 0 and int(zeros[3, 0]) == -lo and (codes[3, :g] == lo).all()
    assert float(scales[7, 1]) > 0          # the inexact-difference group went through


@pytest.mark.parametrize("bits", [4, 8])
def test_asym_nearest_level_zero_and_grid(bits):
    rng = np.random.default_rng(5)
    lo, hi = O.qrange(bits)
    g = 64
    W = (rng.standard_normal((32, 4 * g)) * 0.02 + 0.01).astype(np.float16)
    W[:, ::7] = 0
    codes, scales, zeros = O.rtn_quantize_asym(W, bits, g)
    deq = O.rtn_dequantize_asym(codes, scales, zeros, g)
    W64 = W.astype(np.float64)
    s = np.repeat(scales.astype(np.float64), g, axis=1)
    z = np.repeat(zeros.astype(np.float64), g, axis=1)
    assert np.all(deq[W == 0] == 0.0)                                   # zero is a level of every group
    # every code is a nearest level among all 2^b levels of its group (brute force over the levels)
    best = np.full(W.shape, np.inf)
    for q in range(lo, hi + 1):
        best = np.minimum(best, np.abs(W64 - s * (q + z)))
    assert np.all(np.abs(W64 - deq) <= best * (1 + 1e-12) + 1e-300)
    # inside the covered range the error is at most half a step; the range ends can lose at most the scale's rounding
    inside = (codes > lo) & (codes < hi)
    assert np.all(np.abs(W64 - deq)[inside] <= s[inside] / 2)
    assert np.all(np.abs(W64 - deq) <= s * (0.5 + ((1 << bits) - 1) * 2.0 ** -11))
    # a group already on a shifted grid is reproduced exactly, with the shift as its zero point
    c = 2.0 ** -7
    Wg = (c * (np.arange(1 << bits) - 3)).astype(np.float16)[None, :].repeat(2, axis=0)
    codes, scales, zeros = O.rtn_quantize_asym(Wg, bits, 1 << bits)
    assert float(scales[0, 0]) == c and int(zeros[0, 0]) == -3 - lo
    assert codes[0].tolist() == list(range(lo, hi + 1))
    assert np.array_equal(O.rtn_dequantize_asym(codes, scales, zeros, 1 << bits), Wg.astype(np.float64))
    # asymmetric resolution on a one-sided group is twice the symmetric one
    Wp = np.abs(W[:4])
    _, s_sym = O.rtn_quantize(Wp, bits, g)
    _, s_asym, _ = O.rtn_quantize_asym(Wp, bits, g)
    ratio = s_sym.astype(np.float64) / s_asym.astype(np.float64)
    assert np.all(np.abs(ratio - ((1 << bits) - 1) / hi) < 0.01)


def test_asym_linear_identity_and_bruteforce():
    rng = np.random.default_rng(11)
    N, K, M, g = 16, 128, 3, 32
    W = (rng.standard_normal((N, K)) * 0.02 + 0.015).astype(np.float16)
    A = rng.standard_normal((M, K)).astype(np.float16)
    codes, scales, zeros = O.rtn_quantize_asym(W, 4, g)
    C = O.rtn_linear_asym(A, codes, scales, zeros, g)
    # sum_k A S (q + Z) = [symmetric-form linear on the same codes] + sum_groups Z S (sum of A over the group)
    Asum = A.astype(np.float64).reshape(M, K // g, g).sum(axis=2)                     # [M, G]
    corr = Asum @ (zeros.astype(np.float64) * scales.astype(np.float64)).T           # [M, N]
    assert np.allclose(C, O.rtn_linear(A, codes, scales, g) + corr, rtol=1e-12, atol=1e-12)
    # pure-Python loops
    for m in range(M):
        for n in range(0, N, 5):
            acc = 0.0
            for k in range(K):
                acc += float(A[m, k]) * float(scales[n, k // g]) * (int(codes[n, k]) + int(zeros[n, k // g]))
            assert abs(acc - C[m, n]) < 1e-9
    # closeness to the unquantised product: asymmetric beats symmetric on shifted weights
    exact = A.astype(np.float64) @ W.astype(np.float64).T
    cs, ss = O.rtn_quantize(W, 4, g)
    err_a = np.linalg.norm(C - exact)
    err_s = np.linalg.norm(O.rtn_linear(A, cs, ss, g) - exact)
    assert err_a < err_s
