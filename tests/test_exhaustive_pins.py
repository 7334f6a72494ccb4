"""Exhaustive CPU pins (integer arithmetic, vectorised, a few seconds in all):

* the oracle's scale against the exact quotient for EVERY positive finite fp16 group maximum and all four divisors;
* every nibble position and a second byte position of the packed layout, written out by hand from the layout's text;
* the reciprocal-and-snap arithmetic the quantise kernels use per element (r = fp32(1/S), y = fp32(w r + C),
  code = rint(y) - C) against exact round-half-even of w / S for EVERY pair of normalised 11-bit significands, both
  signs, both bit widths and every exponent offset that reaches the code range.
"""
import numpy as np
import pytest

from oracle import rtn_oracle as O


@pytest.mark.parametrize("bits,rule", [(4, "qmax"), (8, "qmax"), (4, "eq2"), (8, "eq2")])
def test_scale_is_the_single_rounding_of_the_exact_quotient_for_every_fp16_amax(bits, rule):
    """fp16 values are integer multiples of 2^-24; with D = Dn / Dd the distance of amax / D from a grid point G is
    |G Dn - A Dd| / Dn in those units, so nearest-even can be checked in int64 for all 31 743 values at once."""
    Dn, Dd = {(4, "qmax"): (7, 1), (8, "qmax"): (127, 1), (4, "eq2"): (15, 2), (8, "eq2"): (255, 2)}[(bits, rule)]
    assert O.scale_divisor(bits, rule) * Dd == Dn
    halves = np.arange(1, 0x7C00, dtype=np.uint16).view(np.float16)
    got = O.rtn_scale(halves, bits, rule).view(np.uint16).astype(np.int64)
    assert got.size == 31743
    grid = (np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64) * 2.0 ** 24).astype(np.int64)
    A = (halves.astype(np.float64) * 2.0 ** 24).astype(np.int64)
    assert np.array_equal(grid[1:], A)                       # the conversion to integer units is exact
    d = np.abs(grid[got] * Dn - A * Dd)
    up = np.abs(grid[np.minimum(got + 1, grid.size - 1)] * Dn - A * Dd)
    dn = np.abs(grid[np.maximum(got - 1, 0)] * Dn - A * Dd)
    has_up, has_dn = got + 1 < grid.size, got > 0
    assert np.all(~has_up | (d <= up)) and np.all(~has_dn | (d <= dn))          # a nearest grid point ...
    assert np.all(~(has_up & (d == up)) | (got % 2 == 0))                       # ... and the even one on a tie
    assert np.all(~(has_dn & (d == dn)) | (got % 2 == 0))


def test_pack_layout_every_nibble_and_byte_position_by_hand():
    # 4-bit: row 0, columns 0..7 of the first tile are the eight elements e = 0..7 of word 0 of chunk 0 (kq = 0).
    # Store the values 1..8 (codes -7..0).  The layout text puts element e into nibble {0,4,1,5,2,6,3,7}[e]:
    #   nibble 0 <- e0 (1), nibble 1 <- e2 (3), nibble 2 <- e4 (5), nibble 3 <- e6 (7),
    #   nibble 4 <- e1 (2), nibble 5 <- e3 (4), nibble 6 <- e5 (6), nibble 7 <- e7 (8)
    # little-endian word 0x86427531: bytes 0x31, 0x75, 0x42, 0x86.
    c = np.full((16, 128), -8, dtype=np.int8)
    c[0, 0:8] = np.arange(1, 9) - 8
    img = O.pack_gfx950(c, 4)
    assert img[0:4].tolist() == [0x31, 0x75, 0x42, 0x86] and int(img.sum()) == 0x31 + 0x75 + 0x42 + 0x86
    # the same eight elements in another word, quarter and row: row 9, columns 32*2 + 8*3 + e = 88..95
    # -> chunk 3*16 + 9 = 57, word 2 -> bytes 57*16 + 8 .. + 11
    c[:] = -8
    c[9, 88:96] = np.arange(1, 9) - 8
    img = O.pack_gfx950(c, 4)
    assert img[57 * 16 + 8: 57 * 16 + 12].tolist() == [0x31, 0x75, 0x42, 0x86] and int(img.sum()) == 0x31 + 0x75 + 0x42 + 0x86
    # 8-bit: chunk byte 8 t + e holds column 32 t + 8 kq + e as q + 128.  Row 5, column 12: t = 0, kq = 1, e = 4
    # -> chunk 16 + 5 = 21, byte 4.  Row 15, column 63: t = 1, kq = 3, e = 7 -> chunk 63, byte 15 (the last byte).
    c8 = np.full((16, 64), -128, dtype=np.int8)
    c8[5, 12] = -27          # stored 101
    c8[15, 63] = 127         # stored 255
    img = O.pack_gfx950(c8, 8)
    assert img[21 * 16 + 4] == 101 and img[1023] == 255 and int(img.sum()) == 101 + 255
    # all eight elements of one 8-bit word pair in order: row 0, columns 0..7 -> chunk 0, bytes 0..7
    c8[:] = -128
    c8[0, 0:8] = np.arange(1, 9) - 128
    img = O.pack_gfx950(c8, 8)
    assert img[0:8].tolist() == [1, 2, 3, 4, 5, 6, 7, 8]


@pytest.mark.parametrize("bits", [4, 8])
def test_reciprocal_and_snap_equals_exact_rne_for_every_significand_pair(bits):
    """w = mw 2^ew and S = ms 2^es with normalised 11-bit significands mw, ms in [1024, 2048): the code depends on
    (mw, ms, ew - es, sign) only (scaling both by a power of two changes neither w / S nor, below overflow and above
    the subnormals, any rounding in r = fp32(1 / S) and y = fp32(w r + C)).  All 1024 x 1024 pairs, every exponent
    offset d with |w / S| < 2^(b-1) + 2, both signs."""
    off = 8 if bits == 4 else 128
    C = 768.0 + off
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    ms = np.arange(1024, 2048, dtype=np.int64)[None, :]
    mw = np.arange(1024, 2048, dtype=np.int64)[:, None]
    s = (ms.astype(np.float64) * 2.0 ** -10).astype(np.float32)           # S in [1, 2): exact in fp32
    r = (np.float32(1.0) / s).astype(np.float32)                          # IEEE fp32 division
    checked = 0
    for d in range(-3, bits + 1):                                         # w / S in [2^(d-1), 2^(d+1))
        if 2.0 ** (d - 1) > hi + 2:
            continue
        w = mw.astype(np.float64) * 2.0 ** (d - 10)
        # exact round-half-even of w / S = mw 2^d / ms in integers (shift so that everything is integral)
        sh = max(0, -d)
        num, den = mw << (d + sh), ms << sh
        q, rem = num // den, num % den
        up = (2 * rem > den) | ((2 * rem == den) & (q % 2 == 1))
        exact = q + up
        for sign in (1.0, -1.0):
            # w r is exact in fp64 (11 x 24 bits), adding C keeps it exact (< 53 bits): one rounding to fp32 = the fma
            y = (sign * w * r.astype(np.float64) + C).astype(np.float32)
            code = np.clip(np.rint(y.astype(np.float64)) - C, lo, hi)
            want = np.clip(sign * exact, lo, hi)
            bad = code != want
            assert not bad.any(), (bits, d, sign, int(bad.sum()))
            checked += code.size
    assert checked >= 2 * 1024 * 1024 * (bits + 2)
