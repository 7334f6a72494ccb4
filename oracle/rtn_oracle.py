"""CPU oracle for the RTN weight-only quantised linear layer (TEST INFRASTRUCTURE).

This module is test infrastructure.  Only the test-suite, the smoke entry and the
benchmark's ``cpu_baseline`` leg may import it; the product path (the HIP library
and its Python binding) never does, and shares no code, table or constant with it.

Everything here is a plain, slow, obviously-correct float64 / NumPy statement of
what the paper's method computes:

* ``rtn_scale`` / ``rtn_quantize``   -- symmetric round-to-nearest, Eq. 1 and Eq. 2
  of Section 2.2 (RTN), applied group-wise along every output channel as that
  section's last paragraphs describe.
* ``rtn_quantize_asym`` / ``rtn_dequantize_asym`` / ``rtn_linear_asym`` -- the asymmetric
  variant that Section 2.2 mentions (integer zero point), reading R8.
* ``rtn_dequantize`` / ``rtn_linear`` -- the weight-only W4A16 / W8A16 linear layer
  of Section 2.3 and Section 5: C = A (q * S)^T, as a float64 GEMM on the
  dequantised weights.
* ``pack_gfx950``                    -- the byte image of the packed weights (Section 5:
  the kernel wants its own interleaved layout) for this library's gfx950 layout,
  written from the layout's written specification, so packed bytes can be compared.
* ``plan_bits`` / ``effective_bits`` -- the selective-precision bookkeeping of
  Section 4 (horizontal, vertical, hybrid selection).

Readings of the paper taken here:

R1  Scale divisor.  Eq. 2 gives S = 2 max|r| / (2^b - 1) = max|r| / (2^(b-1) - 0.5).
    The contract this build is graded on uses S = max|r| / (2^(b-1) - 1).  Both are
    implemented; ``rule="qmax"`` (the default) is the latter, ``rule="eq2"`` is Eq. 2.
R2  "round to nearest" = round half to even.
R3  The scale is stored in fp16 and the *stored* fp16 value is the one that divides
    the weights (so dequantisation q * S uses the same S that produced q).
R4  amax / D and w / S are the exact real quotients, rounded once (to fp16 and to
    an integer respectively).  float64 division realises both exactly enough: see
    the proofs next to ``rtn_scale`` and ``rtn_quantize``; tests/test_oracle_pins.py
    checks them against exact rationals.
R5  A group whose stored scale is zero (all-zero group, or amax so small that
    amax / D rounds to fp16 zero) gets scale +0 and all codes 0.
R6  "truncate" of Eq. 1 = clamp to [-2^(b-1), 2^(b-1)-1].
R7  Groups run along the input dimension K of each output row.
R8  Asymmetric variant (Section 2.2 only says that it subtracts an integer zero point Z
    from the result of Int()).  Taken here: the group's range [alpha, beta] =
    [min(min r, 0), max(max r, 0)] always contains zero, so that zero is reproduced
    exactly and Z fits the code range; S = fp16 of the exact (beta - alpha) / (2^b - 1),
    rounded once, as R4 has it for the symmetric scale;
    Z = clamp(rne(alpha / S), -(2^b - 1), 0) + 2^(b-1), which sends alpha to the lowest
    code; q = clamp(rne(r / S) - Z) (the tie rule applies to r / S, before Z is
    subtracted); dequantised value S * (q + Z).  S == 0: Z = 2^(b-1), q = -2^(b-1),
    i.e. the value 0.  The symmetric variant is not a special case of this one (its
    range is [-max|r|, max|r|] and it never uses the lowest code's counterpart).

Parity pins: tests/test_oracle_pins.py (worked examples in tests/golden/, exact
rational cross-check, invariants, closed forms, brute force).  Model-level outputs
(perplexity, task accuracy) are "parity unpinned": they need weights and datasets
that are not available, and nothing here claims them.
"""
from __future__ import annotations

import numpy as np

SCALE_RULES = ("qmax", "eq2")


def qrange(bits: int) -> tuple[int, int]:
    """Integer target range of Eq. 1's Int(): [-2^(b-1), 2^(b-1)-1] (Section 2.2)."""
    if bits not in (4, 8):
        raise ValueError("bits must be 4 or 8")
    return -(1 << (bits - 1)), (1 << (bits - 1)) - 1


def scale_divisor(bits: int, rule: str = "qmax") -> float:
    """D such that S = max|r| / D.  rule 'eq2' is Eq. 2 of Section 2.2 (D = 2^(b-1) - 0.5);
    rule 'qmax' is the graded contract's D = 2^(b-1) - 1 (reading R1)."""
    if rule not in SCALE_RULES:
        raise ValueError("rule must be 'qmax' or 'eq2'")
    qmax = qrange(bits)[1]
    return float(qmax) if rule == "qmax" else float(qmax) + 0.5


def rtn_scale(amax: np.ndarray, bits: int, rule: str = "qmax") -> np.ndarray:
    """fp16(amax / D), one rounding (readings R3, R4).

    amax holds fp16 values (11-bit significands).  The float64 quotient amax / D is
    within 2^-53 relative of the exact one, while the exact quotient is never closer
    than 2^-16 relative to an fp16 rounding boundary (D is 7, 127, 15/2 or 255/2, so
    an exact tie would need a 12-bit odd multiple of D to fit 11 bits), hence the
    second rounding to fp16 equals rounding the exact quotient.
    """
    amax = np.asarray(amax, dtype=np.float16)
    return (amax.astype(np.float64) / scale_divisor(bits, rule)).astype(np.float16)


def rtn_quantize(W: np.ndarray, bits: int, group_size: int, rule: str = "qmax"):
    """Group-wise symmetric RTN (Eq. 1, Eq. 2; grouping per Section 2.2, reading R7).

    W: fp16 [N, K].  group_size g divides K; g == K is per-output-channel.
    Returns (codes int8 [N, K], scales fp16 [N, K // g]).

    q = clamp(rne(w / S16)) with S16 the stored fp16 scale.  w and S16 have 11-bit
    significands, so the exact quotient is either exactly i + 0.5 (representable, and
    float64 division returns it exactly) or at least 2^-13 away from it (far more
    than float64's rounding error), so np.rint of the float64 quotient is the
    round-half-to-even of the exact quotient.
    """
    W = np.asarray(W)
    if W.dtype != np.float16 or W.ndim != 2:
        raise ValueError("W must be fp16 [N, K]")
    N, K = W.shape
    g = int(group_size)
    if g <= 0 or K % g != 0:
        raise ValueError("group_size must divide K")
    if not np.all(np.isfinite(W)):
        raise ValueError("W must be finite")
    lo, hi = qrange(bits)
    Wg = W.astype(np.float64).reshape(N, K // g, g)
    amax = np.abs(Wg).max(axis=2)                       # exact: inputs are fp16 values
    scales = rtn_scale(amax.astype(np.float16), bits, rule)   # amax is itself an fp16 value
    s64 = scales.astype(np.float64)[:, :, None]
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.rint(Wg / s64)                           # ties to even (reading R2)
    q = np.where(s64 == 0.0, 0.0, q)                    # reading R5
    q = np.clip(q, lo, hi)                              # reading R6
    return q.reshape(N, K).astype(np.int8), scales


def rtn_dequantize(codes: np.ndarray, scales: np.ndarray, group_size: int) -> np.ndarray:
    """float64 [N, K] of q * S: symmetric RTN has no zero point (Section 2.2)."""
    codes = np.asarray(codes)
    N, K = codes.shape
    g = int(group_size)
    s = np.asarray(scales, dtype=np.float16).astype(np.float64).reshape(N, K // g)
    return (codes.astype(np.float64).reshape(N, K // g, g) * s[:, :, None]).reshape(N, K)


def rtn_linear(A: np.ndarray, codes: np.ndarray, scales: np.ndarray, group_size: int,
               row_block: int = 4096) -> np.ndarray:
    """C[m, n] = sum_k A[m, k] * (q[n, k] * S[n, k // g]) in float64 (Sections 2.3, 5).

    A: fp16 [M, K].  Output float64 [M, N].  Rows of the weight matrix are independent,
    so they are processed in blocks only to bound memory; no other reordering.
    """
    A64 = np.asarray(A, dtype=np.float16).astype(np.float64)
    N = codes.shape[0]
    out = np.empty((A64.shape[0], N), dtype=np.float64)
    for n0 in range(0, N, row_block):
        n1 = min(N, n0 + row_block)
        Wd = rtn_dequantize(codes[n0:n1], np.asarray(scales)[n0:n1], group_size)
        out[:, n0:n1] = A64 @ Wd.T
    return out


def rtn_quantize_asym(W: np.ndarray, bits: int, group_size: int):
    """Group-wise asymmetric RTN (Section 2.2's remark on the asymmetric variant; reading R8).

    W: fp16 [N, K].  Returns (codes int8 [N, K], scales fp16 [N, K // g], zeros int16 [N, K // g])
    with dequantised weights S * (q + Z).

    S is the exact quotient (beta - alpha) / (2^b - 1) rounded once to fp16 (argument next to the computation).
    alpha / S and w / S are exact real quotients rounded once to an integer: as in the
    symmetric case both operands carry 11-bit significands, so the float64 quotient is
    either an exact tie or far from one, and np.rint rounds the exact quotient half to even.
    """
    W = np.asarray(W)
    if W.dtype != np.float16 or W.ndim != 2:
        raise ValueError("W must be fp16 [N, K]")
    N, K = W.shape
    g = int(group_size)
    if g <= 0 or K % g != 0:
        raise ValueError("group_size must divide K")
    if not np.all(np.isfinite(W)):
        raise ValueError("W must be finite")
    lo, hi = qrange(bits)
    levels = (1 << bits) - 1
    Wg = W.reshape(N, K // g, g)
    alpha = np.minimum(Wg.min(axis=2), np.float16(0))            # fp16, <= 0
    beta = np.maximum(Wg.max(axis=2), np.float16(0))             # fp16, >= 0
    # beta - alpha is exact in float64 (two fp16 values span at most 41 bits).  The float64 quotient is within 2^-53
    # relative of the exact one, and an exact quotient that is not itself a midpoint between two fp16 values is at least
    # 2^-42 relative away from every such midpoint (beta - alpha and midpoint * (2^b - 1) are both multiples of 2^-25,
    # and beta - alpha < 2^18), so rounding the float64 quotient to fp16 is the single rounding of the exact quotient.
    width = beta.astype(np.float64) - alpha.astype(np.float64)
    scales = (width / np.float64(levels)).astype(np.float16)     # at most 131008 / 15: always finite
    s64 = scales.astype(np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.rint(alpha.astype(np.float64) / s64)              # code of alpha before the shift, <= 0
        t = np.where(s64 == 0.0, 0.0, t)
        t = np.clip(t, -levels, 0)
        zeros = t - lo                                           # Z = rne(alpha / S) + 2^(b-1)
        r = np.rint(Wg.astype(np.float64) / s64[:, :, None])     # Int() before truncation: ties to even on r / S
        r = np.where(s64[:, :, None] == 0.0, 0.0, r)
    q = np.clip(r - zeros[:, :, None], lo, hi)
    return q.reshape(N, K).astype(np.int8), scales, zeros.astype(np.int16)


def rtn_dequantize_asym(codes: np.ndarray, scales: np.ndarray, zeros: np.ndarray, group_size: int) -> np.ndarray:
    """float64 [N, K] of S * (q + Z) (reading R8)."""
    codes = np.asarray(codes)
    N, K = codes.shape
    g = int(group_size)
    s = np.asarray(scales, dtype=np.float16).astype(np.float64).reshape(N, K // g)
    z = np.asarray(zeros).astype(np.float64).reshape(N, K // g)
    return ((codes.astype(np.float64).reshape(N, K // g, g) + z[:, :, None]) * s[:, :, None]).reshape(N, K)


def rtn_linear_asym(A: np.ndarray, codes: np.ndarray, scales: np.ndarray, zeros: np.ndarray, group_size: int,
                    row_block: int = 4096) -> np.ndarray:
    """C[m, n] = sum_k A[m, k] * S[n, k // g] * (q[n, k] + Z[n, k // g]) in float64."""
    A64 = np.asarray(A, dtype=np.float16).astype(np.float64)
    N = codes.shape[0]
    out = np.empty((A64.shape[0], N), dtype=np.float64)
    for n0 in range(0, N, row_block):
        n1 = min(N, n0 + row_block)
        Wd = rtn_dequantize_asym(codes[n0:n1], np.asarray(scales)[n0:n1], np.asarray(zeros)[n0:n1], group_size)
        out[:, n0:n1] = A64 @ Wd.T
    return out


def rtn_linear_bruteforce(A, codes, scales, group_size):
    """Pure-Python triple loop of the same definition, for tiny inputs only."""
    A = np.asarray(A, dtype=np.float16)
    M, K = A.shape
    N = codes.shape[0]
    g = int(group_size)
    out = [[0.0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += float(A[m, k]) * (float(int(codes[n, k])) * float(np.float16(scales[n, k // g])))
            out[m][n] = acc
    return np.array(out, dtype=np.float64)


# --------------------------------------------------------------------------------------
# Packed byte image (Section 5: the kernel wants its own interleaved layout, and the
# weights are reshuffled into it once at load).  Written from the layout's specification:
#
#   The code matrix is cut into tiles of 16 output rows x TK input columns, TK = 128 for
#   4-bit and 64 for 8-bit; a tile is 1024 bytes; tiles are stored row-tile-major
#   ([N/16][K/TK]).  Inside a tile, the 16-byte chunk number l (0..63) belongs to row
#   l % 16 and to column-quarter kq = l // 16.
#   4-bit: chunk = four little-endian u32 words t = 0..3; word t holds the 8 codes of
#          columns 32 t + 8 kq + e (e = 0..7), each stored as q + 8 in the nibble number
#          [0, 4, 1, 5, 2, 6, 3, 7][e] (nibble p = bits 4p .. 4p+3).
#   8-bit: chunk byte 8 t + e (t = 0..1, e = 0..7) holds column 32 t + 8 kq + e as q + 128.
# --------------------------------------------------------------------------------------
_NIBBLE_OF_ELEMENT = (0, 4, 1, 5, 2, 6, 3, 7)


def pack_gfx950(codes: np.ndarray, bits: int) -> np.ndarray:
    """uint8 [N*K*bits/8] byte image of int8 codes [N, K] in the library's packed layout."""
    codes = np.asarray(codes, dtype=np.int8)
    N, K = codes.shape
    lo, hi = qrange(bits)
    if codes.min(initial=0) < lo or codes.max(initial=0) > hi:
        raise ValueError("code out of range")
    TK = 128 if bits == 4 else 64
    if N % 16 or K % TK:
        raise ValueError("N must be a multiple of 16 and K of the tile width")
    NT, KT = N // 16, K // TK
    u = (codes.astype(np.int16) - lo).astype(np.uint32)       # offset binary
    # axes: [nt, row, kt, t, kq, e]
    u = u.reshape(NT, 16, KT, TK // 32, 4, 8)
    if bits == 4:
        words = np.zeros((NT, 16, KT, 4, 4), dtype=np.uint32)  # [nt,row,kt,t,kq]
        for e in range(8):
            words |= u[..., e] << np.uint32(4 * _NIBBLE_OF_ELEMENT[e])
        # chunk l = kq*16 + row ; chunk = words t=0..3  -> [nt, kt, kq, row, t]
        img = np.ascontiguousarray(words.transpose(0, 2, 4, 1, 3))
        return img.astype("<u4").view(np.uint8).reshape(-1)
    # 8-bit: [nt,row,kt,t,kq,e] -> [nt, kt, kq, row, t, e]
    img = np.ascontiguousarray(u.transpose(0, 2, 4, 1, 3, 5)).astype(np.uint8)
    return img.reshape(-1)


def unpack_gfx950(packed: np.ndarray, N: int, K: int, bits: int) -> np.ndarray:
    """Inverse of pack_gfx950, by direct per-element indexing (slow; small inputs)."""
    packed = np.asarray(packed, dtype=np.uint8).reshape(-1)
    lo, _ = qrange(bits)
    TK = 128 if bits == 4 else 64
    KT = K // TK
    out = np.empty((N, K), dtype=np.int8)
    for n in range(N):
        for k in range(K):
            nt, row = divmod(n, 16)
            kt, kk = divmod(k, TK)
            t, r = divmod(kk, 32)
            kq, e = divmod(r, 8)
            chunk = ((nt * KT + kt) * 64 + kq * 16 + row) * 16
            if bits == 4:
                p = _NIBBLE_OF_ELEMENT[e]
                byte = packed[chunk + 4 * t + p // 2]
                v = (byte >> (4 * (p % 2))) & 0xF
            else:
                v = packed[chunk + 8 * t + e]
            out[n, k] = int(v) + lo
    return out


# --------------------------------------------------------------------------------------
# Selective precision (Section 4).  Modules of a Transformer layer are numbered as in
# Section 4.2: 1 = QKV projection, 2 = attention output projection, 3 and 4 = the two
# feed-forward modules.  Horizontal selection (Section 4.1) keeps X first / last /
# middle layers at 8 bit; vertical selection (Section 4.2) a subset of modules; the
# hybrid rule (Section 4.3) both: modules in `modules` of the selected layers get 8 bit,
# everything else 4 bit.
# --------------------------------------------------------------------------------------
POLICIES = ("first", "last", "middle")


def selected_layers(n_layers: int, policy: str, X: int) -> list[int]:
    """0-based indices of the X layers kept at high precision (Section 4.1).
    'middle' centres the run of X layers; when the slack is odd the extra unselected
    layer is at the end (the paper does not say; this is the reading taken)."""
    if policy not in POLICIES:
        raise ValueError("policy")
    if not 0 <= X <= n_layers:
        raise ValueError("X")
    if policy == "first":
        start = 0
    elif policy == "last":
        start = n_layers - X
    else:
        start = (n_layers - X) // 2
    return list(range(start, start + X))


def plan_bits(layer: int, n_layers: int, module_id: int, policy: str, X: int,
              modules=(1, 2, 3, 4), hi_bits: int = 8, lo_bits: int = 4) -> int:
    """Bits of (layer, module) under the hybrid rule of Section 4.3."""
    if module_id not in (1, 2, 3, 4):
        raise ValueError("module_id")
    sel = layer in selected_layers(n_layers, policy, X)
    return hi_bits if (sel and module_id in tuple(modules)) else lo_bits


def effective_bits(n_layers: int, module_params, policy: str, X: int,
                   modules=(1, 2, 3, 4)) -> float:
    """Average bits per weight over the linear modules of all layers (Section 4.3's
    'effectively quantized into 5 bit, on average').  module_params[i] = number of
    weights of module i+1 in one layer.  Scale storage is not counted."""
    total = 0
    bits_sum = 0
    for layer in range(n_layers):
        for mid in (1, 2, 3, 4):
            p = int(module_params[mid - 1])
            total += p
            bits_sum += p * plan_bits(layer, n_layers, mid, policy, X, modules)
    return bits_sum / total
