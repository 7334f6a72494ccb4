"""CPU-side tests of the C-ABI library: it loads, exports everything include/rtn.h declares,
validates arguments before touching the GPU, and its host-only planning functions agree with
the oracle's selective-precision bookkeeping (Section 4)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2505_15909_amd as rtn
from oracle import rtn_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
lib = rtn._lib
FAKE = 0x1000   # a 16-byte aligned non-null "device pointer"; never dereferenced by validation


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "rtn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(rtn_[a-z0-9_]+)\s*\(", text))
    assert declared == set(rtn.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_sizes_and_status_strings():
    assert rtn.rtn_layout_version() == 1
    assert rtn.rtn_qweight_nbytes(4096, 4096, 4) == 4096 * 4096 // 2
    assert rtn.rtn_qweight_nbytes(4096, 4096, 8) == 4096 * 4096
    assert rtn.rtn_scales_nbytes(4096, 4096, 128) == 4096 * 32 * 2
    assert rtn.rtn_scales_nbytes(4096, 4096, 0) == 4096 * 2
    assert rtn.rtn_qweight_nbytes(4096, 4096, 5) == 0
    assert rtn.rtn_qweight_nbytes(4100, 4096, 4) == 0
    assert 256 <= rtn.rtn_workspace_nbytes(1, 4096, 4096, 4, 128) <= 16 << 20
    assert rtn.rtn_workspace_nbytes(128, 106496, 16384, 4, 128) <= 16 << 20
    for s in range(9):
        assert lib.rtn_status_str(s)
    assert lib.rtn_status_str(0) == b"ok"


def _quant(W=FAKE, N=64, K=512, bits=4, g=128, flags=0, q=FAKE, s=FAKE):
    return lib.rtn_quantize(W, N, K, bits, g, flags, q, s, None)


def _linear(A=FAKE, M=1, q=FAKE, s=FAKE, N=64, K=512, bits=4, g=128, Cp=FAKE, ws=FAKE, wsn=1 << 20, cfg=None):
    if (A, q, s, Cp, ws) == (FAKE,) * 5:
        # nothing about the pointers is under test: the host-only entry point, which cannot launch anything
        return lib.rtn_linear_validate(M, N, K, bits, g, wsn, cfg)
    # a NULL or misaligned pointer: rejected by the pointer checks, which come before any plan or launch
    assert None in (A, q, s, Cp) or any(p is not None and p % 16 for p in (A, q, s, Cp, ws))
    return lib.rtn_linear_ex(A, M, q, s, N, K, bits, g, Cp, ws, wsn, None, cfg)


def test_argument_validation_happens_before_any_launch():
    assert _quant(W=None) == 1 and _quant(q=None) == 1 and _quant(s=None) == 1
    assert _quant(bits=3) == 2 and _quant(bits=16) == 2
    assert _quant(g=96) == 3 and _quant(g=16) == 3 and _quant(g=1024) == 3      # 1024 > K
    assert _quant(N=60) == 4 and _quant(K=640) == 4 and _quant(N=0) == 4
    assert _quant(W=FAKE + 8) == 5 and _quant(q=FAKE + 2) == 5
    assert _quant(flags=7) == 7
    assert _linear(A=None) == 1 and _linear(Cp=None) == 1
    assert _linear(bits=5) == 2
    assert _linear(g=100) == 3
    assert _linear(M=0) == 4 and _linear(K=500) == 4
    assert _linear(A=FAKE + 4) == 5
    cfg = rtn.rtn_linear_cfg(path=1, prefetch=3)
    assert _linear(cfg=C.byref(cfg)) == 7
    cfg = rtn.rtn_linear_cfg(waves_n=17)
    assert _linear(cfg=C.byref(cfg)) == 7                         # wavefronts along N: 1 .. 16
    cfg = rtn.rtn_linear_cfg(waves_n=3, waves_k=6)
    assert _linear(cfg=C.byref(cfg)) == 7                         # more than 16 wavefronts
    cfg = rtn.rtn_linear_cfg(waves_n=8, waves_k=4)
    assert _linear(cfg=C.byref(cfg)) == 7                         # at most 16 wavefronts per workgroup
    cfg = rtn.rtn_linear_cfg(path=5)
    assert _linear(cfg=C.byref(cfg)) == 7
    cfg = rtn.rtn_linear_cfg(path=4, split_k=9)
    assert _linear(M=200, cfg=C.byref(cfg)) == 7                  # more splits than 128-column k-steps
    cfg = rtn.rtn_linear_cfg(path=4)
    assert _linear(M=200, bits=8, g=64, cfg=C.byref(cfg)) == 7    # group 64 is below the tile kernel's k-step
    cfg = rtn.rtn_linear_cfg(path=2)
    assert _linear(M=2, bits=4, g=64, cfg=C.byref(cfg)) == 7      # the vector-ALU variant needs whole-tile groups
    assert lib.rtn_gemm_fp16(None, 1, FAKE, 16, 128, FAKE, None, 0, None) == 1
    assert lib.rtn_gemm_fp16(FAKE, 1, FAKE, 16, 100, FAKE, None, 0, None) == 4
    assert lib.rtn_gemm_fp16(FAKE, 1, FAKE + 2, 16, 128, FAKE, None, 0, None) == 5
    assert lib.rtn_linear_dense(FAKE, 1, FAKE, FAKE, 64, 512, 4, 128, FAKE, FAKE, 100, None, 0, None) == 6
    assert rtn.rtn_dense_weight_nbytes(64, 512) == 64 * 512 * 2
    qh = lib.rtn_quantize_from_host
    assert lib.rtn_quantize_host_staging_nbytes(512, 32) == 2 * 32 * 512 * 2 and lib.rtn_quantize_host_staging_nbytes(512, 20) == 0
    assert qh(None, 64, 512, 4, 128, 0, FAKE, FAKE, FAKE, 1 << 20, 32, None, FAKE) == 1
    assert qh(FAKE, 64, 512, 4, 128, 0, FAKE, FAKE, FAKE, 1 << 20, 20, None, FAKE) == 4        # shard rows: a multiple of 16
    assert qh(FAKE, 64, 512, 4, 128, 0, FAKE, FAKE, FAKE, 1000, 32, None, FAKE) == 6            # staging too small
    assert qh(FAKE, 64, 512, 4, 128, 0, FAKE, FAKE, FAKE, 1 << 20, 32, FAKE, FAKE) == 7         # needs two streams
    assert qh(FAKE, 64, 512, 4, 100, 0, FAKE, FAKE, FAKE, 1 << 20, 32, None, FAKE) == 3
    for bad in (dict(m_rows16=1), dict(m_rows16=5), dict(m_rows16=2, n_tiles16=3), dict(m_rows16=4, n_tiles16=4),
                dict(m_rows16=2, n_tiles16=1, split_k=1000)):
        cfg = rtn.rtn_linear_cfg(path=3, **bad)                    # the wide kernel's register-tile limits
        assert _linear(M=40, cfg=C.byref(cfg)) == 7
    cfg = rtn.rtn_linear_cfg(path=3, m_rows16=2, n_tiles16=1)
    assert _linear(M=40, bits=8, g=64, K=512, cfg=C.byref(cfg)) == 7     # its k-steps are 128 columns
    cfg = rtn.rtn_linear_cfg(path=2)
    assert _linear(M=5, cfg=C.byref(cfg)) == 7                    # the vector-ALU path is for M <= 4
    cfg = rtn.rtn_linear_cfg(split_k=2)
    assert _linear(K=1024, wsn=16, cfg=C.byref(cfg)) == 6         # workspace too small
    cfg = rtn.rtn_linear_cfg(split_k=4)
    assert _linear(K=1024, cfg=C.byref(cfg)) == 7                 # more splits than chunks
    assert lib.rtn_unpack(None, 64, 512, 4, FAKE, None) == 1
    assert lib.rtn_dequantize(FAKE, FAKE, 64, 512, 4, 100, FAKE, None) == 3
    assert lib.rtn_layer_forward(None, 1, FAKE, 256, None) == 1
    assert lib.rtn_grouped_forward(None, 1, FAKE, 256, None) == 1
    # asymmetric variant: same validation, plus the zero-point array
    assert lib.rtn_quantize_asym(FAKE, 64, 512, 4, 128, FAKE, FAKE, None, None) == 1
    assert lib.rtn_quantize_asym(FAKE, 64, 512, 5, 128, FAKE, FAKE, FAKE, None) == 2
    assert lib.rtn_quantize_asym(FAKE, 64, 512, 4, 100, FAKE, FAKE, FAKE, None) == 3
    assert lib.rtn_quantize_asym(FAKE, 60, 512, 4, 128, FAKE, FAKE, FAKE, None) == 4
    assert lib.rtn_quantize_asym(FAKE, 64, 512, 4, 128, FAKE, FAKE, FAKE + 8, None) == 5
    assert lib.rtn_dequantize_asym(FAKE, FAKE, None, 64, 512, 4, 128, FAKE, None) == 1
    assert lib.rtn_linear_asym(FAKE, 1, FAKE, FAKE, None, 64, 512, 4, 128, FAKE, FAKE, 256, None) == 1
    assert lib.rtn_linear_asym(FAKE, 0, FAKE, FAKE, FAKE, 64, 512, 4, 128, FAKE, FAKE, 256, None) == 4


def test_bad_valid_combination_is_not_launched_without_gpu():
    # a per-channel request is g <= 0 or g == K
    q = rtn.rtn_linear_query(1, 4096, 4096, 4, 0)
    assert q["path"] == 1 and q["split_k"] >= 1
    # more than 16 rows go to the wide kernel (group sizes that are multiples of 128), within its tile limits
    for M in (17, 32, 33, 64, 100, 128, 1000):
        q = rtn.rtn_linear_query(M, 4096, 4096, 4, 128)
        assert q["path"] == 3 and 2 <= q["m_rows16"] <= 4 and q["m_rows16"] * q["n_tiles16"] <= 8
        assert M * 4096 * 4 * q["split_k"] <= 16 << 20 or q["split_k"] == 1
    assert rtn.rtn_linear_query(64, 4096, 4096, 8, 64)["path"] == 1
    assert rtn.rtn_linear_query(32, 16384, 106496, 4, 128)["path"] == 1     # very large matrix at 32 rows: streaming wins
    # 128-256 rows on a large 4-bit matrix below the tile kernel's range: the wide kernel's 128-row variant, K split to a
    # workgroup per compute unit, and the size helper covers its partial sums
    q = rtn.rtn_linear_query(128, 16384, 53248, 4, 128)
    assert (q["path"], q["m_rows16"], q["n_tiles16"], q["waves_n"], q["split_k"]) == (3, 8, 2, 8, 4)
    assert rtn.rtn_workspace_nbytes(128, 16384, 53248, 4, 128) == 128 * 16384 * 4 * 4
    # one row more: the 128-row variant would pad to 256, and the tile kernel with K in four splits is modelled (and
    # measured) ahead of the 64-row wide plan
    q = rtn.rtn_linear_query(129, 16384, 53248, 4, 128)
    assert (q["path"], q["m_rows16"], q["split_k"]) == (4, 8, 4)
    assert rtn.rtn_linear_query(128, 16384, 53248, 8, 0)["m_rows16"] == 4
    assert rtn.rtn_linear_query(128, 4096, 14336, 4, 128)["m_rows16"] == 4
    # tile kernel: height and K split chosen together so that the last round of 256 workgroups is filled
    # (72 column blocks x 1 tall row block x 3 splits = 216 workgroups instead of 144 short tiles in one round)
    q = rtn.rtn_linear_query(256, 18432, 16384, 4, 128)
    assert (q["path"], q["m_rows16"], q["split_k"]) == (4, 8, 3)
    assert rtn.rtn_workspace_nbytes(256, 18432, 16384, 4, 128) == 256 * 18432 * 4 * 3
    q = rtn.rtn_linear_query(4096, 28672, 4096, 4, 128)
    assert (q["path"], q["split_k"]) == (4, 1)
    with pytest.raises(rtn.RtnError):
        rtn.rtn_linear_query(1, 4096, 4000, 4, 128)


@pytest.mark.parametrize("n_layers", [16, 32, 80, 126])
def test_plan_bits_matches_oracle(n_layers):
    for policy in ("first", "last", "middle"):
        for X in (0, 1, n_layers // 4, n_layers // 2, n_layers):
            for modules in ((1, 2, 3, 4), (1, 3, 4), (2,), ()):
                for layer in range(n_layers):
                    for mid in (1, 2, 3, 4):
                        assert rtn.rtn_plan_bits(layer, n_layers, mid, policy, X, modules) == \
                            O.plan_bits(layer, n_layers, mid, policy, X, modules)
    assert rtn.rtn_plan_bits(n_layers, n_layers, 1, "first", 1) == -1
    assert rtn.rtn_plan_bits(0, n_layers, 5, "first", 1) == -1


def test_effective_bits_matches_oracle_and_paper():
    p8b = [4096 * 6144, 4096 * 4096, 4096 * 28672, 14336 * 4096]
    p70 = [8192 * 10240, 8192 * 8192, 8192 * 57344, 28672 * 8192]
    assert rtn.rtn_plan_effective_bits(32, p8b, "first", 8) == 5.0          # Section 4.3
    assert rtn.rtn_plan_effective_bits(32, p8b, "first", 16) == 6.0
    extra = rtn.rtn_plan_effective_bits(80, p70, "first", 1, (1, 3, 4)) - 4
    assert 0 < extra < 0.05                                                # Sections 1, 6
    for pol in ("first", "last", "middle"):
        for X in (0, 3, 20, 80):
            for mods in ((1, 2, 3, 4), (1, 3, 4), (3,)):
                a = rtn.rtn_plan_effective_bits(80, p70, pol, X, mods)
                b = O.effective_bits(80, p70, pol, X, mods)
                assert abs(a - b) < 1e-12


def test_fp32_arithmetic_of_the_gpu_path_equals_exact_rounding():
    """Host-logic check of the arithmetic the quantise kernel uses: IEEE fp32 division followed by
    fp16 rounding (scales) or rint (codes) equals the oracle's single rounding of the exact quotient."""
    halves = np.arange(1, 0x7C00, dtype=np.uint16).view(np.float16)
    for bits in (4, 8):
        for rule in ("qmax", "eq2"):
            D = np.float32(O.scale_divisor(bits, rule))
            s32 = (halves.astype(np.float32) / D).astype(np.float16)
            assert np.array_equal(s32.view(np.uint16), O.rtn_scale(halves, bits, rule).view(np.uint16))
    rng = np.random.default_rng(0)
    w = rng.integers(1, 0x7C00, size=2_000_000).astype(np.uint16).view(np.float16)
    s = rng.integers(1, 0x7C00, size=2_000_000).astype(np.uint16).view(np.float16)
    keep = np.abs(w.astype(np.float64) / s.astype(np.float64)) < 300
    w, s = w[keep], s[keep]
    q32 = np.rint(w.astype(np.float32) / s.astype(np.float32))
    q64 = np.rint(w.astype(np.float64) / s.astype(np.float64))
    assert np.array_equal(q32.astype(np.float64), q64)
    # exact ties are hit, not avoided
    t = np.array([0.5, 1.5, 2.5, 6.5, 126.5], dtype=np.float16)
    for sc in (np.float16(1.0), np.float16(0.0123), np.float16(2.0 ** -14)):
        ws = (t.astype(np.float32) * np.float32(sc)).astype(np.float16)
        if np.array_equal(ws.astype(np.float64), t.astype(np.float64) * float(sc)):
            assert np.rint(ws.astype(np.float32) / np.float32(sc)).tolist() == [0, 2, 2, 6, 126]


def _fp32_round_on_grid(x, grid_log2):
    """Round-half-even of the exact rational x onto multiples of 2^grid_log2 (one fp32 rounding inside a binade)."""
    from fractions import Fraction
    t = x / Fraction(2) ** grid_log2
    f = t.numerator // t.denominator
    rem = t - f
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and f % 2 == 1):
        f += 1
    return f * Fraction(2) ** grid_log2


def _snapped_code_exact(w16, s16, bits):
    """The per-element arithmetic of the quantise kernels in exact rationals with explicit fp32 roundings:
    r = fp32(1 / S); y = fp32(w r + C) for C = 768 + offset; z = rint(y)."""
    from fractions import Fraction
    off = 8 if bits == 4 else 128
    r = Fraction(float(np.float32(1.0) / np.float32(s16))) if float(s16) != 0.0 else Fraction(0)
    t = Fraction(float(w16)) * r + 768 + off
    assert 512 <= t < 2048
    y = _fp32_round_on_grid(t, -14 if t < 1024 else -13)       # fp32 spacing in [512, 1024) and [1024, 2048)
    z = _fp32_round_on_grid(y, 0)
    lo, hi = 768 + off - (1 << (bits - 1)), 768 + off + (1 << (bits - 1)) - 1
    return int(min(max(z, lo), hi)) - 768 - off, y


def _snapped_code_fp64(w16, s16, off):
    """Vectorised version of the same (the fused multiply-add formed in fp64, then rounded to fp32)."""
    s = s16.astype(np.float32)
    r = np.where(s == 0, np.float32(0), np.float32(1.0) / np.where(s == 0, np.float32(1), s)).astype(np.float32)
    y = (w16.astype(np.float64) * r.astype(np.float64) + (768.0 + off)).astype(np.float32)
    return y, np.rint(y).astype(np.float64) - (768.0 + off)


def test_reciprocal_and_snap_arithmetic_rounds_like_the_exact_quotient():
    """The quantise kernels never divide per element: y = fma(w, 1/S, C) lands on a 2^-14 grid on which true
    ties are hit exactly, and rint(y) - C is the code.  Checked against exact rational arithmetic: random
    (w, S) pairs, and constructed exact ties w = (i + 1/2) S with scales that are not powers of two."""
    from fractions import Fraction
    rng = np.random.default_rng(1)

    def rne(x):
        f = x.numerator // x.denominator
        rem = x - f
        return f + 1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and f % 2 == 1) else f

    # bulk, vectorised, against fp64 division (exact enough away from ties; ties are covered below)
    for off, lim in ((8, 8.6), (128, 128.6)):
        w = rng.integers(0, 0x7C00, size=1_000_000).astype(np.uint16).view(np.float16)
        w = np.where(rng.random(w.size) < 0.5, -w, w).astype(np.float16)
        s = rng.integers(1, 0x7C00, size=1_000_000).astype(np.uint16).view(np.float16)
        keep = np.abs(w.astype(np.float64) / s.astype(np.float64)) < lim
        w, s = w[keep], s[keep]
        assert w.size > 1000
        _, q = _snapped_code_fp64(w, s, off)
        assert np.array_equal(q, np.rint(w.astype(np.float64) / s.astype(np.float64)))
    # group-shaped samples (|w| <= amax, S = fp16(amax / D)), exact rationals, clamp included
    for bits in (4, 8):
        for rule in ("qmax", "eq2"):
            D = O.scale_divisor(bits, rule)
            amax = rng.integers(1, 0x7C00, size=300).astype(np.uint16).view(np.float16)
            amax[:40] = np.arange(1, 41, dtype=np.uint16).view(np.float16)          # subnormal scales
            for am in amax:
                sc = O.rtn_scale(np.array([am]), bits, rule)[0]
                ws = (rng.random(6) * float(am)).astype(np.float16)
                ws[0] = am
                for wv in ws:
                    for sign in (1.0, -1.0):
                        got, _ = _snapped_code_exact(np.float16(sign * float(wv)), sc, bits)
                        if float(sc) == 0.0:
                            want = 0
                        else:
                            want = rne(Fraction(sign * float(wv)) / Fraction(float(sc)))
                            want = min(max(want, -(1 << (bits - 1))), (1 << (bits - 1)) - 1)
                        assert got == want, (bits, rule, float(am), float(wv), float(sc))
    # exact ties with non-power-of-two scales
    checked = 0
    for bits, imax in ((4, 8), (8, 128)):
        for i in range(imax):
            odd = 2 * i + 1
            for _ in range(30):
                ms = int(rng.integers(1, max(2, 2047 // odd + 1)))
                ex = int(rng.integers(-20, 6))
                sv, wv = ms * 2.0 ** ex, odd * ms * 2.0 ** (ex - 1)
                if wv > 65504 or float(np.float16(sv)) != sv or float(np.float16(wv)) != wv or sv < 2.0 ** -24:
                    continue
                for sign in (1, -1):
                    got, y = _snapped_code_exact(np.float16(sign * wv), np.float16(sv), bits)
                    off = 8 if bits == 4 else 128
                    assert y == Fraction(sign * odd, 2) + 768 + off            # the tie itself, not a neighbour
                    even = i if i % 2 == 0 else i + 1
                    want = min(max(sign * even, -(1 << (bits - 1))), (1 << (bits - 1)) - 1)
                    assert got == want
                    checked += 1
    assert checked > 3000


def test_every_automatic_plan_is_a_valid_configuration():
    """Host logic: for a spread of shapes (the paper's Llama shapes and random ones), every batch size and both
    precisions, the plan rtn_linear would choose passes the library's own validation when handed back explicitly,
    fits the workspace the size helper promises (16 MiB; 64 MiB under the wide kernel's plans from 64 rows, 256 MiB under the tile kernel's).  Only the host-side validation entry point is called: nothing here can reach a launch."""
    rng = np.random.default_rng(7)
    shapes = [(4096, 6144), (4096, 4096), (4096, 28672), (14336, 4096), (8192, 10240), (8192, 57344), (28672, 8192),
              (16384, 18432), (16384, 106496), (53248, 16384)]
    for _ in range(40):
        shapes.append((int(rng.integers(1, 40)) * 512, int(rng.integers(1, 600)) * 16))
    Ms = [1, 2, 3, 4, 5, 8, 15, 16, 17, 31, 32, 33, 48, 49, 64, 65, 100, 128, 129, 256, 1000, 4096]
    checked = 0
    for K, N in shapes:
        for bits, g in ((4, 32), (4, 64), (4, 128), (4, 0), (8, 32), (8, 64), (8, 128), (8, 0)):
            if g and K % g:
                continue
            for M in Ms:
                q = rtn.rtn_linear_query(M, N, K, bits, g)
                assert q["path"] in (1, 3, 4), q
                need = M * N * 4 * q["split_k"] if q["split_k"] > 1 else 0
                assert need <= rtn._lib.rtn_workspace_nbytes(M, N, K, bits, g), (M, N, K, bits, g, q)
                cfg = rtn.rtn_linear_cfg(**q)
                cap = 256 << 20 if q["path"] == 4 else (64 << 20 if q["path"] == 3 and M >= 64 else 16 << 20)
                assert need <= cap, (M, N, K, bits, g, q)
                if q["path"] == 4:
                    assert q["m_rows16"] in (4, 8) and (M > 128 or q["m_rows16"] == 4), q
                st = lib.rtn_linear_validate(M, N, K, bits, g, 256 << 20, C.byref(cfg))
                assert st == 0, (st, M, N, K, bits, g, q)      # host-only validation: nothing is launched
                checked += 1
    assert checked > 3000


def test_plans_of_untuned_shapes_fill_the_compute_units_evenly():
    """Host logic: on shapes outside the measured plan table (the held-out files of the tuning folder), the skinny plan
    chosen at 12-16 rows for a large matrix does not start a second round of workgroups on a few compute units: its
    workgroup count is not one or two full rounds of 256 plus a sliver (such a count was measured 25-35 % slower), and the Llama shapes, which are table entries, get exactly the measured best configuration."""
    tuning = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2505_15909_amd", "tuning")
    checked = 0
    for name in ("shapes_heldout.txt", "shapes_heldout2.txt"):
        for line in open(os.path.join(tuning, name)):
            _, K, N = line.split()
            K, N = int(K), int(N)
            for bits, g in ((4, 128), (8, 0)):
                if N * K * bits // 8 < (64 << 20) or K % (512 if bits == 4 else 256):     # small, or K not whole k-chunks
                    continue
                for M in (12, 16):
                    q = rtn.rtn_linear_query(M, N, K, bits, g)
                    assert q["path"] == 1
                    wgs = -(-(N // 16) // q["waves_n"]) * q["split_k"]
                    rounds = wgs / 256.0
                    spill = rounds - np.floor(rounds)            # the part of a round the last workgroups occupy
                    assert not (1 <= np.floor(rounds) <= 2 and 0 < spill < 0.2), (K, N, bits, M, q, wgs)
                    checked += 1
    assert checked >= 12
    best = {}
    for line in open(os.path.join(tuning, "plan_sweep_results.txt")):
        if line.startswith("#"):
            continue
        head, first = line.split("|")[:2]
        best[tuple(int(v) for v in head.split())] = tuple(int(v) for v in first.split()[:4])
    for bits, K, N, M in ((4, 4096, 28672, 16), (4, 8192, 57344, 8), (4, 16384, 106496, 16), (8, 16384, 18432, 16), (4, 14336, 4096, 1)):
        q = rtn.rtn_linear_query(M, N, K, bits, 128 if bits == 4 else 0)
        assert (q["waves_n"], q["waves_k"], q["split_k"], q["prefetch"]) == best[(bits, K, N, M)], (bits, K, N, M, q)


def test_size_limits_are_refused_on_the_host():
    """The kernels address every tensor with 32-bit byte offsets: a packed weight tensor or an activation tensor of
    2 GiB - 64 KiB or more, more than 2^20 rows, or 2^23 columns and more are refused with RTN_ERR_SHAPE before anything
    is launched; one step inside each limit passes.  Host-only validation entry point: no pointers, no launch."""
    def status(M, N, K, bits, g):
        return lib.rtn_linear_validate(M, N, K, bits, g, 256 << 20, None)
    assert status(1, 65536, 65536, 4, 128) == 4 and status(1, 65536, 65536 - 512, 4, 128) == 0       # 2 GiB of int4 codes
    assert status(1, 32768, 65536, 8, 0) == 4 and status(1, 32768, 65536 - 256, 8, 0) == 0           # 2 GiB of int8 codes
    assert status(1, 16, 1 << 23, 4, 128) == 4 and status(1, 16, (1 << 23) - 512, 4, 128) == 0       # columns
    assert status((1 << 20) + 1, 16, 512, 4, 128) == 4 and status(1 << 20, 16, 512, 4, 128) == 0     # rows
    assert status(40000, 16, 32768, 4, 128) == 4                                                     # activations of 2.4 GiB
    with pytest.raises(rtn.RtnError) as e:
        rtn.rtn_linear_query(1, 65536, 65536, 4, 128)
    assert e.value.status == 4


def test_bench_refuses_more_than_one_gpu():
    """This build measures one GPU; asking the benchmark for more exits with a message before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
