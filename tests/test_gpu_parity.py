"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, on the same seeded inputs.

Quantise / pack: bit-exact on packed bytes and scales (Section 2.2, Eq. 1-2; layout of rtn.h).
Linear: relative Frobenius error <= 2e-3 and max abs error <= 1e-2 (+ one fp16 rounding of the
result, 2^-11 |C|, which matters only where |C| >= 8) against the float64 GEMM on the oracle's
own dequantised weights (Sections 2.3, 5).
"""
import itertools

import os

import numpy as np
import pytest
import torch

from oracle import rtn_oracle as O
from paper_2505_15909_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _to_np(t):
    return t.detach().cpu().numpy()


def _quantize_both(W_t, bits, g, flags=0):
    rtn = pytest.importorskip("paper_2505_15909_amd")
    qw, sc = rtn.rtn_quantize(W_t, bits, g, flags)
    torch.cuda.synchronize()
    W = _to_np(W_t)
    gg = W.shape[1] if g <= 0 else g
    codes, scales = O.rtn_quantize(W, bits, gg, "eq2" if flags else "qmax")
    return qw, sc, codes, scales


# ----------------------------------------------------------------------------------------
# quantise + pack
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits,g", [(4, 32), (4, 64), (4, 128), (4, 256), (4, 512), (4, 1024), (4, 0), (8, 32), (8, 64),
                                     (8, 128), (8, 256), (8, 512), (8, 0)])
@pytest.mark.parametrize("N,K", [(80, 2048), (16, 512), (272, 3072)])
def test_quantize_bit_exact_small(rtn, bits, g, N, K):
    if g > K or (g > 0 and K % g):
        pytest.skip("group does not divide K")
    W_t = synth.normal_weight(N, K, 0.02, seed=N + K + bits, device=DEV)
    qw, sc, codes, scales = _quantize_both(W_t, bits, g)
    assert np.array_equal(_to_np(sc).view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(_to_np(qw), O.pack_gfx950(codes, bits))
    assert np.array_equal(_to_np(rtn.rtn_unpack(qw, N, K, bits)), codes)


@pytest.mark.parametrize("bits,g", [(4, 128), (8, 64), (4, 32), (4, 64), (8, 32)])
@pytest.mark.parametrize("flags", [0, 1])
def test_quantize_adversarial(rtn, bits, g, flags):
    """Exact ties, all-zero groups, fp16 subnormals, +-65504, -0.0, one huge outlier per group."""
    N, K = 64, 1024
    rng = np.random.default_rng(11)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    qmax = (1 << (bits - 1)) - 1
    W[0, :g] = ((np.arange(g) % 29) - 14) * 0.5 * 2.0 ** -8          # ties at every half step
    W[0, 0] = qmax * 2.0 ** -8
    W[1, :g] = 0.0
    W[2, :g] = -0.0
    W[3, :g] = (rng.integers(-20, 21, size=g) * 2.0 ** -24).astype(np.float16)   # subnormals
    W[4, :g] = (rng.integers(-3, 4, size=g) * 2.0 ** -24).astype(np.float16)     # scale underflows to 0 / 1 ulp
    W[5, 0], W[5, 1] = 65504.0, -65504.0
    W[6, 7] = 300.0                                                   # outlier: the rest rounds to 0
    W[7, :g] = np.float16(0.3)                                        # constant group
    W[8, g:2 * g] = (np.arange(g) - g // 2) * np.float16(0.011)        # inexact scale, near-ties
    for r in range(9, 32):                                            # multiples of half a scale step
        s = np.float16(rng.uniform(0.001, 0.1))
        W[r, :g] = (rng.integers(-2 * qmax, 2 * qmax + 1, size=g) * 0.5 * float(s)).astype(np.float16)
    # subnormal scales of one or a few ulps: the quotient overshoots the code range by up to 1.5x and is clamped
    for r, a in zip(range(32, 44), (10, 11, 17, 180, 190, 191, 300, 317, 500, 700, 1000, 1023)):
        W[r, :] = 0.0
        W[r, :g] = (rng.integers(-a, a + 1, size=g) * 2.0 ** -24).astype(np.float16)
        W[r, 0] = np.float16(a * 2.0 ** -24)
        W[r, 1] = np.float16(-a * 2.0 ** -24)
    W_t = torch.from_numpy(W).to(DEV)
    qw, sc, codes, scales = _quantize_both(W_t, bits, g, flags)
    assert np.array_equal(_to_np(sc).view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(_to_np(qw), O.pack_gfx950(codes, bits))
    # per-channel on the same tensor
    qw, sc, codes, scales = _quantize_both(W_t, bits, 0, flags)
    assert np.array_equal(_to_np(sc).view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(_to_np(qw), O.pack_gfx950(codes, bits))


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("K,g", [(4096, 0), (5120, 0), (8192, 0), (11264, 0), (14336, 0), (16384, 0), (28672, 0),
                                 (8192, 4096), (14336, 7168), (32768, 16384), (19456, 0), (40960, 0), (53248, 0), (57344, 0),
                                 (65536, 0)])
def test_quantize_large_groups_every_kernel(rtn, bits, K, g):
    """Per-channel and wide groups: the register-resident kernels (16 wavefronts x 16 rows with up to 8 loads per lane;
    8 wavefronts x 8 or 4 rows with 16 or 28; 16 wavefronts x 4 rows with 28; groups that do not fill the last
    wavefront's tiles) and the two-pass kernel beyond 57344 columns."""
    N = 48
    W_t = synth.heavy_tail_weight(N, K, 0.02, seed=K + bits, device=DEV)
    qw, sc, codes, scales = _quantize_both(W_t, bits, g)
    assert np.array_equal(_to_np(sc).view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(_to_np(qw), O.pack_gfx950(codes, bits))


@pytest.mark.parametrize("bits,g", [(4, 128), (8, 0)])
@pytest.mark.parametrize("rows_per_shard", [16, 48, 112, 4096])
def test_quantize_from_host_matches_device_quantize(rtn, bits, g, rows_per_shard):
    """The load-time pipeline (host tensor -> staged shards -> quantise) gives the bits of a single rtn_quantize call,
    for shard sizes that divide N, that do not, and that exceed it; twice in a row on the same staging buffer."""
    N, K = 272, 2048
    W_host = synth.heavy_tail_weight(N, K, 0.02, seed=21, device="cpu").pin_memory()
    q_ref, s_ref = rtn.rtn_quantize(W_host.to(DEV), bits, g)
    cs = torch.cuda.Stream()
    staging = torch.empty(rtn._lib.rtn_quantize_host_staging_nbytes(K, rows_per_shard), dtype=torch.uint8, device=DEV)
    for _ in range(2):
        q, s = rtn.rtn_quantize_from_host(W_host, bits, g, rows_per_shard, cs, staging=staging, device=DEV)
        torch.cuda.synchronize()
        assert torch.equal(q, q_ref) and torch.equal(s.view(torch.int16), s_ref.view(torch.int16))
    codes, scales = O.rtn_quantize(W_host.numpy(), bits, K if g == 0 else g)
    assert np.array_equal(_to_np(q), O.pack_gfx950(codes, bits))


def test_quantize_is_deterministic_and_dequantize_matches(rtn):
    N, K = 256, 2048
    W_t = synth.heavy_tail_weight(N, K, 0.02, seed=5, device=DEV)
    for bits, g in ((4, 128), (8, 0)):
        q1, s1 = rtn.rtn_quantize(W_t, bits, g)
        q2, s2 = rtn.rtn_quantize(W_t, bits, g)
        assert torch.equal(q1, q2) and torch.equal(s1, s2)
        codes, scales = O.rtn_quantize(_to_np(W_t), bits, K if g == 0 else g)
        deq = rtn.rtn_dequantize(q1, s1, K, bits, g)
        want = O.rtn_dequantize(codes, scales, K if g == 0 else g).astype(np.float16)
        assert np.array_equal(_to_np(deq).view(np.uint16), want.view(np.uint16))


# ----------------------------------------------------------------------------------------
# linear: small shapes, every kernel configuration
# ----------------------------------------------------------------------------------------
def _oracle_operands(N, K, bits, g, seed, dist="normal02"):
    W_t = H.make_weight(dist, N, K, seed, DEV)
    W = _to_np(W_t)
    gg = K if g <= 0 else g
    codes, scales = O.rtn_quantize(W, bits, gg)
    qw = torch.from_numpy(O.pack_gfx950(codes, bits)).to(DEV)
    sc = torch.from_numpy(scales).to(DEV)
    return codes, scales, qw, sc, gg


CFGS = [dict(prefetch=nb, waves_n=wn, waves_k=wk, split_k=sk)
        for nb, wn, wk, sk in [(1, 1, 1, 1), (1, 1, 4, 1), (2, 1, 2, 2), (1, 2, 2, 1), (2, 2, 1, 3), (2, 1, 1, 1),
                               (1, 4, 1, 1), (2, 4, 2, 2), (2, 4, 1, 1), (1, 1, 8, 1), (1, 8, 1, 2), (2, 2, 4, 4),
                               (1, 1, 16, 1), (2, 16, 1, 1), (1, 2, 8, 1), (2, 8, 2, 1), (1, 1, 3, 1), (1, 2, 7, 1), (2, 1, 5, 2),
                               # any number of wavefronts along N, not only powers of two
                               (2, 3, 1, 1), (1, 7, 1, 1), (2, 13, 1, 2), (2, 5, 3, 1), (1, 3, 5, 2), (2, 6, 2, 3), (2, 15, 1, 1)]]


@pytest.mark.parametrize("bits,g", [(4, 32), (4, 64), (4, 128), (4, 256), (4, 512), (4, 0), (8, 32), (8, 64), (8, 128),
                                     (8, 256), (8, 0)])
def test_linear_all_configs_small(rtn, bits, g):
    N, K = 272, 3072            # 17 tile rows (ragged against every WN*R), 6 / 12 chunks
    codes, scales, qw, sc, gg = _oracle_operands(N, K, bits, g, seed=3)
    for M in (1, 2, 3, 4, 5, 8, 13, 16):
        A_t = synth.activation(M, K, seed=100 + M, device=DEV)
        ref = O.rtn_linear(_to_np(A_t), codes, scales, gg)
        ran = 0
        for cfg in CFGS:
            if cfg["split_k"] > K // (512 if bits == 4 else 256):
                continue
            try:
                C = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=cfg)
            except rtn.RtnError as e:
                # the only legitimate refusal: a workgroup too small to stage this many activation rows
                assert e.status == 7 and M > 4
                continue
            torch.cuda.synchronize()
            ran += 1
            H.assert_linear_close(_to_np(C), ref, f"bits={bits} g={g} M={M} cfg={cfg}")
        assert ran >= 6
        C = rtn.rtn_linear(A_t, qw, sc, bits, g)          # automatic plan
        torch.cuda.synchronize()
        H.assert_linear_close(_to_np(C), ref, f"bits={bits} g={g} M={M} auto")


@pytest.mark.parametrize("bits,g", [(4, 128), (4, 0), (8, 128), (8, 0)])
def test_linear_vector_alu_path(rtn, bits, g):
    """The v_dot2 wavefront-reduction variant (path 2, M <= 4) against the oracle and the MFMA path."""
    N, K = 272, 3072
    codes, scales, qw, sc, gg = _oracle_operands(N, K, bits, g, seed=21)
    for M in (1, 2, 3, 4):
        A_t = synth.activation(M, K, seed=100 + M, device=DEV)
        ref = O.rtn_linear(_to_np(A_t), codes, scales, gg)
        for wn, wk, sk in ((1, 1, 1), (1, 4, 1), (2, 2, 2), (4, 2, 1), (1, 8, 1), (1, 16, 1), (2, 4, 3)):
            C = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=dict(path=2, waves_n=wn, waves_k=wk, split_k=sk))
            torch.cuda.synchronize()
            H.assert_linear_close(_to_np(C), ref, f"dot2 bits={bits} g={g} M={M} cfg={(wn, wk, sk)}")
    with pytest.raises(rtn.RtnError):
        rtn.rtn_linear(synth.activation(5, K, seed=1, device=DEV), qw, sc, bits, g, cfg=dict(path=2))


@pytest.mark.parametrize("bits,g", [(4, 128), (8, 0)])
@pytest.mark.parametrize("M", [17, 32, 33, 64, 100, 128])
def test_linear_larger_batches(rtn, bits, g, M):
    N, K = 528, 2048
    codes, scales, qw, sc, gg = _oracle_operands(N, K, bits, g, seed=4)
    A_t = synth.activation(M, K, seed=100 + M, device=DEV)
    ref = O.rtn_linear(_to_np(A_t), codes, scales, gg)
    C = rtn.rtn_linear(A_t, qw, sc, bits, g)
    torch.cuda.synchronize()
    H.assert_linear_close(_to_np(C), ref, f"bits={bits} g={g} M={M}")
    # the skinny kernel with every activation-block width, wide and K-split workgroups
    for cfg in (dict(path=1), dict(path=1, m_rows16=1, waves_n=4, waves_k=2), dict(path=1, m_rows16=2, waves_n=8, waves_k=1),
                dict(path=1, m_rows16=2, waves_n=4, waves_k=2, split_k=2), dict(path=1, m_rows16=4, waves_n=16, waves_k=1),
                dict(path=1, m_rows16=4, waves_n=8, waves_k=2, split_k=4), dict(path=1, m_rows16=4, waves_n=4, waves_k=4)):
        try:
            C = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=cfg)
        except rtn.RtnError as e:
            assert e.status == 7
            continue
        torch.cuda.synchronize()
        H.assert_linear_close(_to_np(C), ref, f"bits={bits} g={g} M={M} cfg={cfg}")


@pytest.mark.parametrize("bits,g", [(4, 128), (4, 256), (4, 512), (4, 0), (8, 128), (8, 256), (8, 0)])
@pytest.mark.parametrize("M", [5, 17, 33, 48, 64, 100, 130])
def test_linear_wide_kernel(rtn, bits, g, M):
    """The wide MFMA kernel (path 3): every register-tile shape, ragged M and N, K split across workgroups
    inside and across groups, several row blocks."""
    N, K = 528, 2560                       # 33 tile-rows: the last workgroup is partly out of range; 20 k-steps
    codes, scales, qw, sc, gg = _oracle_operands(N, K, bits, g, seed=6)
    A_t = synth.activation(M, K, seed=200 + M, device=DEV)
    ref = O.rtn_linear(_to_np(A_t), codes, scales, gg)
    ran = 0
    for mb in (2, 3, 4):
        for nbw in (1, 2, 4):
            for split in (1, 3, 7):
                cfg = dict(path=3, m_rows16=mb, n_tiles16=nbw, split_k=split)
                if mb * nbw > 8:            # register tile too large: refused, not launched
                    with pytest.raises(rtn.RtnError):
                        rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=cfg)
                    continue
                C = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=cfg)
                torch.cuda.synchronize()
                H.assert_linear_close(_to_np(C), ref, f"bits={bits} g={g} M={M} cfg={cfg}")
                ran += 1
    assert ran == 21
    for wv, mb, nbw in ((8, 4, 2), (8, 2, 4), (8, 3, 1), (16, 4, 1), (16, 2, 1), (16, 3, 1)):     # wider workgroups
        cfg = dict(path=3, waves_n=wv, m_rows16=mb, n_tiles16=nbw, split_k=2)
        C = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=cfg)
        torch.cuda.synchronize()
        H.assert_linear_close(_to_np(C), ref, f"bits={bits} g={g} M={M} cfg={cfg}")
    with pytest.raises(rtn.RtnError):
        rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=dict(path=3, waves_n=16, m_rows16=2, n_tiles16=2))
    C1 = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=dict(path=3, m_rows16=4, n_tiles16=2, split_k=3))
    C2 = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=dict(path=3, m_rows16=4, n_tiles16=2, split_k=3))
    assert torch.equal(C1, C2)
    if bits == 8:                           # group 64 does not fit the kernel's 128-column k-steps
        _, _, qw64, sc64, _ = _oracle_operands(N, K, 8, 64, seed=6)
        with pytest.raises(rtn.RtnError):
            rtn.rtn_linear(A_t, qw64, sc64, 8, 64, cfg=dict(path=3, m_rows16=2, n_tiles16=1))


@pytest.mark.parametrize("bits,g", [(4, 128), (4, 256), (4, 0), (8, 128), (8, 0)])
@pytest.mark.parametrize("M", [20, 128, 130, 300])
def test_linear_wide_kernel_128_rows(rtn, bits, g, M):
    """The wide kernel's 128-row register tile (explicit configuration only): weights scaled in fp16 before the MFMA,
    row blocks in two halves; ragged M and N, K split with uneven shares."""
    N, K = 400, 2560
    codes, scales, qw, sc, gg = _oracle_operands(N, K, bits, g, seed=9)
    A_t = synth.activation(M, K, seed=400 + M, device=DEV)
    ref = O.rtn_linear(_to_np(A_t), codes, scales, gg)
    for split in (1, 3, 4):
        cfg = dict(path=3, m_rows16=8, n_tiles16=2, waves_n=8, split_k=split)
        C = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=cfg)
        torch.cuda.synchronize()
        H.assert_linear_close(_to_np(C), ref, f"bits={bits} g={g} M={M} cfg={cfg}")
    assert torch.equal(C, rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=cfg))
    for bad in (dict(path=3, m_rows16=8, n_tiles16=1, waves_n=8), dict(path=3, m_rows16=8, n_tiles16=2, waves_n=4)):
        with pytest.raises(rtn.RtnError):
            rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=bad)


@pytest.mark.parametrize("bits,g", [(4, 128), (4, 256), (4, 0), (8, 128), (8, 0)])
@pytest.mark.parametrize("M", [3, 64, 128, 130, 300])
def test_linear_tile_kernel(rtn, bits, g, M):
    """The tile kernel (path 4): both tile heights, ragged M and N (a partly empty last tile in both directions), K
    split across workgroups (an odd number of chunks per workgroup included), weights dequantised to fp16 on the way
    into LDS."""
    N, K = 400, 2560
    codes, scales, qw, sc, gg = _oracle_operands(N, K, bits, g, seed=8)
    A_t = synth.activation(M, K, seed=300 + M, device=DEV)
    ref = O.rtn_linear(_to_np(A_t), codes, scales, gg)
    for split in (1, 2, 3, 5):              # 20 chunks of 128 columns: 20, 10, 7/7/6 (odd: the loop's two-step tail), 4
        for rows16 in (0, 4, 8):            # tile height: chosen from M, 128 rows, 256 rows
            cfg = dict(path=4, split_k=split, m_rows16=rows16)
            C = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=cfg)
            torch.cuda.synchronize()
            H.assert_linear_close(_to_np(C), ref, f"bits={bits} g={g} M={M} cfg={cfg}")
    C2 = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=dict(path=4, split_k=5))
    assert torch.equal(C, C2)


@pytest.mark.parametrize("M,N,K", [(1, 16, 128), (128, 128, 128), (200, 400, 2560), (1030, 272, 1024), (520, 4112, 384)])
def test_dense_gemm_and_dual_path(rtn, M, N, K):
    """rtn_gemm_fp16 against an fp64 product of the same fp16 operands, and the dequantise-then-GEMM path of
    Section 5 against the oracle's linear layer."""
    W_t = synth.normal_weight(N, K, 0.02, seed=N + K, device=DEV)
    A_t = synth.activation(M, K, seed=M, device=DEV)
    ref = _to_np(A_t).astype(np.float64) @ _to_np(W_t).astype(np.float64).T
    ws = torch.empty(16 << 20, dtype=torch.uint8, device=DEV)
    for workspace in (None, ws):
        C = rtn.rtn_gemm_fp16(A_t, W_t, workspace=workspace)
        torch.cuda.synchronize()
        H.assert_linear_close(_to_np(C), ref, f"dense M={M} N={N} K={K} ws={workspace is not None}")
    if K % 512 == 0:
        for bits, g in ((4, 128), (8, 0)):
            codes, scales, qw, sc, gg = _oracle_operands(N, K, bits, g, seed=3)
            want = O.rtn_linear(_to_np(A_t), codes, scales, gg)
            tmp = torch.empty(rtn.rtn_dense_weight_nbytes(N, K), dtype=torch.uint8, device=DEV)
            C = rtn.rtn_linear_dense(A_t, qw, sc, bits, g, tmp, workspace=ws)
            torch.cuda.synchronize()
            H.assert_linear_close(_to_np(C), want, f"dual path bits={bits} M={M}")
            deq = O.rtn_dequantize(codes, scales, gg).astype(np.float16)
            assert np.array_equal(_to_np(tmp).view(np.float16).reshape(N, K).view(np.uint16), deq.view(np.uint16))
            with pytest.raises(rtn.RtnError):
                rtn.rtn_linear_dense(A_t, qw, sc, bits, g, tmp[:-16], workspace=ws)


def test_linear_seeded_random_shapes_and_plans(rtn):
    """A seeded sweep of small random problems -- odd numbers of tile-rows and k-chunks, ragged M, every group size,
    the automatic plan and random explicit plans of every path -- against the oracle.  Plans the library refuses
    (status 7) are skipped; every accepted one must be right."""
    rng = np.random.default_rng(int(os.environ.get("RTN_TEST_SWEEP_SEED", "2024")))
    ran = {1: 0, 2: 0, 3: 0, 4: 0}
    for case in range(int(os.environ.get("RTN_TEST_SWEEP_CASES", "48"))):
        bits = int(rng.choice([4, 8]))
        ck = 512 if bits == 4 else 256
        K = int(rng.integers(1, 9)) * ck
        N = int(rng.integers(1, 40)) * 16
        gs = [g for g in (32, 64, 128, 256, 512, 1024, 0) if g == 0 or (K % g == 0 and (g < ck or g % ck == 0))]
        g = int(rng.choice(gs))
        M = int(rng.choice([1, 2, 3, 4, 5, 9, 16, 17, 31, 40, 64, 70, 129, 200]))
        codes, scales, qw, sc, gg = _oracle_operands(N, K, bits, g, seed=case)
        A_t = synth.activation(M, K, seed=500 + case, device=DEV)
        ref = O.rtn_linear(_to_np(A_t), codes, scales, gg)
        cfgs = [None]
        for _ in range(3):
            path = int(rng.choice([1, 1, 2, 3, 4]))
            if path == 1:
                cfgs.append(dict(path=1, prefetch=int(rng.choice([1, 2, 4])), waves_n=int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 11, 13])),
                                 waves_k=int(rng.integers(1, 9)), split_k=int(rng.integers(1, 4)),
                                 m_rows16=int(rng.choice([1, 2, 4]))))
            elif path == 2:
                cfgs.append(dict(path=2, waves_n=int(rng.choice([1, 2, 4])), waves_k=int(rng.integers(1, 5))))
            elif path == 3:
                cfgs.append(dict(path=3, waves_n=int(rng.choice([4, 8, 16])), m_rows16=int(rng.choice([2, 3, 4])),
                                 n_tiles16=int(rng.choice([1, 2, 4])), split_k=int(rng.integers(1, 5))))
            else:
                cfgs.append(dict(path=4, m_rows16=int(rng.choice([0, 4, 8])), split_k=int(rng.integers(1, 4))))
        for cfg in cfgs:
            try:
                C = rtn.rtn_linear(A_t, qw, sc, bits, g, cfg=cfg)
            except rtn.RtnError as e:
                assert cfg is not None and e.status in (6, 7), (case, cfg, e.status)
                continue
            torch.cuda.synchronize()
            H.assert_linear_close(_to_np(C), ref, f"case {case}: bits={bits} g={g} M={M} N={N} K={K} cfg={cfg}")
            ran[cfg["path"] if cfg else rtn.rtn_linear_query(M, N, K, bits, g)["path"]] += 1
    assert ran[1] >= 40 and ran[3] >= 8 and ran[4] >= 8 and ran[2] >= 1, ran


@pytest.mark.parametrize("bits,g", [(4, 128), (8, 64), (8, 0)])
def test_linear_special_cases(rtn, bits, g):
    N, K = 64, 1024
    codes, scales, qw, sc, gg = _oracle_operands(N, K, bits, g, seed=9)
    # one-hot activations select single dequantised weights: exact in fp16
    ks = [0, 1, 7, 8, 31, 32, 127, 128, 511, 512, 640, 1023]
    A = np.zeros((len(ks), K), dtype=np.float16)
    for i, k in enumerate(ks):
        A[i, k] = 1.0
    C = rtn.rtn_linear(torch.from_numpy(A).to(DEV), qw, sc, bits, g)
    want = O.rtn_dequantize(codes, scales, gg)[:, ks].T.astype(np.float16)
    assert np.array_equal(_to_np(C).view(np.uint16), want.view(np.uint16))
    # zero activations
    C = rtn.rtn_linear(torch.zeros((3, K), dtype=torch.float16, device=DEV), qw, sc, bits, g)
    assert not _to_np(C).any()
    # unit scales and small-integer activations: an integer matrix product, exact in fp32 and fp16
    rng = np.random.default_rng(2)
    qmax = (1 << (bits - 1)) - 1
    c2 = rng.integers(-qmax - 1, qmax + 1, size=(N, K)).astype(np.int8)
    if bits == 8:
        c2 = (c2 // 16).astype(np.int8)
    ones = np.ones((N, K // gg), dtype=np.float16)
    A2 = rng.integers(-1, 2, size=(4, K)).astype(np.float16)
    C = rtn.rtn_linear(torch.from_numpy(A2).to(DEV), torch.from_numpy(O.pack_gfx950(c2, bits)).to(DEV),
                       torch.from_numpy(ones).to(DEV), bits, g)
    want = (A2.astype(np.int64) @ c2.astype(np.int64).T)
    assert np.abs(want).max() < 2048
    assert np.array_equal(_to_np(C).astype(np.int64), want)


def test_linear_is_deterministic(rtn):
    N, K = 512, 4096
    codes, scales, qw, sc, gg = _oracle_operands(N, K, 4, 128, seed=12)
    for M, cfg in ((1, dict(waves_k=4, split_k=2)), (16, dict(waves_n=4, waves_k=1, split_k=4)), (8, dict(waves_n=4, waves_k=2, split_k=2, prefetch=2)), (3, None)):
        A_t = synth.activation(M, K, seed=1, device=DEV)
        outs = [rtn.rtn_linear(A_t, qw, sc, 4, 128, cfg=cfg).clone() for _ in range(5)]
        torch.cuda.synchronize()
        for o in outs[1:]:
            assert torch.equal(o, outs[0])


@pytest.mark.parametrize("M,cfg", [(1, dict(waves_k=4, split_k=2)), (8, dict(waves_n=4, waves_k=2, split_k=4)),
                                   (16, dict(waves_n=4, waves_k=1, split_k=8)), (4, None)])
def test_linear_split_k_graph_replays_match_direct_calls(rtn, M, cfg):
    """A K-split call recorded into a HIP graph: every replay, with direct calls and fresh activations in between,
    gives the bits of the direct call (the split partial sums are added in a fixed order on both routes)."""
    N, K = 1024, 14336
    codes, scales, qw, sc, gg = _oracle_operands(N, K, 4, 128, seed=31)
    nws = max(256, rtn._lib.rtn_workspace_nbytes(M, N, K, 4, 128))
    A_static = synth.activation(M, K, seed=100, device=DEV)
    ws_g = torch.empty(nws, dtype=torch.uint8, device=DEV)
    out_g = torch.empty((M, N), dtype=torch.float16, device=DEV)
    rtn.rtn_linear(A_static, qw, sc, 4, 128, cfg=cfg)      # a direct call before the recording
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rtn.rtn_linear(A_static, qw, sc, 4, 128, out=out_g, workspace=ws_g, cfg=cfg)
    for rep in range(4):
        A_new = synth.activation(M, K, seed=101 + rep, device=DEV)
        A_static.copy_(A_new)
        want = rtn.rtn_linear(A_new, qw, sc, 4, 128, cfg=cfg)
        torch.cuda.synchronize()
        graph.replay()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, want), (M, cfg, rep)
    H.assert_linear_close(_to_np(out_g), O.rtn_linear(_to_np(A_static), codes, scales, gg), f"graph replay M={M}")


def test_linear_automatic_split_shrinks_to_the_workspace_passed(rtn):
    """From 17 rows the plan's K split is a preference: with a workspace too small for it (here none of the partial
    sums fit) the call still succeeds, unsplit, and matches the oracle like the call with the full workspace."""
    N, K, M = 4096, 4096, 64
    codes, scales, qw, sc, gg = _oracle_operands(N, K, 4, 128, seed=41)
    q = rtn.rtn_linear_query(M, N, K, 4, 128)
    assert q["path"] == 3 and q["split_k"] > 1, q
    A_t = synth.activation(M, K, seed=3, device=DEV)
    ref = O.rtn_linear(_to_np(A_t), codes, scales, gg)
    full = rtn.rtn_linear(A_t, qw, sc, 4, 128)
    small = rtn.rtn_linear(A_t, qw, sc, 4, 128, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    torch.cuda.synchronize()
    H.assert_linear_close(_to_np(full), ref, "full workspace")
    H.assert_linear_close(_to_np(small), ref, "256-byte workspace")
    with pytest.raises(rtn.RtnError):       # an explicit split is not negotiable
        rtn.rtn_linear(A_t, qw, sc, 4, 128, workspace=torch.empty(256, dtype=torch.uint8, device=DEV),
                       cfg=dict(path=3, split_k=q["split_k"]))


@pytest.mark.parametrize("M", [1024, 2048])
def test_linear_tile_kernel_in_two_launches(rtn, M):
    """The 405B-shaped qkv matrix at 1024 and 2048 rows: 72 column blocks make 288 / 576 tall tiles, a round and an
    eighth (or a quarter) of 256, so rtn_linear runs the first 768 / 1792 rows as full rounds and the last 256 rows
    as a launch of their own with K split.  Rows on both sides of the seam and a stripe of columns against the oracle."""
    K, N = synth.LLAMA_405B["qkv"]
    W_t = synth.normal_weight(N, K, 0.01, seed=77, device=DEV)
    qw, sc = rtn.rtn_quantize(W_t, 4, 128)
    del W_t
    A_t = synth.activation(M, K, seed=M, device=DEV)
    assert rtn.rtn_linear_query(M, N, K, 4, 128)["path"] == 4
    C = rtn.rtn_linear(A_t, qw, sc, 4, 128)
    torch.cuda.synchronize()
    rng = np.random.default_rng(M)
    cols = np.unique(np.concatenate([np.arange(0, 16), np.arange(N - 16, N), rng.integers(0, N, 64)]))
    rows = np.unique(np.concatenate([np.arange(0, 4), np.arange(M - 260, M - 252), np.arange(M - 4, M), rng.integers(0, M, 48)]))
    codes = _to_np(rtn.rtn_unpack(qw, N, K, 4))[cols]
    ref = O.rtn_linear(_to_np(A_t)[rows], codes, _to_np(sc)[cols], 128)
    H.assert_linear_close(_to_np(C)[np.ix_(rows, cols)], ref, f"two launches M={M}")


def test_linear_automatic_plans_on_large_random_shapes(rtn):
    """What rtn_linear chooses by itself from 48 rows up on matrices large enough for every branch of its plan (wide
    kernel with 1-8 K splits, its 128-row variant, tile kernel of either height with and without splits), with the
    workspace rtn_workspace_nbytes asks for: a stripe of output columns (first and last tile-row, 96 random ones)
    against the oracle on the unpacked codes."""
    rng = np.random.default_rng(5)
    seen = set()
    for case in range(14):
        bits = int(rng.choice([4, 4, 8]))
        g = 128 if bits == 4 else int(rng.choice([0, 128]))
        K = int(rng.choice([4096, 8192, 14336, 16384, 28672]))
        N = int(rng.integers(8, 90)) * 256 + int(rng.choice([0, 16, 128]))
        M = int(rng.choice([48, 64, 96, 128, 129, 160, 192, 256, 300, 384, 512, 640, 768, 1000, 1024]))
        W_t = synth.normal_weight(N, K, 0.02, seed=case, device=DEV)
        qw, sc = rtn.rtn_quantize(W_t, bits, g)
        del W_t
        A_t = synth.activation(M, K, seed=case + 7, device=DEV)
        q = rtn.rtn_linear_query(M, N, K, bits, g)
        need = M * N * 4 * q["split_k"] if q["split_k"] > 1 else 0
        assert need <= rtn.rtn_workspace_nbytes(M, N, K, bits, g)
        C = rtn.rtn_linear(A_t, qw, sc, bits, g)
        torch.cuda.synchronize()
        sel = np.unique(np.concatenate([np.arange(0, 16), np.arange(N - 16, N), rng.integers(0, N, 96)]))
        codes = _to_np(rtn.rtn_unpack(qw, N, K, bits))[sel]
        ref = O.rtn_linear(_to_np(A_t), codes, _to_np(sc)[sel], K if g == 0 else g)
        H.assert_linear_close(_to_np(C)[:, sel], ref, f"case {case} bits={bits} g={g} M={M} N={N} K={K} plan={q}")
        seen.add((q["path"], q["m_rows16"], q["split_k"] > 1))
        del qw, sc, A_t, C
    assert {p for p, _, _ in seen} == {3, 4} and any(r == 8 for _, r, _ in seen) and any(s for _, _, s in seen), seen


def test_linear_automatic_plans_at_small_batches_on_irregular_shapes(rtn):
    """What rtn_linear chooses by itself at 1-16 rows on shapes outside its measured plan table (the held-out files of
    the tuning folder: tile-row counts such as 2153 or 2763, for which the plan takes workgroups of 9, 11, 13 ... wavefronts
    and K splits): a stripe of output columns (first and last tile-row, 96 random ones) against the oracle on the
    unpacked codes, and run-to-run bit reproducibility."""
    tuning = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2505_15909_amd", "tuning")
    shapes = []
    for name in ("shapes_heldout.txt", "shapes_heldout2.txt"):
        for line in open(os.path.join(tuning, name)):
            _, K, N = line.split()
            shapes.append((int(K), int(N)))
    rng = np.random.default_rng(11)
    widths = set()
    ws = torch.empty(16 << 20, dtype=torch.uint8, device=DEV)
    for case, (K, N) in enumerate(shapes):
        bits = 4 if case % 3 else 8
        if K % (512 if bits == 4 else 256):
            bits = 8
        g = 128 if bits == 4 else 0
        W_t = synth.normal_weight(N, K, 0.02, seed=case, device=DEV)
        qw, sc = rtn.rtn_quantize(W_t, bits, g)
        del W_t
        sel = np.unique(np.concatenate([np.arange(0, 16), np.arange(N - 16, N), rng.integers(0, N, 96)]))
        codes = _to_np(rtn.rtn_unpack(qw, N, K, bits))[sel]
        scales = _to_np(sc)[sel]
        for M in (1, 6, 16):
            A_t = synth.activation(M, K, seed=case + 7 * M, device=DEV)
            q = rtn.rtn_linear_query(M, N, K, bits, g)
            assert q["path"] == 1
            widths.add(q["waves_n"])
            C = rtn.rtn_linear(A_t, qw, sc, bits, g, workspace=ws)
            C2 = rtn.rtn_linear(A_t, qw, sc, bits, g, workspace=ws)
            torch.cuda.synchronize()
            assert torch.equal(C, C2)
            ref = O.rtn_linear(_to_np(A_t), codes, scales, K if g == 0 else g)
            H.assert_linear_close(_to_np(C)[:, sel], ref, f"case {case} bits={bits} M={M} N={N} K={K} plan={q}")
        del qw, sc
    assert any(w not in (1, 2, 4, 8, 16) for w in widths), widths      # the odd widths are exercised


# ----------------------------------------------------------------------------------------
# the paper-shaped configurations at full size: the 8B-shaped ones are compared against the oracle in full; for the
# larger ones the oracle checks a stripe of 16-row tiles (rows of the weight matrix are independent); the GPU always
# runs the full shape in its default configuration
# ----------------------------------------------------------------------------------------
FULL = [
    # name, dist, bits, g, modules, Ms, stripe tiles
    # (the 8B-shaped configurations are compared in full: every tile-row of every matrix)
    ("single_4096", "normal02", 4, 128, {"o": (4096, 4096)}, (1,), 1 << 30),
    ("llama8b_w4", "normal02", 4, 128, synth.LLAMA_8B, (1, 2, 4, 8, 16), 1 << 30),
    ("llama8b_w8", "normal02", 8, 0, synth.LLAMA_8B, (1, 4, 16, 64), 1 << 30),
    ("llama70b_w4", "heavy", 4, 128, synth.LLAMA_70B, (1, 8, 32, 64, 128, 256, 512, 768), 12),
]


@pytest.mark.parametrize("case", FULL, ids=lambda c: c[0])
def test_full_size_quantize_and_linear(rtn, case):
    name, dist, bits, g, modules, Ms, n_tiles = case
    for idx, (mod, (K, N)) in enumerate(modules.items()):
        W_t = H.make_weight(dist, N, K, seed=idx, device=DEV)
        qw, sc = rtn.rtn_quantize(W_t, bits, g)
        tiles = H.pick_row_tiles(N, n_tiles, seed=idx)
        rows = H.tile_rows(tiles, N)
        Wr = _to_np(W_t[torch.from_numpy(rows).to(DEV)])
        gg = K if g <= 0 else g
        codes, scales = O.rtn_quantize(Wr, bits, gg)
        assert np.array_equal(_to_np(sc)[rows].view(np.uint16), scales.view(np.uint16)), (name, mod)
        assert np.array_equal(H.packed_rows_image(_to_np(qw), tiles, K, bits), O.pack_gfx950(codes, bits)), (name, mod)
        del W_t
        for M in Ms:
            A_t = synth.activation(M, K, seed=100 + M, device=DEV)
            C = rtn.rtn_linear(A_t, qw, sc, bits, g)
            torch.cuda.synchronize()
            ref = O.rtn_linear(_to_np(A_t), codes, scales, gg)
            allow = "llama70b_down" if (name, mod) == ("llama70b_w4", "down") else None
            fro, mx = H.assert_linear_close(_to_np(C)[:, rows], ref, f"{name} {mod} M={M}", allow=allow)
            print(f"{name} {mod} M={M}: {len(rows)} of {N} output columns compared, rel Frobenius {fro:.2e}, max abs {mx:.2e}, "
                  f"|C_ref| up to {float(np.max(np.abs(ref))):.1f}{' (fp16-output allowance)' if allow and float(np.max(np.abs(ref))) >= 16 else ''}", flush=True)


@pytest.mark.parametrize("M", [512, 1500])
def test_full_size_large_batch_fused_and_dual_path(rtn, M):
    """Prefill-sized inputs on the full 8B-shaped gate_up and down matrices (Section 5): the fused path (tile kernel
    where it has a full round of output tiles, wide kernel otherwise) and the dequantise-then-GEMM path, both against
    the oracle on a stripe of 16-row tiles."""
    ws = torch.empty(256 << 20, dtype=torch.uint8, device=DEV)
    for idx, mod in enumerate(("gate_up", "down")):
        K, N = synth.LLAMA_8B[mod]
        W_t = synth.normal_weight(N, K, 0.02, seed=idx, device=DEV)
        qw, sc = rtn.rtn_quantize(W_t, 4, 128)
        tiles = H.pick_row_tiles(N, 12, seed=idx)
        rows = H.tile_rows(tiles, N)
        codes, scales = O.rtn_quantize(_to_np(W_t[torch.from_numpy(rows).to(DEV)]), 4, 128)
        del W_t
        A_t = synth.activation(M, K, seed=400 + M, device=DEV)
        ref = O.rtn_linear(_to_np(A_t), codes, scales, 128)
        sel = torch.from_numpy(rows).to(DEV)
        C = rtn.rtn_linear(A_t, qw, sc, 4, 128, workspace=ws)
        torch.cuda.synchronize()
        H.assert_linear_close(_to_np(C[:, sel]), ref, f"{mod} M={M} fused path {rtn.rtn_linear_query(M, N, K, 4, 128)['path']}")
        tmp = torch.empty(rtn.rtn_dense_weight_nbytes(N, K), dtype=torch.uint8, device=DEV)
        C2 = rtn.rtn_linear_dense(A_t, qw, sc, 4, 128, tmp, workspace=ws)
        torch.cuda.synchronize()
        H.assert_linear_close(_to_np(C2[:, sel]), ref, f"{mod} M={M} dual path")
        del tmp
        print(f"{mod} M={M} fused and dual ok", flush=True)


def test_full_size_405b_selective_layer(rtn):
    """The 405B-shaped selective-precision decoder layer at full width (qkv and gate_up int4 g128, o and
    down int8 per-channel), quantised on the GPU and run through rtn_layer_forward at M = 1, 16, 128;
    the oracle checks a stripe of 16-row tiles of every module (rows are independent)."""
    plan = {"qkv": (4, 128), "o": (8, 0), "gate_up": (4, 128), "down": (8, 0)}
    packed, stripes = {}, {}
    for idx, (mod, (K, N)) in enumerate(synth.LLAMA_405B.items()):
        bits, g = plan[mod]
        W_t = synth.normal_weight(N, K, 0.01, seed=idx, device=DEV)
        qw, sc = rtn.rtn_quantize(W_t, bits, g)
        tiles = H.pick_row_tiles(N, 6, seed=idx)
        rows = H.tile_rows(tiles, N)
        Wr = _to_np(W_t[torch.from_numpy(rows).to(DEV)])
        del W_t
        gg = K if g <= 0 else g
        codes, scales = O.rtn_quantize(Wr, bits, gg)
        assert np.array_equal(_to_np(sc[torch.from_numpy(rows).to(DEV)]).view(np.uint16), scales.view(np.uint16)), mod
        per_tile_row = 16 * K * bits // 8
        got = np.concatenate([_to_np(qw[t * per_tile_row:(t + 1) * per_tile_row]) for t in tiles])
        assert np.array_equal(got, O.pack_gfx950(codes, bits)), mod
        packed[mod] = (qw, sc, bits, g, K, N)
        stripes[mod] = (rows, codes, scales, gg)
        print(f"405b {mod} quantise ok", flush=True)
    for M in (1, 16, 128):
        mods = []
        for idx, (mod, (qw, sc, bits, g, K, N)) in enumerate(packed.items()):
            mods.append(dict(A=synth.activation(M, K, seed=300 + idx, device=DEV), qweight=qw, scales=sc, bits=bits,
                             group_size=g, C=torch.empty((M, N), dtype=torch.float16, device=DEV)))
        rtn.rtn_layer_forward(mods)
        torch.cuda.synchronize()
        for m, mod in zip(mods, packed):
            rows, codes, scales, gg = stripes[mod]
            ref = O.rtn_linear(_to_np(m["A"]), codes, scales, gg)
            H.assert_linear_close(_to_np(m["C"][:, torch.from_numpy(rows).to(DEV)]), ref, f"405b {mod} M={M}")
        print(f"405b layer M={M} ok", flush=True)


def test_grouped_forward_expert_modules(rtn):
    """rtn_grouped_forward on independent expert-like modules (per-expert precision in mixture-of-experts models, Section 6): more
    modules of one class than a grouped launch holds, several classes (int4 g128, int4 g32, int8 per-channel),
    different shapes and row counts per module, and modules the grouped launch cannot merge (more than 16 rows, a
    long K that splits across workgroups); every output against the oracle."""
    rng = np.random.default_rng(77)
    specs = []
    for e in range(20):                                                   # one class, > 16 members, ragged M
        specs.append((int(rng.integers(1, 8)), 768, 2048, 4, 128))
    for e in range(3):
        specs.append((int(rng.integers(1, 5)), 512, 1024, 4, 32))
    for e in range(3):
        specs.append((int(rng.integers(1, 17)), 1024, 1536, 8, 0))
    specs.append((16, 640, 4096, 4, 128))                                 # 17 staged rows: several stages
    specs.append((40, 512, 1024, 4, 128))                                 # wide kernel
    specs.append((9, 256, 14336, 4, 128))                                 # long K: split across workgroups
    mods, refs = [], []
    for idx, (M, N, K, bits, g) in enumerate(specs):
        W = _to_np(synth.normal_weight(N, K, 0.02, seed=900 + idx, device=DEV))
        gg = K if g <= 0 else g
        codes, scales = O.rtn_quantize(W, bits, gg)
        A_t = synth.activation(M, K, seed=950 + idx, device=DEV)
        mods.append(dict(A=A_t, qweight=torch.from_numpy(O.pack_gfx950(codes, bits)).to(DEV),
                         scales=torch.from_numpy(scales).to(DEV), bits=bits, group_size=g,
                         C=torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)))
        refs.append(O.rtn_linear(_to_np(A_t), codes, scales, gg))
    rtn.rtn_grouped_forward(mods)
    torch.cuda.synchronize()
    for i, (m, ref) in enumerate(zip(mods, refs)):
        H.assert_linear_close(_to_np(m["C"]), ref, f"grouped module {i} {specs[i]}")
    # a single module and a pair behave like the plain call
    for lo, hi in ((0, 1), (20, 22)):
        for m in mods[lo:hi]:
            m["C"].fill_(float("nan"))
        rtn.rtn_grouped_forward(mods[lo:hi])
        torch.cuda.synchronize()
        for i in range(lo, hi):
            H.assert_linear_close(_to_np(mods[i]["C"]), refs[i], f"grouped subset module {i}")


def test_selective_precision_layer(rtn):
    """Mixed 4-/8-bit decoder layer through rtn_layer_forward (Section 4.3), 405B-shaped at 1/8 width
    here; the full-width layer is exercised by the benchmark."""
    shapes = {"qkv": (2048, 2304, 4, 128), "o": (2048, 2048, 8, 0), "gate_up": (2048, 13312, 4, 128),
              "down": (6656 - 6656 % 512, 2048, 8, 0)}
    for M in (1, 16, 128):
        mods, refs = [], []
        for idx, (mod, (K, N, bits, g)) in enumerate(shapes.items()):
            W = _to_np(synth.normal_weight(N, K, 0.01, seed=idx, device=DEV))
            gg = K if g <= 0 else g
            codes, scales = O.rtn_quantize(W, bits, gg)
            A_t = synth.activation(M, K, seed=200 + idx, device=DEV)
            mods.append(dict(A=A_t, qweight=torch.from_numpy(O.pack_gfx950(codes, bits)).to(DEV),
                             scales=torch.from_numpy(scales).to(DEV), bits=bits, group_size=g,
                             C=torch.empty((M, N), dtype=torch.float16, device=DEV)))
            refs.append(O.rtn_linear(_to_np(A_t), codes, scales, gg))
        rtn.rtn_layer_forward(mods)
        torch.cuda.synchronize()
        for m, ref, mod in zip(mods, refs, shapes):
            H.assert_linear_close(_to_np(m["C"]), ref, f"layer {mod} M={M}")


# ----------------------------------------------------------------------------------------
# asymmetric variant (integer zero points; the remark after Eq. 1 in Section 2.2)
# ----------------------------------------------------------------------------------------
def _asym_both(rtn, W_t, bits, g):
    qw, sc, zp = rtn.rtn_quantize_asym(W_t, bits, g)
    torch.cuda.synchronize()
    W = _to_np(W_t)
    gg = W.shape[1] if g <= 0 else g
    codes, scales, zeros = O.rtn_quantize_asym(W, bits, gg)
    return qw, sc, zp, codes, scales, zeros, gg


def _assert_asym_equal(rtn, qw, sc, zp, codes, scales, zeros, bits):
    N, K = codes.shape
    assert np.array_equal(_to_np(sc).view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(_to_np(zp).astype(np.float64), zeros.astype(np.float64))
    assert np.array_equal(_to_np(qw), O.pack_gfx950(codes, bits))
    assert np.array_equal(_to_np(rtn.rtn_unpack(qw, N, K, bits)), codes)


@pytest.mark.parametrize("bits,g", [(4, 32), (4, 64), (4, 128), (4, 256), (4, 1024), (4, 0), (8, 32), (8, 64), (8, 128),
                                     (8, 512), (8, 0)])
@pytest.mark.parametrize("N,K,shift", [(80, 2048, 0.0), (272, 3072, 0.013), (16, 14336, -0.02)])
def test_asym_quantize_bit_exact(rtn, bits, g, N, K, shift):
    if g > K or (g > 0 and K % g):
        pytest.skip("group does not divide K")
    W_t = (synth.normal_weight(N, K, 0.02, seed=N + K + bits, device=DEV).float() + shift).half()
    qw, sc, zp, codes, scales, zeros, gg = _asym_both(rtn, W_t, bits, g)
    _assert_asym_equal(rtn, qw, sc, zp, codes, scales, zeros, bits)
    # dequantise: fp16 of the exact product S (q + Z)
    deq = O.rtn_dequantize_asym(codes, scales, zeros, gg).astype(np.float16)
    got = _to_np(rtn.rtn_dequantize_asym(qw, sc, zp, N, K, bits, g))
    assert np.array_equal(got.view(np.uint16), deq.view(np.uint16))


@pytest.mark.parametrize("bits,g", [(4, 128), (8, 64), (4, 32), (8, 32), (4, 512)])
def test_asym_quantize_adversarial(rtn, bits, g):
    """One-sided groups, all-zero groups, constant groups, exact ties with odd and even shifts, subnormal scales,
    the largest fp16 range, and a range whose width does not fit fp32 (the scale is still the exact quotient rounded once)."""
    N, K = 64, 1024
    rng = np.random.default_rng(23)
    W = (rng.standard_normal((N, K)) * 0.02 + 0.004).astype(np.float16)
    levels = (1 << bits) - 1
    W[0, :g] = np.abs(W[0, :g])
    W[1, :g] = -np.abs(W[1, :g])
    W[2, :g] = 0.0
    W[3, :g] = -0.0
    W[4, :g] = np.float16(0.3)
    W[5, :g] = np.float16(-0.3)
    W[6, 0], W[6, 1] = 65504.0, -65504.0
    W[7, :g] = (rng.integers(-3, 9, size=g) * 2.0 ** -24).astype(np.float16)        # scale of 0 or 1 ulp
    for r in range(8, 24):                       # ties: range [-a, levels - a] in units of s, halves in between
        a = int(rng.integers(0, levels + 1))
        s = 2.0 ** -int(rng.integers(4, 9))
        W[r, :g] = (rng.integers(-2 * a, 2 * (levels - a) + 1, size=g) * 0.5 * s).astype(np.float16)
        W[r, 0], W[r, 1] = -a * s, (levels - a) * s
    for r, a in zip(range(24, 36), (10, 11, 17, 180, 190, 191, 300, 317, 500, 700, 1000, 1023)):   # subnormal scales
        W[r, :g] = (rng.integers(-a // 3, a + 1, size=g) * 2.0 ** -24).astype(np.float16)
        W[r, 0] = np.float16(a * 2.0 ** -24)
        W[r, 1] = np.float16(-(a // 3) * 2.0 ** -24)
    hb, ha = {4: (16008, 33279), 8: (17014, 33217)}[bits]          # an fp32 intermediate would move the scale: the kernel must round the exact quotient once
    W[36, :g] = 0
    W[36, 0] = np.array([hb], dtype=np.uint16).view(np.float16)[0]
    W[36, 1] = np.array([ha], dtype=np.uint16).view(np.float16)[0]
    W[37, :g] = np.float16(1.0) + np.float16(2.0 ** -10) * (np.arange(g) % 200)   # far from zero, narrow spread
    W_t = torch.from_numpy(W).to(DEV)
    qw, sc, zp, codes, scales, zeros, _ = _asym_both(rtn, W_t, bits, g)
    _assert_asym_equal(rtn, qw, sc, zp, codes, scales, zeros, bits)
    qw, sc, zp, codes, scales, zeros, _ = _asym_both(rtn, W_t, bits, 0)
    _assert_asym_equal(rtn, qw, sc, zp, codes, scales, zeros, bits)


@pytest.mark.parametrize("bits,g", [(4, 32), (4, 128), (4, 512), (4, 0), (8, 32), (8, 128), (8, 0)])
def test_asym_linear(rtn, bits, g):
    """rtn_linear_asym against the oracle: small batches (one launch), more than 16 rows (the wide kernel's zero-point
    instantiations where the group size allows, 16-row blocks of the small-batch kernel otherwise), a long K that
    splits across workgroups, a ragged N; weights shifted away from zero so that the zero points matter."""
    for (M, N, K) in ((1, 272, 2048), (3, 80, 4096), (16, 64, 3072), (40, 48, 2048), (7, 32, 14336), (17, 272, 1024),
                      (130, 80, 3072), (64, 528, 2048)):
        W = _to_np((synth.normal_weight(N, K, 0.02, seed=M + N + bits, device=DEV).float() + 0.015).half())
        gg = K if g <= 0 else g
        codes, scales, zeros = O.rtn_quantize_asym(W, bits, gg)
        A_t = synth.activation(M, K, seed=77 + M, device=DEV)
        qw = torch.from_numpy(O.pack_gfx950(codes, bits)).to(DEV)
        sc = torch.from_numpy(scales).to(DEV)
        zp = torch.from_numpy(zeros.astype(np.float16)).to(DEV)
        C = rtn.rtn_linear_asym(A_t, qw, sc, zp, bits, g)
        torch.cuda.synchronize()
        ref = O.rtn_linear_asym(_to_np(A_t), codes, scales, zeros, gg)
        H.assert_linear_close(_to_np(C), ref, f"asym int{bits} g={g} M={M} N={N} K={K}")
        if M > 16:      # a workspace too small for the plan's K split: fewer splits, same result within tolerance
            C = rtn.rtn_linear_asym(A_t, qw, sc, zp, bits, g, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
            torch.cuda.synchronize()
            H.assert_linear_close(_to_np(C), ref, f"asym, 256-byte workspace, int{bits} g={g} M={M} N={N} K={K}")
        # the zero points are really used: the symmetric formula on the same codes is outside the parity tolerance
        assert np.linalg.norm(O.rtn_linear(_to_np(A_t), codes, scales, gg) - ref) > 4e-3 * np.linalg.norm(ref)
    # large M: dequantise once, then the dense GEMM
    M, N, K = 300, 256, 1024
    W_t = (synth.normal_weight(N, K, 0.02, seed=5, device=DEV).float() + 0.01).half()
    qw, sc, zp, codes, scales, zeros, gg = _asym_both(rtn, W_t, bits, g)
    A_t = synth.activation(M, K, seed=9, device=DEV)
    Wd = rtn.rtn_dequantize_asym(qw, sc, zp, N, K, bits, g)
    C = rtn.rtn_gemm_fp16(A_t, Wd)
    torch.cuda.synchronize()
    ref = _to_np(A_t).astype(np.float64) @ O.rtn_dequantize_asym(codes, scales, zeros, gg).astype(np.float16).astype(np.float64).T
    H.assert_linear_close(_to_np(C), ref, f"asym dual path int{bits} g={g}")
