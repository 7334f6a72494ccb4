"""Shared helpers of the GPU parity tests: workload definitions and comparison metrics."""
from __future__ import annotations

import numpy as np
import torch

from oracle import rtn_oracle as O
from paper_2505_15909_amd import synth

REL_FRO_TOL = 2e-3       # relative Frobenius error bound of the linear layer
MAX_ABS_TOL = 1e-2       # max abs error bound, taken literally ...
HALF_ULP_REL = 2.0 ** -11  # ... except in the cases listed below, which get one fp16 rounding of the result on top

# The only cases where the literal max-abs bound cannot hold: outputs so large that the fp16 output format itself uses
# up the bound.  For |C| in [16, 32) the half-ulp is 7.8e-3, which leaves 2.2e-3 for everything else (measured: up to
# 1.08e-2 in total at |C| = 30 on the path that rounds each dequantised weight to fp16 first); from |C| = 32 the half-ulp
# is 1.6e-2 and a correctly rounded result already misses 1e-2.  Keyed by the `allow` tag the test passes; each entry
# states where such outputs come from.  Everything else, and the listed cases while |C| stays below 16, is held to
# max|dC| <= 1e-2.
FP16_OUTPUT_ALLOWANCE = {
    "llama70b_down": "70B-shaped down projection, K = 28672, heavy-tailed weights with 1 % of input columns x10: "
                     "|C| reaches 23-35 depending on the batch",
}


def linear_errors(C_gpu: np.ndarray, C_ref: np.ndarray):
    d = C_gpu.astype(np.float64) - C_ref
    fro = float(np.linalg.norm(d) / max(np.linalg.norm(C_ref), 1e-300))
    max_abs = float(np.max(np.abs(d))) if d.size else 0.0
    excess = float(np.max(np.abs(d) - (MAX_ABS_TOL + HALF_ULP_REL * np.abs(C_ref)))) if d.size else -1.0
    return fro, max_abs, excess


def assert_linear_close(C_gpu, C_ref, what="", allow=None):
    """rel Frobenius <= 2e-3 and max abs <= 1e-2 (literal).  allow: a key of FP16_OUTPUT_ALLOWANCE for the listed cases
    whose outputs reach 16 and more in magnitude; where they do, the case is held to 1e-2 + 2^-11 |C_ref| instead."""
    fro, max_abs, excess = linear_errors(C_gpu, C_ref)
    assert fro <= REL_FRO_TOL, f"{what}: rel Frobenius {fro:.3e} > {REL_FRO_TOL}"
    c_max = float(np.max(np.abs(C_ref))) if C_ref.size else 0.0
    if allow is not None:
        assert allow in FP16_OUTPUT_ALLOWANCE, allow
    if allow is None or c_max < 16.0:      # a listed case still gets the literal bound while its outputs stay below 16
        assert max_abs <= MAX_ABS_TOL, f"{what}: max abs {max_abs:.3e} > 1e-2 (|C_ref| up to {c_max:.2f})"
    else:
        assert excess <= 0.0, f"{what}: max abs {max_abs:.3e} exceeds 1e-2 + 2^-11 |C| (|C_ref| up to {c_max:.2f})"
    return fro, max_abs


def tile_rows(row_tiles, N):
    """Row indices of the given 16-row tiles."""
    rows = np.concatenate([np.arange(t * 16, t * 16 + 16) for t in row_tiles])
    assert rows.max() < N
    return rows


def packed_rows_image(packed: np.ndarray, row_tiles, K: int, bits: int) -> np.ndarray:
    """Bytes of the given row tiles from a full packed image (tiles are row-tile-major)."""
    per_tile_row = 16 * K * bits // 8
    return np.concatenate([packed[t * per_tile_row:(t + 1) * per_tile_row] for t in row_tiles])


def pick_row_tiles(N: int, count: int, seed: int):
    NT = N // 16
    if NT <= count:
        return np.arange(NT)
    rng = np.random.default_rng(seed)
    picks = set(rng.choice(NT, size=count - 2, replace=False).tolist())
    picks.update([0, NT - 1])                                   # always the first and last tile row
    return np.array(sorted(picks))


def make_weight(cfg_dist: str, N: int, K: int, seed: int, device):
    if cfg_dist == "normal02":
        return synth.normal_weight(N, K, 0.02, seed, device)
    if cfg_dist == "normal01":
        return synth.normal_weight(N, K, 0.01, seed, device)
    if cfg_dist == "heavy":
        return synth.heavy_tail_weight(N, K, 0.02, seed, device)
    raise ValueError(cfg_dist)
