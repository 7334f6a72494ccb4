"""rtn_linear_noalloc (the entry point for callers that cannot allocate: split-K partial sums in the library's fixed
device array) against rtn_linear with a caller's workspace, through the C ABI: same plan, so the outputs must be
bit-identical.  Two calls in a row, the second on a smaller problem, so stale partial sums of the first call would
show; plans with a K split across workgroups are forced by the shapes chosen (long K, few output columns)."""
import ctypes as C

import pytest
import torch

pytestmark = pytest.mark.gpu


def _run_pair(rtn, synth, M, N, K, bits, g, seed):
    dev = "cuda:0"
    W = synth.normal_weight(N, K, 0.02, seed, dev)
    A = synth.activation(M, K, 100 + seed, dev)
    qw, sc = rtn.rtn_quantize(W, bits, g)
    ws = torch.empty(max(256, rtn.rtn_workspace_nbytes(M, N, K, bits, g)), dtype=torch.uint8, device=dev)
    ref = torch.empty((M, N), dtype=torch.float16, device=dev)
    got = torch.full((M, N), float("nan"), dtype=torch.float16, device=dev)
    lib = rtn._lib
    st = torch.cuda.current_stream().cuda_stream
    assert lib.rtn_linear(A.data_ptr(), M, qw.data_ptr(), sc.data_ptr(), N, K, bits, g, ref.data_ptr(), ws.data_ptr(),
                          ws.numel(), st) == 0
    assert lib.rtn_linear_noalloc(A.data_ptr(), M, qw.data_ptr(), sc.data_ptr(), N, K, bits, g, got.data_ptr(), st) == 0
    torch.cuda.synchronize()
    plan = rtn.rtn_linear_query(M, N, K, bits, g)
    return torch.equal(ref, got), plan


def _first_that_splits(rtn, candidates):
    for M, N, K, bits, g in candidates:
        if rtn.rtn_linear_query(M, N, K, bits, g)["split_k"] > 1:
            return M, N, K, bits, g
    pytest.fail(f"none of {candidates} has an automatic plan with a K split across workgroups: update the list")


def test_noalloc_matches_rtn_linear_on_two_calls_in_a_row(rtn):
    from paper_2505_15909_amd import synth
    # first call: a long-K projection at 16 rows whose automatic plan splits K across workgroups (partials in scratch)
    big = _first_that_splits(rtn, [(16, 4096, 14336, 4, 128), (16, 8192, 28672, 4, 128), (16, 16384, 53248, 4, 128)])
    same, _ = _run_pair(rtn, synth, *big, seed=1)
    assert same
    # second call, smaller (fewer rows, fewer output columns), also with a K split: stale partials of the first call
    # would show
    small = _first_that_splits(rtn, [(8, 4096, 14336, 4, 128), (4, 2048, 28672, 4, 128), (8, 4096, 14336, 8, 0),
                                     (8, 2048, 53248, 4, 128)])
    assert small[0] * small[1] < big[0] * big[1]
    same, _ = _run_pair(rtn, synth, *small, seed=2)
    assert same
    # and one without a K split, and an 8-bit one above 16 rows (wide kernel)
    same, _ = _run_pair(rtn, synth, 1, 2048, 2048, 4, 128, seed=3)
    assert same
    same, _ = _run_pair(rtn, synth, 40, 1024, 8192, 8, 0, seed=4)
    assert same


def test_noalloc_rejects_what_the_fixed_array_cannot_hold(rtn):
    lib = rtn._lib
    t = torch.empty(4096, dtype=torch.uint8, device="cuda:0")
    p = t.data_ptr()
    # 256 rows on the 405B-shaped down projection: the plan's partial sums exceed 16 MiB
    assert rtn.rtn_workspace_nbytes(256, 16384, 53248, 4, 128) > 16 << 20
    assert lib.rtn_linear_noalloc(p, 256, p, p, 16384, 53248, 4, 128, p, None) == 6
    assert lib.rtn_linear_noalloc(None, 1, p, p, 64, 512, 4, 128, p, None) == 1
    assert lib.rtn_linear_noalloc(p, 1, p, p, 64, 500, 4, 128, p, None) == 4
