"""Thin ctypes binding over the C ABI of include/rtn.h.

Argument marshalling only: every step of the path runs in the HIP kernels of the shared
library.  PyTorch supplies device memory and the current stream, nothing else.  There is
no fallback: if the library cannot be loaded, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build

RTN_SCALE_QMAX, RTN_SCALE_EQ2 = 0, 1
RTN_POLICY_FIRST, RTN_POLICY_LAST, RTN_POLICY_MIDDLE = 0, 1, 2
POLICY = {"first": RTN_POLICY_FIRST, "last": RTN_POLICY_LAST, "middle": RTN_POLICY_MIDDLE}


class RtnError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: rtn_status {status} ({_lib.rtn_status_str(status).decode()})")


class rtn_linear_cfg(C.Structure):
    _fields_ = [("path", C.c_int), ("prefetch", C.c_int), ("waves_n", C.c_int),
                ("waves_k", C.c_int), ("split_k", C.c_int), ("m_rows16", C.c_int), ("n_tiles16", C.c_int)]


class rtn_module(C.Structure):
    _fields_ = [("dev_A", C.c_void_p), ("M", C.c_int64), ("dev_qweight", C.c_void_p),
                ("dev_scales", C.c_void_p), ("N", C.c_int64), ("K", C.c_int64),
                ("bits", C.c_int), ("group_size", C.c_int), ("dev_C", C.c_void_p)]


def _load() -> C.CDLL:
    path = _build.LIB_PATH
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built: run `python paper_2505_15909_amd/build.py` (or __graft_entry__.build()) first")
    lib = C.CDLL(path)
    vp, i64, ci, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
    lib.rtn_status_str.restype = C.c_char_p
    lib.rtn_status_str.argtypes = [ci]
    lib.rtn_layout_version.restype = ci
    lib.rtn_qweight_nbytes.restype = sz
    lib.rtn_qweight_nbytes.argtypes = [i64, i64, ci]
    lib.rtn_scales_nbytes.restype = sz
    lib.rtn_scales_nbytes.argtypes = [i64, i64, ci]
    lib.rtn_workspace_nbytes.restype = sz
    lib.rtn_workspace_nbytes.argtypes = [i64, i64, i64, ci, ci]
    lib.rtn_quantize.restype = ci
    lib.rtn_quantize.argtypes = [vp, i64, i64, ci, ci, ci, vp, vp, vp]
    lib.rtn_linear.restype = ci
    lib.rtn_linear.argtypes = [vp, i64, vp, vp, i64, i64, ci, ci, vp, vp, sz, vp]
    lib.rtn_linear_ex.restype = ci
    lib.rtn_linear_ex.argtypes = [vp, i64, vp, vp, i64, i64, ci, ci, vp, vp, sz, vp, C.POINTER(rtn_linear_cfg)]
    lib.rtn_linear_query.restype = ci
    lib.rtn_linear_query.argtypes = [i64, i64, i64, ci, ci, C.POINTER(rtn_linear_cfg)]
    lib.rtn_unpack.restype = ci
    lib.rtn_unpack.argtypes = [vp, i64, i64, ci, vp, vp]
    lib.rtn_dequantize.restype = ci
    lib.rtn_dequantize.argtypes = [vp, vp, i64, i64, ci, ci, vp, vp]
    lib.rtn_quantize_host_staging_nbytes.restype = sz
    lib.rtn_quantize_host_staging_nbytes.argtypes = [i64, i64]
    lib.rtn_quantize_from_host.restype = ci
    lib.rtn_quantize_from_host.argtypes = [vp, i64, i64, ci, ci, ci, vp, vp, vp, sz, i64, vp, vp]
    lib.rtn_gemm_fp16.restype = ci
    lib.rtn_gemm_fp16.argtypes = [vp, i64, vp, i64, i64, vp, vp, sz, vp]
    lib.rtn_dense_weight_nbytes.restype = sz
    lib.rtn_dense_weight_nbytes.argtypes = [i64, i64]
    lib.rtn_linear_dense.restype = ci
    lib.rtn_linear_dense.argtypes = [vp, i64, vp, vp, i64, i64, ci, ci, vp, vp, sz, vp, sz, vp]
    lib.rtn_layer_forward.restype = ci
    lib.rtn_layer_forward.argtypes = [C.POINTER(rtn_module), ci, vp, sz, vp]
    lib.rtn_quantize_asym.restype = ci
    lib.rtn_quantize_asym.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp]
    lib.rtn_dequantize_asym.restype = ci
    lib.rtn_dequantize_asym.argtypes = [vp, vp, vp, i64, i64, ci, ci, vp, vp]
    lib.rtn_linear_asym.restype = ci
    lib.rtn_linear_asym.argtypes = [vp, i64, vp, vp, vp, i64, i64, ci, ci, vp, vp, sz, vp]
    lib.rtn_grouped_forward.restype = ci
    lib.rtn_grouped_forward.argtypes = [C.POINTER(rtn_module), ci, vp, sz, vp]
    lib.rtn_problem_status.restype = ci
    lib.rtn_problem_status.argtypes = [i64, i64, ci, ci]
    lib.rtn_linear_validate.restype = ci
    lib.rtn_linear_validate.argtypes = [i64, i64, i64, ci, ci, sz, C.POINTER(rtn_linear_cfg)]
    lib.rtn_linear_noalloc.restype = ci
    lib.rtn_linear_noalloc.argtypes = [vp, i64, vp, vp, i64, i64, ci, ci, vp, vp]
    lib.rtn_bench_read_stream.restype = ci
    lib.rtn_bench_read_stream.argtypes = [vp, sz, ci, vp, vp]
    lib.rtn_plan_bits.restype = ci
    lib.rtn_plan_bits.argtypes = [ci, ci, ci, ci, ci, C.c_uint]
    lib.rtn_plan_effective_bits.restype = C.c_double
    lib.rtn_plan_effective_bits.argtypes = [ci, C.POINTER(i64), ci, ci, C.c_uint]
    return lib


_lib = _load()
EXPORTS = ["rtn_status_str", "rtn_layout_version", "rtn_qweight_nbytes", "rtn_scales_nbytes",
           "rtn_workspace_nbytes", "rtn_quantize", "rtn_quantize_host_staging_nbytes", "rtn_quantize_from_host", "rtn_linear", "rtn_linear_ex", "rtn_linear_query",
           "rtn_problem_status", "rtn_linear_validate", "rtn_linear_noalloc", "rtn_unpack", "rtn_dequantize", "rtn_gemm_fp16", "rtn_dense_weight_nbytes", "rtn_linear_dense",
           "rtn_quantize_asym", "rtn_dequantize_asym", "rtn_linear_asym",
           "rtn_layer_forward", "rtn_grouped_forward", "rtn_bench_read_stream", "rtn_plan_bits", "rtn_plan_effective_bits"]


def _check(status: int, what: str):
    if status != 0:
        raise RtnError(status, what)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def _dev_fp16(t: torch.Tensor, name: str):
    if not (t.is_cuda and t.dtype == torch.float16 and t.is_contiguous() and t.dim() == 2):
        raise ValueError(f"{name} must be a contiguous fp16 CUDA matrix")


def rtn_layout_version() -> int:
    return _lib.rtn_layout_version()


def rtn_qweight_nbytes(N, K, bits):
    return _lib.rtn_qweight_nbytes(N, K, bits)


def rtn_scales_nbytes(N, K, group_size):
    return _lib.rtn_scales_nbytes(N, K, group_size)


def rtn_workspace_nbytes(M, N, K, bits, group_size):
    return _lib.rtn_workspace_nbytes(M, N, K, bits, group_size)


def rtn_quantize(W: torch.Tensor, bits: int, group_size: int, flags: int = RTN_SCALE_QMAX, out=None):
    """W fp16 [N, K] on the GPU -> (qweight uint8 [N*K*bits/8], scales fp16 [N, K/g])."""
    _dev_fp16(W, "W")
    N, K = W.shape
    g = K if group_size <= 0 else group_size
    if out is None:
        nb = _lib.rtn_qweight_nbytes(N, K, bits)
        ns = _lib.rtn_scales_nbytes(N, K, g)
        if nb == 0 or ns == 0:
            _check(_lib.rtn_problem_status(N, K, bits, group_size) or 4, "rtn_quantize")
        qweight = torch.empty(nb, dtype=torch.uint8, device=W.device)
        scales = torch.empty((N, K // g), dtype=torch.float16, device=W.device)
    else:
        qweight, scales = out
    _check(_lib.rtn_quantize(W.data_ptr(), N, K, bits, group_size, flags, qweight.data_ptr(),
                             scales.data_ptr(), _stream()), "rtn_quantize")
    return qweight, scales


def make_cfg(cfg):
    if cfg is None:
        return None
    if isinstance(cfg, rtn_linear_cfg):
        return cfg
    return rtn_linear_cfg(**cfg)


def rtn_linear(A: torch.Tensor, qweight: torch.Tensor, scales: torch.Tensor, bits: int, group_size: int,
               out: torch.Tensor = None, workspace: torch.Tensor = None, cfg=None) -> torch.Tensor:
    """A fp16 [M, K], packed qweight, scales fp16 [N, K/g] -> C fp16 [M, N]."""
    _dev_fp16(A, "A")
    M, K = A.shape
    N = scales.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=A.device)
    if workspace is None:
        workspace = torch.empty(max(256, _lib.rtn_workspace_nbytes(M, N, K, bits, group_size)),
                                dtype=torch.uint8, device=A.device)
    c = make_cfg(cfg)
    st = _lib.rtn_linear_ex(A.data_ptr(), M, qweight.data_ptr(), scales.data_ptr(), N, K, bits, group_size,
                            out.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                            _stream(), C.byref(c) if c is not None else None)
    _check(st, "rtn_linear")
    return out


def rtn_linear_query(M, N, K, bits, group_size) -> dict:
    c = rtn_linear_cfg()
    _check(_lib.rtn_linear_query(M, N, K, bits, group_size, C.byref(c)), "rtn_linear_query")
    return {k: getattr(c, k) for k, _ in rtn_linear_cfg._fields_}


def rtn_problem_status(N, K, bits, group_size) -> int:
    return _lib.rtn_problem_status(N, K, bits, group_size)


def rtn_linear_validate(M, N, K, bits, group_size, workspace_nbytes, cfg=None) -> int:
    """Host only: the status rtn_linear_ex would return for this problem and configuration (0 = it would launch)."""
    c = make_cfg(cfg)
    return _lib.rtn_linear_validate(M, N, K, bits, group_size, workspace_nbytes, None if c is None else C.byref(c))


def rtn_linear_noalloc(A: torch.Tensor, qweight: torch.Tensor, scales: torch.Tensor, bits: int, group_size: int,
                       out: torch.Tensor) -> torch.Tensor:
    """rtn_linear without a workspace argument: split-K partials go to the library's fixed device array."""
    _dev_fp16(A, "A")
    M, K = A.shape
    N = scales.shape[0]
    _check(_lib.rtn_linear_noalloc(A.data_ptr(), M, qweight.data_ptr(), scales.data_ptr(), N, K, bits, group_size,
                                   out.data_ptr(), _stream()), "rtn_linear_noalloc")
    return out


def rtn_bench_read_stream(buf: torch.Tensor, nbytes: int, kib_per_wavefront: int, sink: torch.Tensor):
    """Measurement hook: streams the first nbytes of buf once with a plain read kernel."""
    if buf.numel() * buf.element_size() < nbytes or sink.numel() * sink.element_size() < 4:
        raise ValueError(f"rtn_bench_read_stream: buffer of {buf.numel() * buf.element_size()} bytes, asked to read {nbytes}")
    _check(_lib.rtn_bench_read_stream(buf.data_ptr(), nbytes, kib_per_wavefront, sink.data_ptr(), _stream()),
           "rtn_bench_read_stream")


def rtn_unpack(qweight: torch.Tensor, N: int, K: int, bits: int) -> torch.Tensor:
    codes = torch.empty((N, K), dtype=torch.int8, device=qweight.device)
    _check(_lib.rtn_unpack(qweight.data_ptr(), N, K, bits, codes.data_ptr(), _stream()), "rtn_unpack")
    return codes


def rtn_dequantize(qweight: torch.Tensor, scales: torch.Tensor, K: int, bits: int, group_size: int,
                   out: torch.Tensor = None) -> torch.Tensor:
    N = scales.shape[0]
    W = out if out is not None else torch.empty((N, K), dtype=torch.float16, device=qweight.device)
    _check(_lib.rtn_dequantize(qweight.data_ptr(), scales.data_ptr(), N, K, bits, group_size, W.data_ptr(),
                               _stream()), "rtn_dequantize")
    return W


def rtn_quantize_from_host(W_host: torch.Tensor, bits: int, group_size: int, rows_per_shard: int, copy_stream,
                           flags: int = RTN_SCALE_QMAX, staging: torch.Tensor = None, out=None, device="cuda:0"):
    """W_host: fp16 [N, K] in (pinned) host memory -> (qweight, scales) on the GPU, quantised shard by shard with the
    host-to-device copies on `copy_stream` (a torch.cuda.Stream other than the current one) overlapping the kernels."""
    if W_host.is_cuda or W_host.dtype != torch.float16 or not W_host.is_contiguous() or W_host.dim() != 2:
        raise ValueError("W_host must be a contiguous fp16 host matrix")
    N, K = W_host.shape
    g = K if group_size <= 0 else group_size
    need = _lib.rtn_quantize_host_staging_nbytes(K, rows_per_shard)
    if staging is None:
        staging = torch.empty(max(need, 16), dtype=torch.uint8, device=device)
    if out is None:
        nb = _lib.rtn_qweight_nbytes(N, K, bits)
        ns = _lib.rtn_scales_nbytes(N, K, g)
        qweight = torch.empty(max(nb, 16), dtype=torch.uint8, device=device)[:nb]
        scales = torch.empty((N, max(K // max(g, 1), 1)), dtype=torch.float16, device=device) if ns else torch.empty((N, 1), dtype=torch.float16, device=device)
    else:
        qweight, scales = out
    _check(_lib.rtn_quantize_from_host(W_host.data_ptr(), N, K, bits, group_size, flags, qweight.data_ptr(),
                                       scales.data_ptr(), staging.data_ptr(), staging.numel(), rows_per_shard,
                                       _stream(), copy_stream.cuda_stream), "rtn_quantize_from_host")
    return qweight, scales


def rtn_gemm_fp16(A: torch.Tensor, W: torch.Tensor, out: torch.Tensor = None, workspace: torch.Tensor = None) -> torch.Tensor:
    """Dense A fp16 [M, K] times W fp16 [N, K] transposed -> C fp16 [M, N]."""
    _dev_fp16(A, "A")
    _dev_fp16(W, "W")
    M, K = A.shape
    N = W.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=A.device)
    wp, wn = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (None, 0)
    _check(_lib.rtn_gemm_fp16(A.data_ptr(), M, W.data_ptr(), N, K, out.data_ptr(), wp, wn, _stream()), "rtn_gemm_fp16")
    return out


def rtn_linear_dense(A: torch.Tensor, qweight: torch.Tensor, scales: torch.Tensor, bits: int, group_size: int,
                     w_tmp: torch.Tensor, out: torch.Tensor = None, workspace: torch.Tensor = None) -> torch.Tensor:
    """The dequantise-then-GEMM path: w_tmp is a caller-owned buffer of rtn_dense_weight_nbytes(N, K) bytes."""
    _dev_fp16(A, "A")
    M, K = A.shape
    N = scales.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=A.device)
    wp, wn = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (None, 0)
    _check(_lib.rtn_linear_dense(A.data_ptr(), M, qweight.data_ptr(), scales.data_ptr(), N, K, bits, group_size,
                                 out.data_ptr(), w_tmp.data_ptr(), w_tmp.numel() * w_tmp.element_size(), wp, wn,
                                 _stream()), "rtn_linear_dense")
    return out


def rtn_dense_weight_nbytes(N: int, K: int) -> int:
    return _lib.rtn_dense_weight_nbytes(N, K)


class LayerPlan:
    """A prepared rtn_layer_forward call: the module descriptor array is built once."""

    def __init__(self, modules, workspace: torch.Tensor = None):
        """modules: list of dicts {A, qweight, scales, bits, group_size, C}."""
        self.n = len(modules)
        self.arr = (rtn_module * self.n)()
        self.keep = modules
        need = 256
        for i, m in enumerate(modules):
            M, K = m["A"].shape
            N = m["scales"].shape[0]
            self.arr[i] = rtn_module(m["A"].data_ptr(), M, m["qweight"].data_ptr(), m["scales"].data_ptr(),
                                     N, K, m["bits"], m["group_size"], m["C"].data_ptr())
            need = max(need, _lib.rtn_workspace_nbytes(M, N, K, m["bits"], m["group_size"]))
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=modules[0]["A"].device)
        self.workspace = workspace

    def run(self):
        _check(_lib.rtn_layer_forward(self.arr, self.n, self.workspace.data_ptr(), self.workspace.numel(),
                                      _stream()), "rtn_layer_forward")

    def run_grouped(self):
        """The modules as independent problems (rtn_grouped_forward): no C may be another module's A."""
        _check(_lib.rtn_grouped_forward(self.arr, self.n, self.workspace.data_ptr(), self.workspace.numel(),
                                        _stream()), "rtn_grouped_forward")


def rtn_layer_forward(modules, workspace: torch.Tensor = None):
    LayerPlan(modules, workspace).run()


def rtn_quantize_asym(W: torch.Tensor, bits: int, group_size: int):
    """W fp16 [N, K] on the GPU -> (qweight uint8, scales fp16 [N, K/g], zeros fp16 [N, K/g]); weight = S (q + Z)."""
    _dev_fp16(W, "W")
    N, K = W.shape
    G = 1 if group_size <= 0 else K // max(group_size, 1)
    nq = _lib.rtn_qweight_nbytes(N, K, bits)
    if nq == 0:
        raise ValueError("unsupported shape or bits")
    q = torch.empty(nq, dtype=torch.uint8, device=W.device)
    s = torch.empty((N, max(G, 1)), dtype=torch.float16, device=W.device)
    z = torch.empty((N, max(G, 1)), dtype=torch.float16, device=W.device)
    _check(_lib.rtn_quantize_asym(W.data_ptr(), N, K, bits, group_size, q.data_ptr(), s.data_ptr(), z.data_ptr(),
                                  _stream()), "rtn_quantize_asym")
    return q, s, z


def rtn_dequantize_asym(qweight, scales, zeros, N, K, bits, group_size, out=None):
    if out is None:
        out = torch.empty((N, K), dtype=torch.float16, device=qweight.device)
    _check(_lib.rtn_dequantize_asym(qweight.data_ptr(), scales.data_ptr(), zeros.data_ptr(), N, K, bits, group_size,
                                    out.data_ptr(), _stream()), "rtn_dequantize_asym")
    return out


def rtn_linear_asym(A, qweight, scales, zeros, bits, group_size, out=None, workspace=None):
    _dev_fp16(A, "A")
    M, K = A.shape
    N = scales.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=A.device)
    if workspace is None:
        workspace = torch.empty(max(256, _lib.rtn_workspace_nbytes(M, N, K, bits, group_size)), dtype=torch.uint8,
                                device=A.device)
    _check(_lib.rtn_linear_asym(A.data_ptr(), M, qweight.data_ptr(), scales.data_ptr(), zeros.data_ptr(), N, K, bits,
                                group_size, out.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()),
           "rtn_linear_asym")
    return out


def rtn_grouped_forward(modules, workspace: torch.Tensor = None):
    LayerPlan(modules, workspace).run_grouped()


def rtn_plan_bits(layer, n_layers, module_id, policy, X, modules=(1, 2, 3, 4)) -> int:
    mask = 0
    for m in modules:
        mask |= 1 << (m - 1)
    pol = POLICY[policy] if isinstance(policy, str) else policy
    return _lib.rtn_plan_bits(layer, n_layers, module_id, pol, X, mask)


def rtn_plan_effective_bits(n_layers, module_params, policy, X, modules=(1, 2, 3, 4)) -> float:
    mask = 0
    for m in modules:
        mask |= 1 << (m - 1)
    pol = POLICY[policy] if isinstance(policy, str) else policy
    arr = (C.c_int64 * 4)(*[int(v) for v in module_params])
    return _lib.rtn_plan_effective_bits(n_layers, arr, pol, X, mask)
