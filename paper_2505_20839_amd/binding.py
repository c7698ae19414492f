"""Thin Python binding of the C ABI in ``include/fireq.h``: argument marshalling only.

Every step of the path runs in the HIP kernels of ``libfireq.so``; torch is used for device
memory and the current stream.  There is no CPU fallback: if the library cannot be loaded or a
tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

from . import build as _build

GROUP = 128

_lib = None


class FireqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


def lib() -> ctypes.CDLL:
    """The loaded shared library (built in-tree on first use if it was never built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        _build.build_library()
    L = ctypes.CDLL(_build.LIB_PATH)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    L.fq_w4a8_gemm.restype = ci
    L.fq_w4a8_gemm.argtypes = [vp, vp, vp, vp, cf, vp, ci, ci, ci, vp]
    L.fq_w4a8_gemm_static.restype = ci
    L.fq_w4a8_gemm_static.argtypes = [vp, vp, vp, vp, cf, vp, ci, ci, ci, vp]
    L.fq_w4a8_gemm_static_max_workspace.restype = ctypes.c_size_t
    L.fq_w4a8_gemm_static_max_workspace.argtypes = []
    L.fq_w4a8_gemm_lut.restype = ci
    L.fq_w4a8_gemm_lut.argtypes = [vp, vp, vp, vp, cf, vp, ci, ci, ci, vp]
    L.fq_kv4_packed_bytes.restype = ctypes.c_size_t
    L.fq_kv4_packed_bytes.argtypes = [ci, ci, ci]
    L.fq_kv4_pack.restype = ci
    L.fq_kv4_pack.argtypes = [vp, vp, ci, ci, ci, vp]
    L.fq_kv4_unpack.restype = ci
    L.fq_kv4_unpack.argtypes = [vp, vp, ci, ci, ci, vp]
    L.fq_kv4_scores.restype = ci
    L.fq_kv4_scores.argtypes = [vp, vp, vp, vp, cf, vp, ci, ci, ci, vp]
    L.fq_kv4_output.restype = ci
    L.fq_kv4_output.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, vp]
    L.fq_w4a8_gemm_ws.restype = ci
    L.fq_w4a8_gemm_ws.argtypes = [vp, vp, vp, vp, cf, vp, ci, ci, ci, vp, ctypes.c_size_t, ci, vp]
    L.fq_w4a8_gemm_add_ws.restype = ci
    L.fq_w4a8_gemm_add_ws.argtypes = [vp, vp, vp, vp, cf, vp, vp, ci, ci, ci, vp, ctypes.c_size_t, ci, vp]
    L.fq_w4a8_gemm_swiglu_quant_ws.restype = ci
    L.fq_w4a8_gemm_swiglu_quant_ws.argtypes = [vp, vp, vp, vp, cf, vp, vp, vp, ci, ci, ci, vp, ctypes.c_size_t, ci, vp,
                                               ctypes.c_size_t, vp]
    L.fq_w4a8_gemm_swiglu_ws.restype = ci
    L.fq_w4a8_gemm_swiglu_ws.argtypes = [vp, vp, vp, vp, cf, vp, ci, ci, ci, vp, ctypes.c_size_t, ci, vp]
    L.fq_quantize_act_ws.restype = ci
    L.fq_quantize_act_ws.argtypes = [vp, vp, vp, ci, ci, vp, ctypes.c_size_t, vp]
    L.fq_w4a8_gemm_workspace_bytes.restype = ctypes.c_size_t
    L.fq_w4a8_gemm_workspace_bytes.argtypes = [ci, ci, ci]
    L.fq_quantize_act.restype = ci
    L.fq_quantize_act.argtypes = [vp, vp, vp, ci, ci, vp]
    L.fq_packed_weight_bytes.restype = ctypes.c_size_t
    L.fq_packed_weight_bytes.argtypes = [ci, ci]
    L.fq_pack_weights.restype = ci
    L.fq_pack_weights.argtypes = [vp, vp, ci, ci, vp]
    L.fq_unpack_weights.restype = ci
    L.fq_unpack_weights.argtypes = [vp, vp, ci, ci, vp]
    L.fq_w4a8_linear_workspace_bytes.restype = ctypes.c_size_t
    L.fq_w4a8_linear_workspace_bytes.argtypes = [ci, ci, ci]
    L.fq_w4a8_linear_ws.restype = ci
    L.fq_w4a8_linear_ws.argtypes = [vp, vp, vp, cf, vp, ci, ci, ci, vp, ctypes.c_size_t, vp]
    L.fq_cas_scales.restype = ci
    L.fq_cas_scales.argtypes = [vp, cf, vp, ci, ci, vp]
    L.fq_pts_exponent.restype = ci
    L.fq_pts_exponent.argtypes = [vp, vp, vp, ci, ci, vp]
    L.fq_quantize_weights.restype = ci
    L.fq_quantize_weights.argtypes = [vp, vp, ci, ci, vp, vp, ci, ci, vp]
    L.fq_w4a8_gemm_plan.restype = ci
    L.fq_w4a8_gemm_plan.argtypes = [ci, ci, ci, ci, ctypes.POINTER(ctypes.c_int)]
    L.fq_diag_stream_read.restype = ci
    L.fq_diag_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    L.fq_diag_stream_read_sink_bytes.restype = ctypes.c_size_t
    L.fq_diag_stream_read_sink_bytes.argtypes = []
    L.fq_test_force_kernel.restype = ci
    L.fq_test_force_kernel.argtypes = [ctypes.c_char_p]
    L.fq_layout_version.restype = ci
    L.fq_layout_version.argtypes = []
    L.fq_status_string.restype = ctypes.c_char_p
    L.fq_status_string.argtypes = [ci]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().fq_status_string(int(status)).decode()


def fq_layout_version() -> int:
    return int(lib().fq_layout_version())


def fq_packed_weight_bytes(N: int, K: int) -> int:
    return int(lib().fq_packed_weight_bytes(int(N), int(K)))


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a GPU tensor" % name)
    if t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def fq_cas_scales(W: torch.Tensor, target: float) -> torch.Tensor:
    """float32 [K]: lambda[k] = target / absmean_n(W[n,k]) of a bf16 weight matrix [N,K]."""
    W = _dev(W, torch.bfloat16, "W")
    N, K = W.shape
    lam = torch.empty((K,), dtype=torch.float32, device=W.device)
    rc = lib().fq_cas_scales(W.data_ptr(), ctypes.c_float(float(target)), lam.data_ptr(), N, K, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_cas_scales")
    return lam


def _lambda_ptr(lam, K):
    if lam is None:
        return 0
    lam = _dev(lam, torch.float32, "lam")
    if lam.numel() != K:
        raise FireqError(-2, "lambda")
    return lam.data_ptr()


def fq_pts_exponent(W: torch.Tensor, lam: Optional[torch.Tensor] = None) -> torch.Tensor:
    """int32 device tensor of 16 ints whose first element is the per-tensor exponent n (delta = 2^n) of the
    bf16 matrix W [N,K] scaled by lam [K]; reading it (``int(t[0])``) synchronises, the call does not."""
    W = _dev(W, torch.bfloat16, "W")
    N, K = W.shape
    out = torch.empty((16,), dtype=torch.int32, device=W.device)
    rc = lib().fq_pts_exponent(W.data_ptr(), _lambda_ptr(lam, K), out.data_ptr(), N, K, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_pts_exponent")
    return out


def fq_quantize_weights(W: torch.Tensor, lam: Optional[torch.Tensor] = None, n_pts: int = 0,
                        sigma_nearest: bool = False):
    """(int8 [N,K] INT4 codes, uint8 [N,K/128] E4M3 group scales) of W * lam * 2^n_pts."""
    W = _dev(W, torch.bfloat16, "W")
    N, K = W.shape
    if K % GROUP:
        raise FireqError(-2, "fq_quantize_weights")
    q = torch.empty((N, K), dtype=torch.int8, device=W.device)
    gs = torch.empty((N, K // GROUP), dtype=torch.uint8, device=W.device)
    rc = lib().fq_quantize_weights(W.data_ptr(), _lambda_ptr(lam, K), int(n_pts), 1 if sigma_nearest else 0,
                                   q.data_ptr(), gs.data_ptr(), N, K, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_quantize_weights")
    return q, gs


def fq_pack_weights(q: torch.Tensor) -> torch.Tensor:
    """int8 [N,K] codes in -8..7 -> packed uint8 buffer of fq_packed_weight_bytes(N,K) bytes."""
    q = _dev(q, torch.int8, "q")
    N, K = q.shape
    nbytes = fq_packed_weight_bytes(N, K)
    if nbytes == 0:
        raise FireqError(-2, "fq_pack_weights")
    out = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
    rc = lib().fq_pack_weights(q.data_ptr(), out.data_ptr(), N, K, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_pack_weights")
    return out


def fq_unpack_weights(packed: torch.Tensor, N: int, K: int) -> torch.Tensor:
    packed = _dev(packed, torch.uint8, "packed")
    if packed.numel() < fq_packed_weight_bytes(N, K) or fq_packed_weight_bytes(N, K) == 0:
        raise FireqError(-2, "fq_unpack_weights")
    out = torch.empty((N, K), dtype=torch.int8, device=packed.device)
    rc = lib().fq_unpack_weights(packed.data_ptr(), out.data_ptr(), N, K, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_unpack_weights")
    return out


def fq_quantize_act(X: torch.Tensor, workspace: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """bf16 [M,K] -> (uint8 [M,K] E4M3 codes, float32 [M] per-row scales).

    With `workspace` (a device tensor of fq_w4a8_gemm_workspace_bytes(M, N, K) bytes or more) the call is
    fq_quantize_act_ws, which also prepares that workspace for fq_w4a8_gemm(..., workspace_prepared=True)."""
    X = _dev(X, torch.bfloat16, "X")
    M, K = X.shape
    A = torch.empty((M, K), dtype=torch.uint8, device=X.device)
    s = torch.empty((M,), dtype=torch.float32, device=X.device)
    if workspace is None:
        rc = lib().fq_quantize_act(X.data_ptr(), A.data_ptr(), s.data_ptr(), M, K, _stream())
    else:
        rc = lib().fq_quantize_act_ws(X.data_ptr(), A.data_ptr(), s.data_ptr(), M, K, workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), _stream())
    if rc != 0:
        raise FireqError(rc, "fq_quantize_act")
    return A, s


def fq_w4a8_gemm(A: torch.Tensor, a_scale: torch.Tensor, Wq_packed: torch.Tensor,
                 w_gscale: torch.Tensor, w_tscale: float, N: int,
                 out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                 workspace_prepared: bool = False) -> torch.Tensor:
    """Y[M,N] (bf16) = W4A8-FP GEMM of E4M3 activations and packed INT4 weights.

    Calls fq_w4a8_gemm_ws; `workspace` (a device tensor of at least
    fq_w4a8_gemm_workspace_bytes(M, N, K) bytes) is allocated here when not given;
    `workspace_prepared` says that fq_quantize_act(X, workspace) has filled it for this A."""
    A = _dev(A, torch.uint8, "A")
    a_scale = _dev(a_scale, torch.float32, "a_scale")
    Wq_packed = _dev(Wq_packed, torch.uint8, "Wq_packed")
    w_gscale = _dev(w_gscale, torch.uint8, "w_gscale")
    M, K = A.shape
    if a_scale.numel() != M or K % GROUP or w_gscale.numel() != N * (K // GROUP) \
            or Wq_packed.numel() < fq_packed_weight_bytes(N, K):
        raise FireqError(-2, "fq_w4a8_gemm")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    else:
        out = _dev(out, torch.bfloat16, "out")
        if tuple(out.shape) != (M, N):
            raise FireqError(-2, "fq_w4a8_gemm")
    # the workspace comes from torch's caching allocator (stream-ordered, no hipMalloc per call)
    need = lib().fq_w4a8_gemm_workspace_bytes(M, N, K)
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=A.device)
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (0, 0)
    rc = lib().fq_w4a8_gemm_ws(A.data_ptr(), a_scale.data_ptr(), Wq_packed.data_ptr(),
                               w_gscale.data_ptr(), ctypes.c_float(float(w_tscale)), out.data_ptr(),
                               M, N, K, ws_ptr, ws_bytes, 1 if (workspace_prepared and workspace is not None) else 0,
                               _stream())
    if rc != 0:
        raise FireqError(rc, "fq_w4a8_gemm_ws")
    return out


def fq_w4a8_gemm_swiglu(A: torch.Tensor, a_scale: torch.Tensor, Wq_packed: torch.Tensor,
                        w_gscale: torch.Tensor, w_tscale: float, N: int,
                        out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                        workspace_prepared: bool = False) -> torch.Tensor:
    """H[M,N/2] (bf16) = SiLU(gate) * up of the W4A8-FP GEMM whose N weight rows interleave gate (even)
    and up (odd) channels.  Calls fq_w4a8_gemm_swiglu_ws; workspace handling as in fq_w4a8_gemm."""
    A = _dev(A, torch.uint8, "A")
    a_scale = _dev(a_scale, torch.float32, "a_scale")
    Wq_packed = _dev(Wq_packed, torch.uint8, "Wq_packed")
    w_gscale = _dev(w_gscale, torch.uint8, "w_gscale")
    M, K = A.shape
    if N % 2 or a_scale.numel() != M or K % GROUP or w_gscale.numel() != N * (K // GROUP) \
            or Wq_packed.numel() < fq_packed_weight_bytes(N, K):
        raise FireqError(-2, "fq_w4a8_gemm_swiglu")
    if out is None:
        out = torch.empty((M, N // 2), dtype=torch.bfloat16, device=A.device)
    else:
        out = _dev(out, torch.bfloat16, "out")
        if tuple(out.shape) != (M, N // 2):
            raise FireqError(-2, "fq_w4a8_gemm_swiglu")
    need = lib().fq_w4a8_gemm_workspace_bytes(M, N, K)
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=A.device)
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (0, 0)
    rc = lib().fq_w4a8_gemm_swiglu_ws(A.data_ptr(), a_scale.data_ptr(), Wq_packed.data_ptr(),
                                      w_gscale.data_ptr(), ctypes.c_float(float(w_tscale)), out.data_ptr(),
                                      M, N, K, ws_ptr, ws_bytes,
                                      1 if (workspace_prepared and workspace is not None) else 0, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_w4a8_gemm_swiglu_ws")
    return out


def fq_w4a8_gemm_swiglu_quant(A: torch.Tensor, a_scale: torch.Tensor, Wq_packed: torch.Tensor,
                              w_gscale: torch.Tensor, w_tscale: float, N: int,
                              out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                              workspace_prepared: bool = False, next_workspace: Optional[torch.Tensor] = None
                              ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """(H bf16 [M,N/2], H as E4M3 codes [M,N/2], float32 [M] scales): fq_w4a8_gemm_swiglu whose output also leaves
    quantised for the next layer, as fq_quantize_act would give it.  Calls fq_w4a8_gemm_swiglu_quant_ws;
    `next_workspace` (fq_w4a8_gemm_workspace_bytes(M, N', N/2) bytes or more) is prepared for a GEMM on the codes."""
    A = _dev(A, torch.uint8, "A")
    a_scale = _dev(a_scale, torch.float32, "a_scale")
    Wq_packed = _dev(Wq_packed, torch.uint8, "Wq_packed")
    w_gscale = _dev(w_gscale, torch.uint8, "w_gscale")
    M, K = A.shape
    if N % 2 or a_scale.numel() != M or K % GROUP or w_gscale.numel() != N * (K // GROUP) \
            or Wq_packed.numel() < fq_packed_weight_bytes(N, K):
        raise FireqError(-2, "fq_w4a8_gemm_swiglu_quant")
    if out is None:
        out = torch.empty((M, N // 2), dtype=torch.bfloat16, device=A.device)
    else:
        out = _dev(out, torch.bfloat16, "out")
        if tuple(out.shape) != (M, N // 2):
            raise FireqError(-2, "fq_w4a8_gemm_swiglu_quant")
    codes = torch.empty((M, N // 2), dtype=torch.uint8, device=A.device)
    scales = torch.empty((M,), dtype=torch.float32, device=A.device)
    need = lib().fq_w4a8_gemm_workspace_bytes(M, N, K)
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=A.device)
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (0, 0)
    nws_ptr, nws_bytes = (next_workspace.data_ptr(), next_workspace.numel() * next_workspace.element_size()) \
        if next_workspace is not None else (0, 0)
    rc = lib().fq_w4a8_gemm_swiglu_quant_ws(A.data_ptr(), a_scale.data_ptr(), Wq_packed.data_ptr(),
                                            w_gscale.data_ptr(), ctypes.c_float(float(w_tscale)), out.data_ptr(),
                                            codes.data_ptr(), scales.data_ptr(), M, N, K, ws_ptr, ws_bytes,
                                            1 if (workspace_prepared and workspace is not None) else 0,
                                            nws_ptr, nws_bytes, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_w4a8_gemm_swiglu_quant_ws")
    return out, codes, scales


def fq_w4a8_gemm_add(A: torch.Tensor, a_scale: torch.Tensor, Wq_packed: torch.Tensor,
                     w_gscale: torch.Tensor, w_tscale: float, N: int, residual: torch.Tensor,
                     out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                     workspace_prepared: bool = False) -> torch.Tensor:
    """Y[M,N] (bf16) = GEMM + residual, rounded once.  Calls fq_w4a8_gemm_add_ws; `out` may be
    `residual` itself (in-place update); workspace handling as in fq_w4a8_gemm."""
    A = _dev(A, torch.uint8, "A")
    a_scale = _dev(a_scale, torch.float32, "a_scale")
    Wq_packed = _dev(Wq_packed, torch.uint8, "Wq_packed")
    w_gscale = _dev(w_gscale, torch.uint8, "w_gscale")
    residual = _dev(residual, torch.bfloat16, "residual")
    M, K = A.shape
    if a_scale.numel() != M or K % GROUP or w_gscale.numel() != N * (K // GROUP) \
            or Wq_packed.numel() < fq_packed_weight_bytes(N, K) or tuple(residual.shape) != (M, N):
        raise FireqError(-2, "fq_w4a8_gemm_add")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    else:
        out = _dev(out, torch.bfloat16, "out")
        if tuple(out.shape) != (M, N):
            raise FireqError(-2, "fq_w4a8_gemm_add")
    need = lib().fq_w4a8_gemm_workspace_bytes(M, N, K)
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=A.device)
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (0, 0)
    rc = lib().fq_w4a8_gemm_add_ws(A.data_ptr(), a_scale.data_ptr(), Wq_packed.data_ptr(),
                                   w_gscale.data_ptr(), ctypes.c_float(float(w_tscale)), residual.data_ptr(),
                                   out.data_ptr(), M, N, K, ws_ptr, ws_bytes,
                                   1 if (workspace_prepared and workspace is not None) else 0, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_w4a8_gemm_add_ws")
    return out


def fq_w4a8_linear_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().fq_w4a8_linear_workspace_bytes(M, N, K))


def fq_w4a8_linear(X: torch.Tensor, Wq_packed: torch.Tensor, w_gscale: torch.Tensor, w_tscale: float, N: int,
                   out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y[M,N] (bf16) of a whole linear layer from bf16 activations X[M,K] (quantiser + GEMM; one kernel
    for M <= 6 and K <= 4096).  Calls fq_w4a8_linear_ws; the workspace is allocated here when not given."""
    X = _dev(X, torch.bfloat16, "X")
    Wq_packed = _dev(Wq_packed, torch.uint8, "Wq_packed")
    w_gscale = _dev(w_gscale, torch.uint8, "w_gscale")
    M, K = X.shape
    if K % GROUP or w_gscale.numel() != N * (K // GROUP) or Wq_packed.numel() < fq_packed_weight_bytes(N, K):
        raise FireqError(-2, "fq_w4a8_linear")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    else:
        out = _dev(out, torch.bfloat16, "out")
        if tuple(out.shape) != (M, N):
            raise FireqError(-2, "fq_w4a8_linear")
    need = fq_w4a8_linear_workspace_bytes(M, N, K)
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=X.device)
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (0, 0)
    rc = lib().fq_w4a8_linear_ws(X.data_ptr(), Wq_packed.data_ptr(), w_gscale.data_ptr(), ctypes.c_float(float(w_tscale)),
                                 out.data_ptr(), M, N, K, ws_ptr, ws_bytes, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_w4a8_linear_ws")
    return out


def fq_w4a8_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().fq_w4a8_gemm_workspace_bytes(M, N, K))


def fq_w4a8_gemm_plan(M: int, N: int, K: int, cus: int = 0) -> dict:
    """How the GEMM entry points would run this shape (see fireq.h); cus = 0 asks the current device."""
    buf = (ctypes.c_int * 8)()
    rc = lib().fq_w4a8_gemm_plan(int(M), int(N), int(K), int(cus), buf)
    if rc != 0:
        raise FireqError(rc, "fq_w4a8_gemm_plan")
    return {"kernel": ("simple", "small16", "smallm", "large", "ksplit256x128", "ksplit128x64", "ksplit64x64")[buf[0]], "whole": buf[1],
            "whole_ragged": buf[2], "half": buf[3], "half_ragged": buf[4], "ksplit_tiles": buf[5], "ksplit_slices": buf[6]}


def fq_test_force_kernel(name: Optional[str]) -> None:
    """Cross-check hook: "simple" | "small" | "large" | "ksplit" forces that GEMM kernel, None or "auto" restores the choice by M."""
    lib().fq_test_force_kernel((name or "").encode() if name != "auto" else b"")


def fq_diag_stream_read(src: torch.Tensor, sink: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Measurement aid: enqueue a kernel that only reads `src` (its bytes must be a multiple of 16)."""
    nbytes = src.numel() * src.element_size()
    if sink is None:
        sink = torch.empty((lib().fq_diag_stream_read_sink_bytes(),), dtype=torch.uint8, device=src.device)
    rc = lib().fq_diag_stream_read(src.data_ptr(), nbytes, sink.data_ptr(), _stream())
    if rc != 0:
        raise FireqError(rc, "fq_diag_stream_read")
    return sink


def fq_w4a8_gemm_lut(A: torch.Tensor, a_scale: torch.Tensor, Wq_packed: torch.Tensor, w_gscale: torch.Tensor,
                     w_tscale: float, N: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y[M,N] (bf16) of the GEMM in the paper's table mode (weights rounded to E4M3(q * sigma)); calls fq_w4a8_gemm_lut."""
    A = _dev(A, torch.uint8, "A")
    a_scale = _dev(a_scale, torch.float32, "a_scale")
    Wq_packed = _dev(Wq_packed, torch.uint8, "Wq_packed")
    w_gscale = _dev(w_gscale, torch.uint8, "w_gscale")
    M, K = A.shape
    if a_scale.numel() != M or K % GROUP or w_gscale.numel() != N * (K // GROUP) \
            or Wq_packed.numel() < fq_packed_weight_bytes(N, K):
        raise FireqError(-2, "fq_w4a8_gemm_lut")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    else:
        out = _dev(out, torch.bfloat16, "out")
        if tuple(out.shape) != (M, N):
            raise FireqError(-2, "fq_w4a8_gemm_lut")
    rc = lib().fq_w4a8_gemm_lut(A.data_ptr(), a_scale.data_ptr(), Wq_packed.data_ptr(), w_gscale.data_ptr(),
                                ctypes.c_float(float(w_tscale)), out.data_ptr(), M, N, K, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_w4a8_gemm_lut")
    return out


def fq_kv4_pack(codes: torch.Tensor, values: bool) -> torch.Tensor:
    """int8 [H,T,128] INT4 codes of a key (values=False) or value (values=True) cache -> the packed cache."""
    codes = _dev(codes, torch.int8, "codes")
    H, T, D = codes.shape
    if D != GROUP:
        raise FireqError(-2, "fq_kv4_pack")
    out = torch.empty((lib().fq_kv4_packed_bytes(H, T, 1 if values else 0),), dtype=torch.uint8, device=codes.device)
    rc = lib().fq_kv4_pack(codes.data_ptr(), out.data_ptr(), H, T, 1 if values else 0, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_kv4_pack")
    return out


def fq_kv4_unpack(packed: torch.Tensor, H: int, T: int, values: bool) -> torch.Tensor:
    packed = _dev(packed, torch.uint8, "packed")
    if packed.numel() < lib().fq_kv4_packed_bytes(H, T, 1 if values else 0):
        raise FireqError(-2, "fq_kv4_unpack")
    out = torch.empty((H, T, GROUP), dtype=torch.int8, device=packed.device)
    rc = lib().fq_kv4_unpack(packed.data_ptr(), out.data_ptr(), H, T, 1 if values else 0, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_kv4_unpack")
    return out


def fq_kv4_scores(Q: torch.Tensor, q_scale: torch.Tensor, K_packed: torch.Tensor, k_scale: torch.Tensor,
                  out_scale: float) -> torch.Tensor:
    """S[H,R,T] (bf16): FP8 queries [H,R,128] against a packed INT4 key cache with E4M3 scales [H,T]."""
    Q = _dev(Q, torch.uint8, "Q"); q_scale = _dev(q_scale, torch.float32, "q_scale")
    K_packed = _dev(K_packed, torch.uint8, "K_packed"); k_scale = _dev(k_scale, torch.uint8, "k_scale")
    H, R, D = Q.shape
    T = k_scale.shape[1]
    if D != GROUP or tuple(q_scale.shape) != (H, R) or k_scale.shape[0] != H \
            or K_packed.numel() < lib().fq_kv4_packed_bytes(H, T, 0):
        raise FireqError(-2, "fq_kv4_scores")
    S = torch.empty((H, R, T), dtype=torch.bfloat16, device=Q.device)
    rc = lib().fq_kv4_scores(Q.data_ptr(), q_scale.data_ptr(), K_packed.data_ptr(), k_scale.data_ptr(),
                             ctypes.c_float(float(out_scale)), S.data_ptr(), H, R, T, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_kv4_scores")
    return S


def fq_kv4_output(P: torch.Tensor, p_scale: torch.Tensor, V_packed: torch.Tensor, v_scale: torch.Tensor) -> torch.Tensor:
    """O[H,R,128] (bf16): FP8 probabilities [H,R,T] against a packed INT4 value cache with E4M3 scales [H,T]."""
    P = _dev(P, torch.uint8, "P"); p_scale = _dev(p_scale, torch.float32, "p_scale")
    V_packed = _dev(V_packed, torch.uint8, "V_packed"); v_scale = _dev(v_scale, torch.uint8, "v_scale")
    H, R, ldp = P.shape
    T = v_scale.shape[1]
    if tuple(p_scale.shape) != (H, R) or v_scale.shape[0] != H or ldp < T \
            or V_packed.numel() < lib().fq_kv4_packed_bytes(H, T, 1):
        raise FireqError(-2, "fq_kv4_output")
    O = torch.empty((H, R, GROUP), dtype=torch.bfloat16, device=P.device)
    rc = lib().fq_kv4_output(P.data_ptr(), p_scale.data_ptr(), V_packed.data_ptr(), v_scale.data_ptr(), O.data_ptr(),
                             H, R, T, ldp, _stream())
    if rc != 0:
        raise FireqError(rc, "fq_kv4_output")
    return O
