"""numpy front end of the CPU oracle in ``fq_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
``cpu_baseline`` leg.  Nothing in the product package imports this module, and this module
imports nothing from the product package.  All arithmetic lives in the C file; this file only
marshals numpy arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fq_oracle.c")
_LIB = os.path.join(_HERE, "libfq_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile ``fq_oracle.c`` with gcc (no fast-math) and return the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    u8p = ctypes.POINTER(ctypes.c_uint8)
    i8p = ctypes.POINTER(ctypes.c_int8)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    f32p = ctypes.POINTER(ctypes.c_float)
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.fqo_e4m3_decode.restype = ctypes.c_double
    lib.fqo_e4m3_decode.argtypes = [ctypes.c_uint8]
    lib.fqo_e4m3_encode_rne.restype = ctypes.c_uint8
    lib.fqo_e4m3_encode_rne.argtypes = [ctypes.c_double]
    lib.fqo_int4_decode.restype = ctypes.c_int
    lib.fqo_int4_decode.argtypes = [ctypes.c_uint8]
    lib.fqo_bf16_decode.restype = ctypes.c_double
    lib.fqo_bf16_decode.argtypes = [ctypes.c_uint16]
    lib.fqo_bf16_encode_rne.restype = ctypes.c_uint16
    lib.fqo_bf16_encode_rne.argtypes = [ctypes.c_double]
    lib.fqo_bf16_ulp.restype = ctypes.c_double
    lib.fqo_bf16_ulp.argtypes = [ctypes.c_double]
    lib.fqo_bf16_encode_rne_array.restype = None
    lib.fqo_bf16_encode_rne_array.argtypes = [f64p, u16p, ctypes.c_size_t]
    lib.fqo_bf16_ulp_array.restype = None
    lib.fqo_bf16_ulp_array.argtypes = [f64p, f64p, ctypes.c_size_t]
    lib.fqo_w4a8_gemm.restype = ctypes.c_int
    lib.fqo_w4a8_gemm.argtypes = [u8p, f32p, i8p, u8p, ctypes.c_float, f64p, f64p,
                                  ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.fqo_w4a8_gemm_lut.restype = ctypes.c_int
    lib.fqo_w4a8_gemm_lut.argtypes = [u8p, f32p, i8p, u8p, ctypes.c_float, f64p, f64p,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.fqo_kv4_scores.restype = ctypes.c_int
    lib.fqo_kv4_scores.argtypes = [u8p, f32p, i8p, u8p, ctypes.c_float, f64p, f64p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.fqo_kv4_output.restype = ctypes.c_int
    lib.fqo_kv4_output.argtypes = [u8p, f32p, i8p, u8p, f64p, f64p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.fqo_w4a8_gemm_swiglu.restype = ctypes.c_int
    lib.fqo_w4a8_gemm_swiglu.argtypes = [u8p, f32p, i8p, u8p, ctypes.c_float, f64p, f64p,
                                         ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.fqo_w4a8_gemm_add.restype = ctypes.c_int
    lib.fqo_w4a8_gemm_add.argtypes = [u8p, f32p, i8p, u8p, ctypes.c_float, u16p, f64p, f64p,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.fqo_quantize_act.restype = ctypes.c_int
    lib.fqo_quantize_act.argtypes = [u16p, u8p, f32p, ctypes.c_int, ctypes.c_int]
    lib.fqo_e4m3_encode_rtz.restype = ctypes.c_uint8
    lib.fqo_e4m3_encode_rtz.argtypes = [ctypes.c_double]
    lib.fqo_cas_scales.restype = ctypes.c_int
    lib.fqo_cas_scales.argtypes = [u16p, ctypes.c_double, f64p, ctypes.c_int, ctypes.c_int]
    lib.fqo_scaled_weights.restype = None
    lib.fqo_scaled_weights.argtypes = [u16p, f32p, f32p, ctypes.c_int, ctypes.c_int]
    lib.fqo_quantize_weights.restype = ctypes.c_int
    lib.fqo_quantize_weights.argtypes = [u16p, f32p, ctypes.c_int, ctypes.c_int, i8p, u8p, ctypes.c_int, ctypes.c_int]
    lib.fqo_num_threads.restype = ctypes.c_int
    lib.fqo_num_threads.argtypes = []
    _lib = lib
    return lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.dtype(dtype):
        raise TypeError("expected %s, got %s" % (np.dtype(dtype), a.dtype))
    return a


# ---- scalar format helpers -----------------------------------------------------------------

def e4m3_decode(code: int) -> float:
    return float(_load().fqo_e4m3_decode(int(code) & 0xFF))


def e4m3_encode_rne(x: float) -> int:
    return int(_load().fqo_e4m3_encode_rne(float(x)))


def int4_decode(nibble: int) -> int:
    return int(_load().fqo_int4_decode(int(nibble) & 0xFF))


def bf16_decode(bits: int) -> float:
    return float(_load().fqo_bf16_decode(int(bits) & 0xFFFF))


def bf16_encode_rne(x: float) -> int:
    return int(_load().fqo_bf16_encode_rne(float(x)))


def bf16_ulp(x: float) -> float:
    return float(_load().fqo_bf16_ulp(float(x)))


def num_threads() -> int:
    return int(_load().fqo_num_threads())


# ---- array entry points --------------------------------------------------------------------

def w4a8_gemm(A, a_scale, q, gscale, w_tscale, want_bound: bool = False):
    """FP64 ``Y[M,N]`` (and optionally the absolute-value bound) of the W4A8-FP GEMM.

    A: uint8 [M,K] E4M3 codes; a_scale: float32 [M]; q: int8 [N,K] in -8..7;
    gscale: uint8 [N,K/128] E4M3 codes; w_tscale: float.
    """
    A = _c(A, np.uint8)
    a_scale = _c(a_scale, np.float32)
    q = _c(q, np.int8)
    gscale = _c(gscale, np.uint8)
    M, K = A.shape
    N = q.shape[0]
    if q.shape != (N, K) or a_scale.shape != (M,) or gscale.shape != (N, K // 128):
        raise ValueError("operand shapes do not match")
    Y = np.zeros((M, N), dtype=np.float64)
    B = np.zeros((M, N), dtype=np.float64) if want_bound else None
    rc = _load().fqo_w4a8_gemm(
        _ptr(A, ctypes.c_uint8), _ptr(a_scale, ctypes.c_float), _ptr(q, ctypes.c_int8),
        _ptr(gscale, ctypes.c_uint8), ctypes.c_float(float(np.float32(w_tscale))),
        _ptr(Y, ctypes.c_double),
        _ptr(B, ctypes.c_double) if want_bound else ctypes.POINTER(ctypes.c_double)(),
        M, N, K)
    if rc != 0:
        raise ValueError("fqo_w4a8_gemm failed with %d" % rc)
    return (Y, B) if want_bound else Y


def w4a8_gemm_lut(A, a_scale, q, gscale, w_tscale, want_bound: bool = False):
    """FP64 ``Y[M,N]`` of the GEMM in the paper's table form (Sec. 3.1.1 step 1): every weight is the
    E4M3 rounding of ``q * sigma``.  A measuring stick for that rounding, not the library's target.
    With ``want_bound`` also the same sum over absolute values (the forward-error scale)."""
    A = _c(A, np.uint8)
    a_scale = _c(a_scale, np.float32)
    q = _c(q, np.int8)
    gscale = _c(gscale, np.uint8)
    M, K = A.shape
    N = q.shape[0]
    if q.shape != (N, K) or a_scale.shape != (M,) or gscale.shape != (N, K // 128):
        raise ValueError("operand shapes do not match")
    if q.size and (q.min() < -8 or q.max() > 7):
        raise ValueError("INT4 codes out of range")
    Y = np.zeros((M, N), dtype=np.float64)
    B = np.zeros((M, N), dtype=np.float64) if want_bound else None
    rc = _load().fqo_w4a8_gemm_lut(
        _ptr(A, ctypes.c_uint8), _ptr(a_scale, ctypes.c_float), _ptr(q, ctypes.c_int8),
        _ptr(gscale, ctypes.c_uint8), ctypes.c_float(float(np.float32(w_tscale))),
        _ptr(Y, ctypes.c_double),
        _ptr(B, ctypes.c_double) if want_bound else ctypes.POINTER(ctypes.c_double)(), M, N, K)
    if rc != 0:
        raise ValueError("fqo_w4a8_gemm_lut failed with %d" % rc)
    return (Y, B) if want_bound else Y


def w4a8_gemm_swiglu(A, a_scale, q, gscale, w_tscale, want_bound: bool = False):
    """FP64 ``H[M,N/2] = SiLU(Y[:, 0::2]) * Y[:, 1::2]`` of the W4A8-FP GEMM ``Y`` (gate rows at even,
    up rows at odd indices of ``q``), and optionally the first-order error bound."""
    A = _c(A, np.uint8)
    a_scale = _c(a_scale, np.float32)
    q = _c(q, np.int8)
    gscale = _c(gscale, np.uint8)
    M, K = A.shape
    N = q.shape[0]
    if N % 2 or q.shape != (N, K) or a_scale.shape != (M,) or gscale.shape != (N, K // 128):
        raise ValueError("operand shapes do not match")
    H = np.zeros((M, N // 2), dtype=np.float64)
    B = np.zeros((M, N // 2), dtype=np.float64) if want_bound else None
    rc = _load().fqo_w4a8_gemm_swiglu(
        _ptr(A, ctypes.c_uint8), _ptr(a_scale, ctypes.c_float), _ptr(q, ctypes.c_int8),
        _ptr(gscale, ctypes.c_uint8), ctypes.c_float(float(np.float32(w_tscale))),
        _ptr(H, ctypes.c_double),
        _ptr(B, ctypes.c_double) if want_bound else ctypes.POINTER(ctypes.c_double)(),
        M, N, K)
    if rc != 0:
        raise ValueError("fqo_w4a8_gemm_swiglu failed with %d" % rc)
    return (H, B) if want_bound else H


def w4a8_gemm_add(A, a_scale, q, gscale, w_tscale, R_bf16_bits, want_bound: bool = False):
    """FP64 ``GEMM + R`` with ``R`` given as uint16 [M,N] bf16 bit patterns (the residual
    stream added in the epilogue), and optionally the GEMM's absolute-value bound."""
    A = _c(A, np.uint8)
    a_scale = _c(a_scale, np.float32)
    q = _c(q, np.int8)
    gscale = _c(gscale, np.uint8)
    R = _c(R_bf16_bits, np.uint16)
    M, K = A.shape
    N = q.shape[0]
    if q.shape != (N, K) or a_scale.shape != (M,) or gscale.shape != (N, K // 128) or R.shape != (M, N):
        raise ValueError("operand shapes do not match")
    Y = np.zeros((M, N), dtype=np.float64)
    B = np.zeros((M, N), dtype=np.float64) if want_bound else None
    rc = _load().fqo_w4a8_gemm_add(
        _ptr(A, ctypes.c_uint8), _ptr(a_scale, ctypes.c_float), _ptr(q, ctypes.c_int8),
        _ptr(gscale, ctypes.c_uint8), ctypes.c_float(float(np.float32(w_tscale))),
        _ptr(R, ctypes.c_uint16), _ptr(Y, ctypes.c_double),
        _ptr(B, ctypes.c_double) if want_bound else ctypes.POINTER(ctypes.c_double)(),
        M, N, K)
    if rc != 0:
        raise ValueError("fqo_w4a8_gemm_add failed with %d" % rc)
    return (Y, B) if want_bound else Y


def w4a8_linear(X_bf16_bits, q, gscale, w_tscale, want_bound: bool = False):
    """A whole linear layer from bf16 activations: the quantiser of Sec. 2.1 eq. 2 (quantize_act) followed by
    the GEMM of Sec. 2.2 eq. 3 (w4a8_gemm) -- their composition and nothing else."""
    A, s = quantize_act(X_bf16_bits)
    return w4a8_gemm(A, s, q, gscale, w_tscale, want_bound=want_bound)


def quantize_act(X_bf16_bits):
    """uint16 [M,K] bf16 bit patterns -> (uint8 [M,K] E4M3 codes, float32 [M] scales)."""
    X = _c(X_bf16_bits, np.uint16)
    M, K = X.shape
    A = np.zeros((M, K), dtype=np.uint8)
    s = np.zeros((M,), dtype=np.float32)
    rc = _load().fqo_quantize_act(_ptr(X, ctypes.c_uint16), _ptr(A, ctypes.c_uint8),
                                  _ptr(s, ctypes.c_float), M, K)
    if rc != 0:
        raise ValueError("fqo_quantize_act failed with %d" % rc)
    return A, s


# ---- offline weight quantisation -------------------------------------------------------------

def e4m3_encode_rtz(x: float) -> int:
    return int(_load().fqo_e4m3_encode_rtz(float(x)))


def cas_scales(W_bf16_bits, target: float) -> np.ndarray:
    """float64 [K]: lambda[k] = target / absmean_n(W[n,k]) (Def. 3.1); W: uint16 [N,K] bf16 bits."""
    W = _c(W_bf16_bits, np.uint16)
    N, K = W.shape
    lam = np.zeros((K,), dtype=np.float64)
    rc = _load().fqo_cas_scales(_ptr(W, ctypes.c_uint16), float(target), _ptr(lam, ctypes.c_double), N, K)
    if rc != 0:
        raise ValueError("fqo_cas_scales failed with %d" % rc)
    return lam


def _lambda_ptr(lam, K):
    if lam is None:
        return None, ctypes.POINTER(ctypes.c_float)()
    lam = _c(lam, np.float32)
    if lam.shape != (K,):
        raise ValueError("lambda must be float32 [K]")
    return lam, _ptr(lam, ctypes.c_float)


def scaled_weights(W_bf16_bits, lam=None) -> np.ndarray:
    """float32 [N,K]: bf16 W[n,k] * float32 lambda[k], rounded once to FP32 (lambda None: W itself)."""
    W = _c(W_bf16_bits, np.uint16)
    N, K = W.shape
    lam, lp = _lambda_ptr(lam, K)
    out = np.zeros((N, K), dtype=np.float32)
    _load().fqo_scaled_weights(_ptr(W, ctypes.c_uint16), lp, _ptr(out, ctypes.c_float), N, K)
    return out


def pts_exponent(W_bf16_bits, lam=None) -> int:
    """n of Def. 3.2 for the (channel-scaled) weights; delta = 2^n, the GEMM's w_tscale is 2^-n."""
    from . import pts
    return pts.pts_exponent(scaled_weights(W_bf16_bits, lam))


def quantize_weights(W_bf16_bits, lam=None, n_pts: int = 0, sigma_rne: bool = False):
    """(int8 [N,K] INT4 codes, uint8 [N,K/128] E4M3 group scales) of eq. 1 applied to W * lambda * 2^n."""
    W = _c(W_bf16_bits, np.uint16)
    N, K = W.shape
    lam, lp = _lambda_ptr(lam, K)
    q = np.zeros((N, K), dtype=np.int8)
    gs = np.zeros((N, K // 128), dtype=np.uint8)
    rc = _load().fqo_quantize_weights(_ptr(W, ctypes.c_uint16), lp, int(n_pts), 1 if sigma_rne else 0,
                                      _ptr(q, ctypes.c_int8), _ptr(gs, ctypes.c_uint8), N, K)
    if rc != 0:
        raise ValueError("fqo_quantize_weights failed with %d" % rc)
    return q, gs


def bf16_round_array(Y: np.ndarray) -> np.ndarray:
    """Elementwise nearest-even bf16 bit patterns (uint16) of an FP64 array."""
    flat = np.ascontiguousarray(Y, dtype=np.float64).ravel()
    out = np.empty(flat.shape, dtype=np.uint16)
    _load().fqo_bf16_encode_rne_array(_ptr(flat, ctypes.c_double), _ptr(out, ctypes.c_uint16), flat.size)
    return out.reshape(np.shape(Y))


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact FP64 value of bf16 bit patterns (a pure re-labelling of bits)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return b.view(np.float32).astype(np.float64)


def bf16_ulp_array(Y: np.ndarray) -> np.ndarray:
    """Elementwise size of one bf16 unit in the last place at each value's magnitude."""
    flat = np.ascontiguousarray(Y, dtype=np.float64).ravel()
    out = np.empty(flat.shape, dtype=np.float64)
    _load().fqo_bf16_ulp_array(_ptr(flat, ctypes.c_double), _ptr(out, ctypes.c_double), flat.size)
    return out.reshape(np.shape(Y))


def kv4_scores(Q, q_scale, Kq, k_scale, out_scale, want_bound: bool = False):
    """FP64 attention scores of FP8 queries against an INT4 key cache with one E4M3 scale per token (Sec. 3.2.1):
    ``S[h,r,t] = out_scale * q_scale[h,r] * e4m3(k_scale[h,t]) * sum_c e4m3(Q[h,r,c]) * Kq[h,t,c]``.
    Q uint8 [H,R,128], q_scale float32 [H,R], Kq int8 [H,T,128], k_scale uint8 [H,T]."""
    Q = _c(Q, np.uint8); q_scale = _c(q_scale, np.float32); Kq = _c(Kq, np.int8); k_scale = _c(k_scale, np.uint8)
    H, R, D = Q.shape
    T = Kq.shape[1]
    if D != 128 or Kq.shape != (H, T, 128) or q_scale.shape != (H, R) or k_scale.shape != (H, T):
        raise ValueError("operand shapes do not match")
    if Kq.size and (Kq.min() < -8 or Kq.max() > 7):
        raise ValueError("INT4 codes out of range")
    S = np.zeros((H, R, T), dtype=np.float64)
    B = np.zeros((H, R, T), dtype=np.float64) if want_bound else None
    rc = _load().fqo_kv4_scores(_ptr(Q, ctypes.c_uint8), _ptr(q_scale, ctypes.c_float), _ptr(Kq, ctypes.c_int8),
                                _ptr(k_scale, ctypes.c_uint8), ctypes.c_float(float(np.float32(out_scale))),
                                _ptr(S, ctypes.c_double),
                                _ptr(B, ctypes.c_double) if want_bound else ctypes.POINTER(ctypes.c_double)(), H, R, T)
    if rc != 0:
        raise ValueError("fqo_kv4_scores failed with %d" % rc)
    return (S, B) if want_bound else S


def kv4_output(P, p_scale, Vq, v_scale, want_bound: bool = False):
    """FP64 attention output of FP8 probabilities against an INT4 value cache with one E4M3 scale per token:
    ``O[h,r,c] = p_scale[h,r] * sum_t e4m3(P[h,r,t]) * e4m3(v_scale[h,t]) * Vq[h,t,c]``.
    P uint8 [H,R,T], p_scale float32 [H,R], Vq int8 [H,T,128], v_scale uint8 [H,T]."""
    P = _c(P, np.uint8); p_scale = _c(p_scale, np.float32); Vq = _c(Vq, np.int8); v_scale = _c(v_scale, np.uint8)
    H, R, T = P.shape
    if Vq.shape != (H, T, 128) or p_scale.shape != (H, R) or v_scale.shape != (H, T):
        raise ValueError("operand shapes do not match")
    if Vq.size and (Vq.min() < -8 or Vq.max() > 7):
        raise ValueError("INT4 codes out of range")
    O = np.zeros((H, R, 128), dtype=np.float64)
    B = np.zeros((H, R, 128), dtype=np.float64) if want_bound else None
    rc = _load().fqo_kv4_output(_ptr(P, ctypes.c_uint8), _ptr(p_scale, ctypes.c_float), _ptr(Vq, ctypes.c_int8),
                                _ptr(v_scale, ctypes.c_uint8), _ptr(O, ctypes.c_double),
                                _ptr(B, ctypes.c_double) if want_bound else ctypes.POINTER(ctypes.c_double)(), H, R, T)
    if rc != 0:
        raise ValueError("fqo_kv4_output failed with %d" % rc)
    return (O, B) if want_bound else O
