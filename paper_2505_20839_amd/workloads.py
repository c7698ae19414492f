"""Seeded synthetic inputs for the W4A8-FP GEMM: shapes and value distributions only.

This module holds none of the method's arithmetic (no quantiser, no GEMM, no packing); it
draws random numbers and converts them to storage formats with library casts.  It is the only
module the GPU path's tests and the CPU oracle's tests both use.

The shapes are the linear-layer shapes of the models the paper measures on (Sec. 4.1:
Llama2-7B hidden 4096 / FFN 11008; Llama3-8B hidden 4096 / FFN 14336, 32 query heads and
8 KV heads of 128 => fused QKV width 6144); activations are a Gaussian or Laplace body with a
few strong outlier channels, the qualitative picture of Sec. 1 and Sec. 2.2.  No model
weights or dataset are involved.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
import torch

GROUP = 128


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    N: int
    K: int
    act: str            # "gauss" | "laplace"
    outlier_frac: float  # fraction of K columns multiplied by 20
    gs_lo: float
    gs_hi: float
    w_tscale: float
    seed: int
    epilogue: str = "none"   # "swiglu": the N weight rows interleave gate (even) and up (odd) channels;
                             # "add": a residual [M,N] is added to the result (draw_residual)


def _w(name, M, N, K, act, frac, lo, hi, t, seed, epilogue="none"):
    return Workload(name, M, N, K, act, frac, lo, hi, t, seed, epilogue)


# The five benchmark configurations (config 4 has two shapes, config 5 four batch sizes).
WORKLOADS: Dict[str, Workload] = {w.name: w for w in [
    _w("c1_tiny",          16,   256,   512, "gauss",   0.0,  0.01,  0.1,  0.5, 0),
    _w("c2_l2_7b_gateup", 2048, 11008,  4096, "gauss",   0.01, 0.005, 0.05, 1.0, 1),
    _w("c3_l2_7b_down",   2048,  4096, 11008, "gauss",   0.01, 0.005, 0.05, 1.0, 2),
    _w("c4a_l3_8b_qkv",   8192,  6144,  4096, "laplace", 0.01, 0.005, 0.05, 1.0, 3),
    _w("c4b_l3_8b_up",    8192, 14336,  4096, "laplace", 0.01, 0.005, 0.05, 1.0, 4),
    _w("c5_decode_m1",       1, 14336,  4096, "gauss",   0.0,  0.005, 0.05, 1.0, 5),
    _w("c5_decode_m4",       4, 14336,  4096, "gauss",   0.0,  0.005, 0.05, 1.0, 6),
    _w("c5_decode_m16",     16, 14336,  4096, "gauss",   0.0,  0.005, 0.05, 1.0, 7),
    _w("c5_decode_m64",     64, 14336,  4096, "gauss",   0.0,  0.005, 0.05, 1.0, 8),
    # beyond the five configurations: gate and up projection of the Llama2-7B feed-forward block in one
    # GEMM (rows interleaved) with the SiLU(gate) * up epilogue fused (Sec. 3.1.1 step 3)
    _w("ffn_l2_7b_gateup_swiglu", 2048, 22016, 4096, "gauss", 0.01, 0.005, 0.05, 1.0, 9, "swiglu"),
    # the down projection of the same block with the residual stream added in the epilogue (step 3)
    _w("ffn_l2_7b_down_residual", 2048, 4096, 11008, "gauss", 0.01, 0.005, 0.05, 1.0, 10, "add"),
    # between decode and prefill (batched decode, chunked prefill): the up projection and the down projection
    # of configuration 4 / 3 at 128, 256 and 512 rows
    _w("mid_l3_8b_up_m128",   128, 14336,  4096, "gauss", 0.01, 0.005, 0.05, 1.0, 11),
    _w("mid_l3_8b_up_m256",   256, 14336,  4096, "gauss", 0.01, 0.005, 0.05, 1.0, 12),
    _w("mid_l3_8b_up_m512",   512, 14336,  4096, "gauss", 0.01, 0.005, 0.05, 1.0, 13),
    _w("mid_l2_7b_down_m128", 128,  4096, 11008, "gauss", 0.01, 0.005, 0.05, 1.0, 14),
    _w("mid_l2_7b_down_m256", 256,  4096, 11008, "gauss", 0.01, 0.005, 0.05, 1.0, 15),
    _w("mid_l2_7b_down_m512", 512,  4096, 11008, "gauss", 0.01, 0.005, 0.05, 1.0, 16),
]}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bf16 bit patterns (torch's round-to-nearest-even cast)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def f32_to_e4m3_codes(x: np.ndarray) -> np.ndarray:
    """float32 array (|x| <= 448) -> uint8 OCP E4M3 codes (torch's nearest-even cast)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.float8_e4m3fn)
    return t.view(torch.uint8).numpy().copy()


def draw(M: int, N: int, K: int, *, seed: int, act: str = "gauss", outlier_frac: float = 0.0,
         gs_lo: float = 0.005, gs_hi: float = 0.05, w_tscale: float = 1.0,
         rows: Optional[int] = None):
    """Draw one problem.  Order of draws: activations, weight codes, group scales.

    Returns a dict with
      X_bf16  uint16 [M,K]   activations before quantisation (bf16 bit patterns)
      q       int8   [N,K]   INT4 weight codes, uniform on -8..7
      gscale  uint8  [N,K/128]  E4M3 codes of U[gs_lo, gs_hi] draws
      w_tscale float
    `rows` keeps only the first `rows` activation rows (same stream, so they equal the rows of
    the full problem) -- used to sample a large configuration.
    """
    if K % GROUP:
        raise ValueError("K must be a multiple of 128")
    rng = np.random.default_rng(seed)
    if act == "gauss":
        X = rng.standard_normal((M, K), dtype=np.float32)
    elif act == "laplace":
        X = rng.laplace(0.0, 1.0, (M, K)).astype(np.float32)
    else:
        raise ValueError(act)
    n_out = int(round(outlier_frac * K))
    if n_out:
        cols = rng.choice(K, size=n_out, replace=False)
        X[:, cols] *= 20.0
    q = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    gs = rng.uniform(gs_lo, gs_hi, size=(N, K // GROUP)).astype(np.float32)
    if rows is not None:
        X = X[:rows]
    return {
        "X_bf16": f32_to_bf16_bits(X),
        "q": q,
        "gscale": f32_to_e4m3_codes(gs),
        "w_tscale": float(w_tscale),
    }


RESIDUAL_SCALE = 16.0     # about the standard deviation of the GEMM outputs of the "add" workload


def draw_residual(M: int, N: int, *, scale: float, seed: int) -> np.ndarray:
    """uint16 [M,N] bf16 bit patterns of N(0, scale^2) draws: the residual stream an "add" epilogue takes.
    A stream of its own, so that the other operands of a problem do not depend on it."""
    rng = np.random.default_rng([seed, 0x5EED])
    return f32_to_bf16_bits(rng.standard_normal((M, N), dtype=np.float32) * np.float32(scale))


def draw_weights(N: int, K: int, *, seed: int, std: float = 0.02, channel_spread: float = 0.5,
                 zero_frac: float = 0.0) -> np.ndarray:
    """uint16 [N,K] bf16 bit patterns of a synthetic weight matrix for the offline quantiser: N(0, std^2)
    entries, input channel k scaled by a log-normal factor exp(channel_spread * N(0,1)) (the uneven
    channel magnitudes that channel-wise scaling evens out), a fraction `zero_frac` of entries set to zero."""
    rng = np.random.default_rng([seed, 0xBEEF])
    W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(std)
    W *= np.exp(channel_spread * rng.standard_normal((1, K))).astype(np.float32)
    if zero_frac > 0:
        W[rng.random((N, K)) < zero_frac] = 0.0
    return f32_to_bf16_bits(W)


def draw_workload(name: str, rows: Optional[int] = None):
    w = WORKLOADS[name]
    return draw(w.M, w.N, w.K, seed=w.seed, act=w.act, outlier_frac=w.outlier_frac,
                gs_lo=w.gs_lo, gs_hi=w.gs_hi, w_tscale=w.w_tscale, rows=rows)


def draw_kv_cache(H: int, R: int, T: int, *, seed: int):
    """Operands of decode attention with an INT4 key/value cache (Sec. 3.2.1): shapes and value distributions only.

    H key/value heads of width 128 (Llama heads), R query rows per head, T cached tokens.  Returns
      Q_bf16, P_bf16  uint16 [H,R,128] / [H,R,T]  queries N(0,1) and attention probabilities (softmax of N(0, 2^2)
                      logits) before their FP8 quantisation (bf16 bit patterns)
      Kq, Vq          int8 [H,T,128]  INT4 codes, uniform on -8..7
      k_scale, v_scale uint8 [H,T]    E4M3 codes of U[0.02, 0.2] draws (one per token)
    """
    rng = np.random.default_rng([seed, 0xA77])
    Q = rng.standard_normal((H, R, GROUP), dtype=np.float32)
    logits = 2.0 * rng.standard_normal((H, R, T), dtype=np.float32)
    P = np.exp(logits - logits.max(axis=2, keepdims=True))
    P /= P.sum(axis=2, keepdims=True)
    Kq = rng.integers(-8, 8, size=(H, T, GROUP), dtype=np.int8)
    Vq = rng.integers(-8, 8, size=(H, T, GROUP), dtype=np.int8)
    ks = rng.uniform(0.02, 0.2, size=(H, T)).astype(np.float32)
    vs = rng.uniform(0.02, 0.2, size=(H, T)).astype(np.float32)
    return {"Q_bf16": f32_to_bf16_bits(Q), "P_bf16": f32_to_bf16_bits(P.astype(np.float32)), "Kq": Kq, "Vq": Vq,
            "k_scale": f32_to_e4m3_codes(ks), "v_scale": f32_to_e4m3_codes(vs)}
