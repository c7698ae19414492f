"""Pins for the oracle's fused gate/up epilogue (Sec. 3.1.1 step 3: SiLU and the element-wise
product applied to the GEMM result): hand values, closed forms, the composition of the pinned
GEMM oracle with a library sigmoid, the row interleave, and the error bound.  No GPU here."""
import math

import numpy as np
import pytest
from scipy.special import expit

import oracle

ONE, TWO, THREE, HALF = 0x38, 0x40, 0x44, 0x30


def _pair(g_val_code, u_val_code, qg, qu, K=128):
    """One row of A with a single non-zero element, gate row 0 / up row 1 with single weights."""
    A = np.zeros((1, K), np.uint8); A[0, 3] = ONE
    q = np.zeros((2, K), np.int8); q[0, 3] = qg; q[1, 3] = qu
    gs = np.array([[g_val_code], [u_val_code]], np.uint8)
    return A, np.ones(1, np.float32), q, gs


def test_hand_values():
    # gate = 1 * 1 * 1 = 1, up = 1 * 3 * 2 = 6:  SiLU(1) = 1 / (1 + e^-1) = 0.7310585786300049
    A, a, q, gs = _pair(ONE, TWO, 1, 3)
    H = oracle.w4a8_gemm_swiglu(A, a, q, gs, 1.0)
    assert H.shape == (1, 1)
    assert H[0, 0] == pytest.approx(0.7310585786300049 * 6.0, rel=1e-15)
    # gate = 0: SiLU(0) = 0 whatever up is
    A, a, q, gs = _pair(ONE, TWO, 0, 7)
    assert oracle.w4a8_gemm_swiglu(A, a, q, gs, 1.0)[0, 0] == 0.0
    # gate = -1 * 0.5 = -0.5, up = -2: SiLU(-0.5) = -0.5 / (1 + e^0.5) = -0.18877033439907276
    A, a, q, gs = _pair(HALF, ONE, -1, -2)
    assert oracle.w4a8_gemm_swiglu(A, a, q, gs, 1.0)[0, 0] == pytest.approx(-0.18877033439907276 * -2.0, rel=1e-15)


def test_saturation_limits():
    # large positive gate: SiLU(x) -> x; large negative: -> 0 from below
    A = np.zeros((1, 128), np.uint8); A[0, :] = 0x7E                      # 448 everywhere
    q = np.zeros((2, 128), np.int8); q[0, :] = 7; q[1, 0] = 1
    gs = np.array([[ONE], [ONE]], np.uint8)
    a = np.ones(1, np.float32)
    g = 448.0 * 7 * 128
    assert oracle.w4a8_gemm_swiglu(A, a, q, gs, 1.0)[0, 0] == g * 448.0
    q[0, :] = -7
    h = oracle.w4a8_gemm_swiglu(A, a, q, gs, 1.0)[0, 0]
    assert h == 0.0 or (h < 0 and abs(h) < 1e-300)                          # -g * e^-|g| * u underflows


def test_equals_composition_with_library_sigmoid():
    rng = np.random.default_rng(11)
    M, N, K = 5, 12, 256
    A = rng.integers(0, 0x48, (M, K)).astype(np.uint8) | (rng.integers(0, 2, (M, K)).astype(np.uint8) << 7)
    q = rng.integers(-8, 8, (N, K), dtype=np.int8)
    gs = rng.integers(0x10, 0x30, (N, K // 128)).astype(np.uint8)
    a = rng.uniform(0.01, 0.1, M).astype(np.float32)                        # keeps the gates of order one
    Y, B = oracle.w4a8_gemm(A, a, q, gs, 0.5, want_bound=True)
    H, HB = oracle.w4a8_gemm_swiglu(A, a, q, gs, 0.5, want_bound=True)
    g, u = Y[:, 0::2], Y[:, 1::2]
    assert np.abs(g).max() > 0.5 and np.abs(g).min() < 5                    # the nonlinear range is exercised
    want = g * expit(g) * u                                                 # x * sigmoid(x) = x / (1 + e^-x)
    np.testing.assert_allclose(H, want, rtol=1e-14, atol=0)
    np.testing.assert_allclose(HB, 1.1 * np.abs(u) * B[:, 0::2] + np.abs(g * expit(g)) * B[:, 1::2], rtol=1e-13)


def test_rows_are_interleaved_gate_first():
    # swapping the roles of the two rows changes the result (SiLU is applied to the even row only);
    # a split-halves reading (gate rows first, then all up rows) would pair row 0 with row 2 here
    A = np.zeros((1, 128), np.uint8); A[0, 0] = ONE
    q = np.zeros((4, 128), np.int8); q[:, 0] = [1, 2, 3, 4]
    gs = np.full((4, 1), ONE, np.uint8)
    a = np.ones(1, np.float32)
    H = oracle.w4a8_gemm_swiglu(A, a, q, gs, 1.0)
    silu = lambda x: x / (1.0 + math.exp(-x))
    assert H.shape == (1, 2)
    assert H[0, 0] == pytest.approx(silu(1.0) * 2.0, rel=1e-15)
    assert H[0, 1] == pytest.approx(silu(3.0) * 4.0, rel=1e-15)
    assert abs(H[0, 0] - silu(2.0) * 1.0) > 0.1 and abs(H[0, 0] - silu(1.0) * 3.0) > 0.1


def test_bound_covers_perturbed_sums():
    """The bound is first order: perturbing the two sums by a small fraction of their own bounds moves
    H by no more than that fraction of the bound (plus second-order terms)."""
    rng = np.random.default_rng(5)
    g = rng.normal(0, 3, 2000); u = rng.normal(0, 3, 2000)
    eg = rng.uniform(0, 1e-6, 2000); eu = rng.uniform(0, 1e-6, 2000)
    silu = lambda x: x * expit(x)
    for sg in (-1, 1):
        for su in (-1, 1):
            d = np.abs(silu(g + sg * eg) * (u + su * eu) - silu(g) * u)
            assert np.all(d <= (1.1 * np.abs(u) * eg + np.abs(silu(g)) * eu) * (1 + 1e-3) + 1e-11)


def test_shapes_and_errors():
    A = np.zeros((2, 128), np.uint8)
    with pytest.raises(ValueError):
        oracle.w4a8_gemm_swiglu(A, np.ones(2, np.float32), np.zeros((3, 128), np.int8), np.zeros((3, 1), np.uint8), 1.0)
