"""Pins for the oracle's GEMM with the residual added in the epilogue (Sec. 3.1.1 step 3, the
activation addition; Fig. 1 shows it after the attention-output and the down projections): hand
values, the two special cases that reduce it to functions pinned elsewhere, and the index order of
the residual.  No GPU here."""
import numpy as np
import pytest

import oracle

ONE, TWO = 0x38, 0x40


def _bf16_bits(x):
    """bf16 bit patterns of floats that are exactly representable (top 16 bits of the binary32)."""
    b = np.asarray(x, np.float32).view(np.uint32)
    assert np.all((b & 0xFFFF) == 0)
    return (b >> 16).astype(np.uint16)


def _operands(rng, M, N, K):
    A = rng.integers(0, 0x48, (M, K)).astype(np.uint8) | (rng.integers(0, 2, (M, K)).astype(np.uint8) << 7)
    q = rng.integers(-8, 8, (N, K), dtype=np.int8)
    gs = rng.integers(0x10, 0x30, (N, K // 128)).astype(np.uint8)
    a = rng.uniform(0.01, 0.1, M).astype(np.float32)
    return A, a, q, gs


def test_hand_values():
    # one non-zero product: 1 * (3 * 2) = 6, times a_scale 0.5 and w_tscale 0.25 = 0.75; residual 1.5, -0.75
    A = np.zeros((1, 128), np.uint8); A[0, 5] = ONE
    q = np.zeros((2, 128), np.int8); q[0, 5] = 3; q[1, 5] = 3
    gs = np.array([[TWO], [TWO]], np.uint8)
    R = _bf16_bits([[1.5, -0.75]])
    Y = oracle.w4a8_gemm_add(A, np.array([0.5], np.float32), q, gs, 0.25, R)
    assert Y.tolist() == [[2.25, 0.0]]


def test_zero_residual_is_the_plain_gemm():
    rng = np.random.default_rng(3)
    A, a, q, gs = _operands(rng, 4, 6, 256)
    R = np.zeros((4, 6), np.uint16)
    R[1, 2] = 0x8000                                                     # -0 adds nothing either
    Y0, B0 = oracle.w4a8_gemm(A, a, q, gs, 0.5, want_bound=True)
    Y1, B1 = oracle.w4a8_gemm_add(A, a, q, gs, 0.5, R, want_bound=True)
    assert np.array_equal(Y0, Y1) and np.array_equal(B0, B1)


def test_zero_weights_return_the_residual():
    rng = np.random.default_rng(4)
    A, a, _, gs = _operands(rng, 3, 5, 128)
    q = np.zeros((5, 128), np.int8)
    R = rng.integers(0, 0x7F80, (3, 5)).astype(np.uint16) | (rng.integers(0, 2, (3, 5)).astype(np.uint16) << 15)
    Y = oracle.w4a8_gemm_add(A, a, q, gs, 2.0, R)
    assert np.array_equal(Y, oracle.bf16_bits_to_f64(R))                 # a bf16 is its top 16 binary32 bits


def test_residual_is_indexed_row_major_m_by_n():
    # a residual with a single non-zero entry moves exactly that output, in a non-square problem
    rng = np.random.default_rng(5)
    M, N, K = 3, 7, 128
    A, a, q, gs = _operands(rng, M, N, K)
    Y0 = oracle.w4a8_gemm(A, a, q, gs, 1.0)
    for (m, n) in [(0, 6), (2, 0), (1, 3)]:
        R = np.zeros((M, N), np.uint16)
        R[m, n] = _bf16_bits(1024.0)                                     # large against the sums' rounding
        D = oracle.w4a8_gemm_add(A, a, q, gs, 1.0, R) - Y0
        E = np.zeros((M, N)); E[m, n] = 1024.0
        assert np.allclose(D, E, rtol=0, atol=1e-9)


def test_equals_numpy_sum():
    rng = np.random.default_rng(6)
    A, a, q, gs = _operands(rng, 6, 10, 384)
    Rf = rng.standard_normal((6, 10)).astype(np.float32)
    R = (Rf.view(np.uint32) >> 16).astype(np.uint16)                     # truncation: any bf16 will do
    Y = oracle.w4a8_gemm_add(A, a, q, gs, 0.5, R)
    want = oracle.w4a8_gemm(A, a, q, gs, 0.5) + (R.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(Y, want)


def test_shape_errors():
    rng = np.random.default_rng(7)
    A, a, q, gs = _operands(rng, 2, 4, 128)
    with pytest.raises(ValueError):
        oracle.w4a8_gemm_add(A, a, q, gs, 1.0, np.zeros((4, 2), np.uint16))
    with pytest.raises(TypeError):
        oracle.w4a8_gemm_add(A, a, q, gs, 1.0, np.zeros((2, 4), np.float32))


def test_linear_is_the_quantiser_followed_by_the_gemm():
    """oracle.w4a8_linear: hand value (row [2, -1]: beta = 2/448, codes 448 and -224, both weights 1 and the
    group scale 1 give beta * 224 = 1) and equality with the two pinned functions it chains."""
    X = np.zeros((1, 128), np.float32); X[0, 0] = 2.0; X[0, 1] = -1.0
    q = np.zeros((1, 128), np.int8); q[0, 0] = 1; q[0, 1] = 1
    gs = np.array([[ONE]], np.uint8)
    Y = oracle.w4a8_linear(_bf16_bits(X), q, gs, 1.0)
    assert Y.shape == (1, 1) and abs(Y[0, 0] - 1.0) < 1e-7
    rng = np.random.default_rng(12)
    Xb = (rng.standard_normal((5, 256)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    q = rng.integers(-8, 8, (9, 256), dtype=np.int8)
    gs = rng.integers(0x10, 0x30, (9, 2)).astype(np.uint8)
    A, s = oracle.quantize_act(Xb)
    assert np.array_equal(oracle.w4a8_linear(Xb, q, gs, 0.5), oracle.w4a8_gemm(A, s, q, gs, 0.5))
