"""Pins for the oracle's GEMM against hand-worked values, closed forms, a library matmul on
library-decoded operands, exact rational arithmetic, and invariants of the definition
(Sec. 2.2 eq. 3 with the operand formats of Sec. 2.1 / 3.1 and the delta^-1 output scale of
Def. 3.2).  Nothing here calls the GPU."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2505_20839_amd import workloads

ONE, TWO, THREE, HALF, QUARTER = 0x38, 0x40, 0x44, 0x30, 0x28


def _lib_e4m3(codes: np.ndarray) -> np.ndarray:
    """E4M3 decode done by the library cast, not by the oracle."""
    t = torch.from_numpy(np.ascontiguousarray(codes, dtype=np.uint8))
    return t.view(torch.float8_e4m3fn).to(torch.float64).numpy()


def _rand_problem(M, N, K, seed, *, signed_scales=False):
    rng = np.random.default_rng(seed)
    A = rng.integers(0, 0x7F, (M, K)).astype(np.uint8) | (rng.integers(0, 2, (M, K)).astype(np.uint8) << 7)
    q = rng.integers(-8, 8, (N, K), dtype=np.int8)
    gs = rng.integers(0, 0x40, (N, K // 128)).astype(np.uint8)
    if signed_scales:
        gs |= (rng.integers(0, 2, gs.shape).astype(np.uint8) << 7)
    a = rng.uniform(0.01, 2.0, M).astype(np.float32)
    t = float(np.float32(rng.uniform(0.1, 3.0)))
    return A, a, q, gs, t


# ---- hand-worked tiny cases (expected values written out by hand) ---------------------------

def test_single_product():
    A = np.zeros((1, 128), np.uint8); A[0, 5] = THREE
    q = np.full((1, 128), 3, np.int8); q[0, 5] = -7
    gs = np.array([[HALF]], np.uint8)
    Y = oracle.w4a8_gemm(A, np.array([2.0], np.float32), q, gs, 0.25)
    assert Y.shape == (1, 1) and Y[0, 0] == -5.25            # 2 * 0.25 * 0.5 * (3 * -7)


def test_two_groups_two_scales():
    A = np.zeros((1, 256), np.uint8); A[0, 0] = ONE; A[0, 128] = TWO
    q = np.zeros((1, 256), np.int8); q[0, 0] = 5; q[0, 128] = -8
    gs = np.array([[ONE, QUARTER]], np.uint8)
    Y = oracle.w4a8_gemm(A, np.array([1.0], np.float32), q, gs, 1.0)
    assert Y[0, 0] == 1.0                                    # 1*5*1 + 2*(-8)*0.25


def test_subnormal_operands_and_negative_code():
    A = np.zeros((1, 128), np.uint8); A[0, 127] = 0x03       # 3 * 2^-9
    q = np.zeros((1, 128), np.int8); q[0, 127] = -8
    gs = np.array([[0x05]], np.uint8)                        # 5 * 2^-9
    Y = oracle.w4a8_gemm(A, np.array([1.0], np.float32), q, gs, 1.0)
    assert Y[0, 0] == -120.0 / 262144.0


def test_zero_scale_group_contributes_nothing():
    # App. B, Lemma B.1: an underflowed group has sigma = 0 and dequantises to zero.
    A = np.full((1, 256), ONE, np.uint8)
    q = np.full((1, 256), 7, np.int8)
    gs = np.array([[ONE, 0x00]], np.uint8)
    Y = oracle.w4a8_gemm(A, np.array([1.0], np.float32), q, gs, 1.0)
    assert Y[0, 0] == 7.0 * 128


def test_two_by_three_by_two_groups_indexing():
    # Distinct values everywhere so that a swapped index (m<->n, n<->g, A<->q) changes the result.
    M, N, K = 2, 3, 256
    A = np.zeros((M, K), np.uint8); q = np.zeros((N, K), np.int8)
    A[0, 1] = ONE;  A[0, 130] = TWO          # row 0: 1 at k=1 (g0), 2 at k=130 (g1)
    A[1, 1] = THREE; A[1, 200] = HALF        # row 1: 3 at k=1 (g0), 0.5 at k=200 (g1)
    q[0, 1] = 1; q[0, 130] = 2; q[0, 200] = 4
    q[1, 1] = -3; q[1, 130] = 5; q[1, 200] = -6
    q[2, 1] = 7; q[2, 130] = -8; q[2, 200] = 2
    gs = np.array([[ONE, TWO], [HALF, ONE], [TWO, QUARTER]], np.uint8)  # [n, g]
    a = np.array([1.0, 2.0], np.float32)
    Y = oracle.w4a8_gemm(A, a, q, gs, 0.5)
    want = np.array([
        # m=0: 0.5 * 1 * (s[n,0]*1*q[n,1] + s[n,1]*2*q[n,130])
        [0.5 * (1 * 1 + 2 * 2 * 2), 0.5 * (0.5 * -3 + 1 * 2 * 5), 0.5 * (2 * 7 + 0.25 * 2 * -8)],
        # m=1: 0.5 * 2 * (s[n,0]*3*q[n,1] + s[n,1]*0.5*q[n,200])
        [1.0 * (1 * 3 * 1 + 2 * 0.5 * 4), 1.0 * (0.5 * 3 * -3 + 1 * 0.5 * -6), 1.0 * (2 * 3 * 7 + 0.25 * 0.5 * 2)],
    ])
    assert np.array_equal(Y, want)
    assert want.tolist() == [[4.5, 4.25, 5.0], [7.0, -7.5, 42.25]]


# ---- closed forms ------------------------------------------------------------------------------

@pytest.mark.parametrize("K", [128, 512, 1408])
def test_all_ones_gives_K(K):
    M, N = 3, 5
    Y = oracle.w4a8_gemm(np.full((M, K), ONE, np.uint8), np.ones(M, np.float32),
                         np.ones((N, K), np.int8), np.full((N, K // 128), ONE, np.uint8), 1.0)
    assert np.all(Y == K)


def test_extremes():
    K = 384
    Y = oracle.w4a8_gemm(np.full((2, K), 0x7E, np.uint8), np.ones(2, np.float32),
                         np.full((2, K), -8, np.int8), np.full((2, 3), ONE, np.uint8), 1.0)
    assert np.all(Y == -3584.0 * K)


def test_one_hot_A_reads_back_every_weight_and_scale():
    K = 256; M = K; N = 6
    _, a, q, gs, t = _rand_problem(M, N, K, 3)
    A = np.zeros((M, K), np.uint8); A[np.arange(M), np.arange(K)] = ONE
    Y = oracle.w4a8_gemm(A, a, q, gs, t)
    s = _lib_e4m3(gs)
    for m in range(M):
        for n in range(N):
            want = float(a[m]) * t * (s[n, m // 128] * float(q[n, m]))
            assert Y[m, n] == pytest.approx(want, rel=1e-15, abs=0)


def test_one_hot_weights_read_back_A():
    K = 256; N = K; M = 4
    A, a, _, _, _ = _rand_problem(M, N, K, 4)
    q = np.zeros((N, K), np.int8); q[np.arange(N), np.arange(K)] = 1
    gs = np.full((N, 2), ONE, np.uint8)
    Y = oracle.w4a8_gemm(A, np.ones(M, np.float32), q, gs, 1.0)
    assert np.array_equal(Y, _lib_e4m3(A))


# ---- reduces to a library routine: dense dequantised matmul ---------------------------------

@pytest.mark.parametrize("shape,seed", [((7, 9, 128), 0), ((33, 50, 640), 1), ((64, 130, 1408), 2)])
def test_matches_dense_float64_matmul(shape, seed):
    M, N, K = shape
    A, a, q, gs, t = _rand_problem(M, N, K, seed, signed_scales=True)
    Y, B = oracle.w4a8_gemm(A, a, q, gs, t, want_bound=True)
    Wd = t * np.repeat(_lib_e4m3(gs), 128, axis=1) * q.astype(np.float64)      # [N,K]
    Yd = (a.astype(np.float64)[:, None] * _lib_e4m3(A)) @ Wd.T
    assert np.all(np.abs(Y - Yd) <= 1e-12 * B + 1e-300)
    Bd = (np.abs(a.astype(np.float64))[:, None] * np.abs(_lib_e4m3(A))) @ np.abs(Wd).T
    assert np.allclose(B, Bd, rtol=1e-12, atol=0)
    assert np.all(B >= np.abs(Y))


# ---- exact rational arithmetic on tiny shapes ------------------------------------------------

@pytest.mark.parametrize("shape,seed", [((2, 3, 128), 5), ((4, 4, 256), 6), ((3, 8, 256), 7)])
def test_matches_exact_rationals(shape, seed):
    M, N, K = shape
    A, a, q, gs, t = _rand_problem(M, N, K, seed, signed_scales=True)
    Y, B = oracle.w4a8_gemm(A, a, q, gs, t, want_bound=True)
    Af = [[Fraction(v) for v in row] for row in _lib_e4m3(A).tolist()]
    Sf = [[Fraction(v) for v in row] for row in _lib_e4m3(gs).tolist()]
    tf = Fraction(float(np.float32(t)))
    for m in range(M):
        for n in range(N):
            tot = Fraction(0)
            for g in range(K // 128):
                p = sum(Af[m][k] * int(q[n, k]) for k in range(128 * g, 128 * g + 128))
                tot += Sf[n][g] * p
            exact = Fraction(float(a[m])) * tf * tot
            assert abs(Fraction(Y[m, n]) - exact) <= Fraction(1, 10 ** 15) * Fraction(B[m, n])


# ---- invariants of the definition ---------------------------------------------------------------

def test_invariants():
    M, N, K = 6, 10, 512
    A, a, q, gs, t = _rand_problem(M, N, K, 8)
    Y = oracle.w4a8_gemm(A, a, q, gs, t)
    # delta is a power of two (Def. 3.2): doubling delta^-1 doubles Y exactly
    assert np.array_equal(oracle.w4a8_gemm(A, a, q, gs, 2 * t), 2 * Y)
    # permuting output channels permutes columns
    perm = np.random.default_rng(0).permutation(N)
    assert np.array_equal(oracle.w4a8_gemm(A, a, q[perm], gs[perm], t), Y[:, perm])
    # permuting k inside each group, the same way in A and W, changes nothing (sums are exact)
    kp = np.concatenate([g * 128 + np.random.default_rng(g).permutation(128) for g in range(K // 128)])
    assert np.array_equal(oracle.w4a8_gemm(A[:, kp], a, q[:, kp], gs, t), Y)
    # a row of Y depends on that row of A only
    assert np.array_equal(oracle.w4a8_gemm(A[2:3], a[2:3], q, gs, t), Y[2:3])
    # appending a zero activation group with arbitrary weights changes nothing
    A2 = np.concatenate([A, np.zeros((M, 128), np.uint8)], axis=1)
    q2 = np.concatenate([q, np.full((N, 128), -5, np.int8)], axis=1)
    gs2 = np.concatenate([gs, np.full((N, 1), 0x3F, np.uint8)], axis=1)
    assert np.array_equal(oracle.w4a8_gemm(A2, a, q2, gs2, t), Y)
    # K not a multiple of the group is rejected
    with pytest.raises(ValueError):
        oracle.w4a8_gemm(A[:, :100], a, q[:, :100], gs[:, :0], t)


def test_channel_scaling_equivalence():
    # Sec. 3.1.2 eq. 6: (X Lambda^-1)(Lambda W)^T = X W^T.  With lambda_k = 2 on chosen input
    # channels both scaled operands stay representable, so equality is exact.
    M, N, K = 5, 7, 256
    rng = np.random.default_rng(9)
    A = rng.integers(0x10, 0x7F, (M, K)).astype(np.uint8)     # exponent field >= 2: halving is exact
    q = rng.integers(-4, 4, (N, K), dtype=np.int8)             # doubling stays within -8..7
    gs = rng.integers(1, 0x40, (N, 2)).astype(np.uint8)
    a = rng.uniform(0.5, 1.5, M).astype(np.float32)
    cols = rng.choice(K, 40, replace=False)
    A2 = A.copy(); A2[:, cols] -= 8                            # exponent - 1  == value / 2
    q2 = q.copy(); q2[:, cols] *= 2
    assert np.array_equal(_lib_e4m3(A2[:, cols]), _lib_e4m3(A[:, cols]) / 2)
    assert np.array_equal(oracle.w4a8_gemm(A2, a, q2, gs, 1.0), oracle.w4a8_gemm(A, a, q, gs, 1.0))


def test_config1_shape_runs_and_rounds_once():
    d = workloads.draw_workload("c1_tiny")
    A, s = oracle.quantize_act(d["X_bf16"])
    Y, B = oracle.w4a8_gemm(A, s, d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    assert Y.shape == (16, 256)
    Yb = oracle.bf16_bits_to_f64(oracle.bf16_round_array(Y))
    assert np.all(np.abs(Yb - Y) <= 0.5 * oracle.bf16_ulp_array(Y))
    rel = np.linalg.norm(Yb - Y) / np.linalg.norm(Y)
    assert rel < 2e-3                                           # one bf16 rounding fits the budget
