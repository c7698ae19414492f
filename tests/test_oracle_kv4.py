"""Pins for the oracle's attention operands (Sec. 3.2.1: FP8 queries, INT4 keys and values with one FP8 scale per
token; Sec. 3.1.1: the INT4 x FP8 product also forms S = Q K^T and O = P V).  No GPU here."""
from fractions import Fraction

import numpy as np
import torch

import oracle

ONE, TWO, HALF = 0x38, 0x40, 0x30


def _e4m3(codes):
    """library decode (torch's float8_e4m3fn), independent of the oracle's closed form"""
    return torch.from_numpy(np.ascontiguousarray(codes)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def _rand(H, R, T, seed):
    rng = np.random.default_rng(seed)
    def codes(shape, top=0x78):
        return rng.integers(0, top, shape).astype(np.uint8) | (rng.integers(0, 2, shape).astype(np.uint8) << 7)
    Q = codes((H, R, 128)); P = rng.integers(0, 0x60, (H, R, T)).astype(np.uint8)       # probabilities are non-negative
    Kq = rng.integers(-8, 8, (H, T, 128), dtype=np.int8); Vq = rng.integers(-8, 8, (H, T, 128), dtype=np.int8)
    ks = codes((H, T), 0x50); vs = codes((H, T), 0x50)
    qs = rng.uniform(0.01, 2, (H, R)).astype(np.float32); ps = rng.uniform(0.001, 0.1, (H, R)).astype(np.float32)
    return Q, qs, Kq, ks, P, ps, Vq, vs


def test_scores_hand_values():
    # one head, one query row, two tokens: Q = 2 at dim 5 and 0.5 at dim 9
    Q = np.zeros((1, 1, 128), np.uint8); Q[0, 0, 5] = TWO; Q[0, 0, 9] = HALF
    Kq = np.zeros((1, 2, 128), np.int8); Kq[0, 0, 5] = 3; Kq[0, 0, 9] = -8; Kq[0, 1, 5] = -1; Kq[0, 1, 100] = 7
    ks = np.array([[HALF, 0x03]], np.uint8)                    # 0.5 and the subnormal 3 * 2^-9
    S = oracle.kv4_scores(Q, np.array([[4.0]], np.float32), Kq, ks, 0.25)
    # token 0: 0.25 * 4 * 0.5 * (2*3 + 0.5*(-8)) = 1 ; token 1: 0.25 * 4 * 3*2^-9 * (2*(-1)) = -6 * 2^-9
    assert S.shape == (1, 1, 2) and S[0, 0, 0] == 1.0 and S[0, 0, 1] == -6.0 * 2.0 ** -9


def test_output_hand_values():
    # two tokens with different scales: the factor of a token multiplies that token's term only
    P = np.array([[[ONE, HALF]]], np.uint8)                    # probabilities 1 and 0.5
    Vq = np.zeros((1, 2, 128), np.int8); Vq[0, 0, 7] = 5; Vq[0, 1, 7] = -3; Vq[0, 1, 8] = 7
    vs = np.array([[TWO, 0x3C]], np.uint8)                     # 2 and 1.5
    O = oracle.kv4_output(P, np.array([[0.5]], np.float32), Vq, vs)
    assert O[0, 0, 7] == 0.5 * (1 * 2 * 5 + 0.5 * 1.5 * -3) and O[0, 0, 8] == 0.5 * (0.5 * 1.5 * 7)
    assert not O[0, 0, :7].any() and not O[0, 0, 9:].any()
    # a swapped scale (token 0's factor on token 1) would give 0.5 * (1.5*5 - 0.5*2*3) instead
    assert O[0, 0, 7] != 0.5 * (1 * 1.5 * 5 + 0.5 * 2 * -3)


def test_scores_are_the_linear_layer_with_one_group_per_token():
    """A head's score matrix is the W4A8 GEMM (pinned on its own) whose weight rows are the tokens and whose single
    group per row carries the token's scale; out_scale takes the place of the per-tensor factor."""
    Q, qs, Kq, ks, *_ = _rand(3, 5, 70, seed=1)
    S, B = oracle.kv4_scores(Q, qs, Kq, ks, 0.0884, want_bound=True)
    for h in range(3):
        Y, Bg = oracle.w4a8_gemm(Q[h], qs[h], Kq[h], ks[h][:, None], 0.0884, want_bound=True)
        assert np.allclose(S[h], Y, rtol=1e-14, atol=0) and np.allclose(B[h], Bg, rtol=1e-14, atol=0)


def test_dense_matmul_on_library_decoded_operands():
    Q, qs, Kq, ks, P, ps, Vq, vs = _rand(2, 6, 50, seed=2)
    S, SB = oracle.kv4_scores(Q, qs, Kq, ks, 0.5, want_bound=True)
    want = 0.5 * qs[:, :, None] * _e4m3(ks)[:, None, :] * np.einsum("hrc,htc->hrt", _e4m3(Q), Kq.astype(np.float64))
    assert np.all(np.abs(S - want) <= 1e-13 * SB)
    O, OB = oracle.kv4_output(P, ps, Vq, vs, want_bound=True)
    want = ps[:, :, None] * np.einsum("hrt,ht,htc->hrc", _e4m3(P), _e4m3(vs), Vq.astype(np.float64))
    assert np.all(np.abs(O - want) <= 1e-13 * OB)
    assert np.all(OB >= np.abs(O)) and np.all(SB >= np.abs(S))


def test_exact_rationals_on_a_tiny_case():
    Q, qs, Kq, ks, P, ps, Vq, vs = _rand(1, 2, 5, seed=3)
    S = oracle.kv4_scores(Q, qs, Kq, ks, 0.125); O = oracle.kv4_output(P, ps, Vq, vs)
    F = lambda x: Fraction(float(x))                           # noqa: E731  every operand is a dyadic rational
    for r in range(2):
        for t in range(5):
            exact = F(0.125) * F(qs[0, r]) * F(_e4m3(ks)[0, t]) * sum(F(_e4m3(Q)[0, r, c]) * int(Kq[0, t, c]) for c in range(128))
            assert abs(Fraction(float(S[0, r, t])) - exact) <= abs(exact) * Fraction(1, 10 ** 14)
        for c in range(0, 128, 17):
            exact = F(ps[0, r]) * sum(F(_e4m3(P)[0, r, t]) * F(_e4m3(vs)[0, t]) * int(Vq[0, t, c]) for t in range(5))
            assert abs(Fraction(float(O[0, r, c])) - exact) <= abs(exact) * Fraction(1, 10 ** 14) + Fraction(1, 10 ** 30)


def test_one_hot_operands_read_back_the_cache():
    """A one-hot query reads back one key element per token with its scale; a one-hot probability row reads back one
    token's value row with its scale: every cache element and every scale is seen individually."""
    H, T = 2, 40
    *_, = ()
    rng = np.random.default_rng(4)
    Kq = rng.integers(-8, 8, (H, T, 128), dtype=np.int8); Vq = rng.integers(-8, 8, (H, T, 128), dtype=np.int8)
    ks = rng.integers(1, 0x50, (H, T)).astype(np.uint8); vs = rng.integers(1, 0x50, (H, T)).astype(np.uint8)
    Q = np.zeros((H, 128, 128), np.uint8); Q[:, np.arange(128), np.arange(128)] = ONE
    S = oracle.kv4_scores(Q, np.ones((H, 128), np.float32), Kq, ks, 1.0)
    assert np.array_equal(S, (_e4m3(ks)[:, :, None] * Kq).transpose(0, 2, 1))
    P = np.zeros((H, T, T), np.uint8); P[:, np.arange(T), np.arange(T)] = ONE
    O = oracle.kv4_output(P, np.ones((H, T), np.float32), Vq, vs)
    assert np.array_equal(O, _e4m3(vs)[:, :, None] * Vq)


def test_invariants():
    Q, qs, Kq, ks, P, ps, Vq, vs = _rand(2, 4, 33, seed=5)
    S = oracle.kv4_scores(Q, qs, Kq, ks, 0.25)
    assert np.array_equal(oracle.kv4_scores(Q, qs, Kq, ks, 0.5), 2 * S)                 # a power of two is exact
    perm = np.random.default_rng(6).permutation(33)
    assert np.array_equal(oracle.kv4_scores(Q, qs, Kq[:, perm], ks[:, perm], 0.25), S[:, :, perm])   # tokens are independent
    O = oracle.kv4_output(P, ps, Vq, vs)
    O2 = oracle.kv4_output(P[:, :, perm], ps, Vq[:, perm], vs[:, perm])                 # the sum over tokens in another order
    assert np.allclose(O2, O, rtol=1e-12, atol=1e-300)
    assert np.array_equal(oracle.kv4_scores(Q[1:], qs[1:], Kq[1:], ks[1:], 0.25), S[1:])           # heads are independent
    # a token with scale zero contributes nothing to O and has score zero
    vs0 = vs.copy(); vs0[:, 7] = 0; ks0 = ks.copy(); ks0[:, 7] = 0
    Vz = Vq.copy(); Vz[:, 7] = 0
    assert np.array_equal(oracle.kv4_output(P, ps, Vq, vs0), oracle.kv4_output(P, ps, Vz, vs))
    assert not oracle.kv4_scores(Q, qs, Kq, ks0, 0.25)[:, :, 7].any()
