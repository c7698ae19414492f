"""Pins for the oracle's offline weight quantiser: group-wise INT4 with an FP8 scale (Sec. 2.1 eq. 1,
Sec. 3.1), the underflow lemma (App. B, Lemma B.1), channel-wise absmean scaling (Def. 3.1) and the
per-tensor scaling search (Def. 3.2, App. C.1).  Hand values, the paper's thresholds, closed forms,
invariants and brute force on tiny inputs.  No GPU here."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import pts


def bits(x):
    """bf16 bit patterns of values that bf16 holds exactly."""
    b = np.asarray(x, np.float32).view(np.uint32)
    assert np.all((b & 0xFFFF) == 0), "not a bf16 value"
    return (b >> 16).astype(np.uint16)


def trunc_bits(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> 16).astype(np.uint16)


# ---- the toward-zero E4M3 cast -------------------------------------------------------------------

def test_rtz_cast_is_the_largest_code_not_above():
    vals = [oracle.e4m3_decode(c) for c in range(0x7F)]
    assert vals == sorted(vals) and vals[1] == 2.0 ** -9 and vals[0x7E] == 448.0
    for c in range(0x7F):
        assert oracle.e4m3_encode_rtz(vals[c]) == c                       # exact values stay
        assert oracle.e4m3_encode_rtz(-vals[c]) == (c | 0x80)
        if c < 0x7E:
            mid = (vals[c] + vals[c + 1]) / 2
            assert oracle.e4m3_encode_rtz(mid) == c                       # never up
            assert oracle.e4m3_encode_rtz(np.nextafter(vals[c + 1], 0)) == c
    assert oracle.e4m3_encode_rtz(1e9) == 0x7E
    # Lemma B.1: anything below the smallest subnormal 2^-9 becomes zero; nearest-even does not do that
    assert oracle.e4m3_encode_rtz(0.999 * 2.0 ** -9) == 0
    assert oracle.e4m3_encode_rne(0.999 * 2.0 ** -9) == 1


# ---- eq. 1 on one group -----------------------------------------------------------------------------

def _group(values):
    v = np.zeros(128, np.float32)
    v[:len(values)] = values
    return bits(v.reshape(1, 128))


def test_eq1_hand_values():
    # max |v| = 1.75 -> sigma = 0.25 (E4M3 code 0x28), codes = v / 0.25, dequantised values = v
    v = 0.25 * np.array([7, -7, 3, -1, 0, 5, -6, 2], np.float32)
    q, gs = oracle.quantize_weights(_group(v))
    assert gs.tolist() == [[0x28]] and oracle.e4m3_decode(0x28) == 0.25
    assert q[0, :8].tolist() == [7, -7, 3, -1, 0, 5, -6, 2] and not q[0, 8:].any()
    # the per-tensor factor multiplies the weights before quantisation (Def. 3.2): 2^3 -> sigma = 2
    q, gs = oracle.quantize_weights(_group(v), n_pts=3)
    assert oracle.e4m3_decode(int(gs[0, 0])) == 2.0 and q[0, :8].tolist() == [7, -7, 3, -1, 0, 5, -6, 2]


def test_quotient_rounds_to_nearest_ties_to_even():
    v = np.array([7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.4375, 3.5625, -6.5], np.float32)    # sigma = 1
    q, gs = oracle.quantize_weights(_group(v))
    assert oracle.e4m3_decode(int(gs[0, 0])) == 1.0
    assert q[0, :10].tolist() == [7, 0, 2, 2, 0, -2, -2, 3, 4, -6]


def test_lowered_scale_clamps_to_the_int4_range():
    # max = 7.75: sigma = 1.107 -> toward zero 1.0: 7.75 -> 8 -> clamped to 7; -7.75 -> -8 is a code
    q, gs = oracle.quantize_weights(_group([7.75, -7.75, 7.25]))
    assert oracle.e4m3_decode(int(gs[0, 0])) == 1.0 and q[0, :3].tolist() == [7, -8, 7]
    # nearest-even picks 1.125 instead: 7.75 / 1.125 = 6.89 -> 7
    q, gs = oracle.quantize_weights(_group([7.75, -7.75, 7.25]), sigma_rne=True)
    assert oracle.e4m3_decode(int(gs[0, 0])) == 1.125 and q[0, :3].tolist() == [7, -7, 6]


def test_lemma_b1_underflow_threshold():
    t = 7 * 2.0 ** -9
    below = 1.7421875 * 2.0 ** -7                                         # the bf16 value just under 7 * 2^-9 = 1.75 * 2^-7
    q, gs = oracle.quantize_weights(_group([below, -below / 2, below / 4]))
    assert gs.tolist() == [[0]] and not q.any()                           # sigma_FP8 = 0, the group is all zero
    q, gs = oracle.quantize_weights(_group([t, -t / 2]))                  # at the threshold: sigma = 2^-9
    assert gs.tolist() == [[1]] and q[0, :2].tolist() == [7, -4]          # -3.5 ties to even
    # the nearest-even cast keeps such a group alive (sigma = 0.99 * 2^-9 rounds up to 2^-9)
    q, gs = oracle.quantize_weights(_group([below, -below / 2]), sigma_rne=True)
    assert gs.tolist() == [[1]] and q[0, 0] == 7
    # saturation of sigma at 448 (App. C.1) for absurdly large weights
    q, gs = oracle.quantize_weights(_group([2.0 ** 14]))
    assert gs.tolist() == [[0x7E]] and q[0, 0] == 7


@pytest.mark.parametrize("rne", [False, True])
def test_codes_are_the_nearest_multiples(rne):
    """Brute force: away from ties and clamping, q is the integer c in -8..7 minimising |v - c * sigma8|;
    the rounding error is at most sigma8 / 2 (eq. 1: x ~ sigma * x_hat)."""
    rng = np.random.default_rng(5)
    W = trunc_bits((rng.standard_normal((6, 512)) * rng.uniform(0.01, 3, (6, 1))).astype(np.float32))
    q, gs = oracle.quantize_weights(W, sigma_rne=rne)
    v = oracle.scaled_weights(W).astype(np.float64)
    s8 = np.array([oracle.e4m3_decode(int(c)) for c in gs.ravel()]).reshape(gs.shape).repeat(128, axis=1)
    assert np.all(s8 > 0)
    cand = np.arange(-8, 8)[None, None, :] * s8[:, :, None]
    dist = np.abs(v[:, :, None] - cand)
    best = np.argmin(dist, axis=2) - 8
    srt = np.sort(dist, axis=2)
    clear = (srt[:, :, 1] - srt[:, :, 0]) > 1e-6 * s8                     # not a tie within FP32 rounding
    assert clear.mean() > 0.95 and np.array_equal(q[clear], best[clear])     # bf16 over a 4-bit scale ties often
    inside = np.abs(v) <= 7.5 * s8
    assert np.all(np.abs(v - q * s8)[inside] <= 0.5 * s8[inside] * (1 + 1e-6))
    # sigma8 is the cast of max / 7: never above it toward zero, within half a step to nearest
    gmax = np.abs(v).reshape(6, 4, 128).max(axis=2)
    s8g = s8[:, ::128]
    if rne:
        assert np.all(np.abs(s8g - gmax / 7) <= s8g / 16 + 2.0 ** -10)
    else:
        assert np.all(s8g <= gmax / 7 * (1 + 1e-7)) and np.all(s8g >= gmax / 7 * (1 - 1 / 8) - 2.0 ** -9)


def test_groups_and_channels_are_independent_and_in_place():
    """Each (channel, group of 128) only sees its own elements: quantising a slice gives the slice."""
    rng = np.random.default_rng(6)
    W = trunc_bits(rng.standard_normal((5, 384)).astype(np.float32))
    q, gs = oracle.quantize_weights(W, n_pts=2)
    for n, g in [(0, 0), (4, 2), (2, 1)]:
        q1, g1 = oracle.quantize_weights(W[n:n + 1, 128 * g:128 * g + 128], n_pts=2)
        assert np.array_equal(q1[0], q[n, 128 * g:128 * g + 128]) and g1[0, 0] == gs[n, g]
    with pytest.raises(ValueError):
        oracle.quantize_weights(W[:, :100])


# ---- channel-wise absmean scaling (Def. 3.1) ------------------------------------------------------

def test_cas_hand_values_and_closed_form():
    W = bits(np.array([[1.0, 0.0, -2.0], [-3.0, 0.0, 0.5]], np.float32))    # columns: absmean 2, 0, 1.25
    lam = oracle.cas_scales(W, 0.5)
    assert lam.tolist() == [0.25, 1.0, 0.4]
    rng = np.random.default_rng(7)
    Wf = trunc_bits((rng.standard_normal((40, 16)) * rng.uniform(0.01, 10, (1, 16))).astype(np.float32))
    lam = oracle.cas_scales(Wf, 0.03)
    Wd = oracle.bf16_bits_to_f64(Wf)
    # after scaling every input channel has the target absmean: it is the columns (k) that are scaled
    assert np.allclose(np.abs(Wd * lam[None, :]).mean(axis=0), 0.03, rtol=1e-12)
    assert lam.shape == (16,)


def test_cas_keeps_the_product():
    """Sec. 3.1.2: (X Lambda^-1) (W Lambda)^T = X W^T."""
    rng = np.random.default_rng(8)
    Wf = trunc_bits(rng.standard_normal((12, 8)).astype(np.float32))
    lam = oracle.cas_scales(Wf, 1.0)
    Wd = oracle.bf16_bits_to_f64(Wf)
    X = rng.standard_normal((5, 8))
    assert np.allclose((X / lam) @ (Wd * lam).T, X @ Wd.T, rtol=1e-12, atol=1e-12)


def test_scaled_weights_round_once_to_fp32():
    W = bits(np.array([[1.5, -0.375]], np.float32))
    lam = np.array([1 / 3, 3.0000002], np.float32)
    got = oracle.scaled_weights(W, lam)
    want = np.array([[np.float32(np.float64(1.5) * np.float64(lam[0])), np.float32(np.float64(-0.375) * np.float64(lam[1]))]])
    assert np.array_equal(got, want) and got.dtype == np.float32
    assert np.array_equal(oracle.scaled_weights(W), np.array([[1.5, -0.375]], np.float32))


# ---- per-tensor scaling (Def. 3.2) ----------------------------------------------------------------

T = 7 * 2.0 ** -9


def _n(values):
    return pts.pts_exponent(np.asarray(values, np.float32))


def test_pts_hand_cases():
    assert _n([1.0, -0.5, T]) == 0                      # nothing under the threshold: S is already final
    assert _n([0.0, 0.0]) == 0 and _n([0.0, 1.0]) == 0  # zeros stay under it for every n: they never matter
    assert _n([1.0, T / 8]) == 3                        # condition 1: the small element reaches T at 2^3
    assert _n([1.0, T / 8 * 0.99]) == 4
    assert _n([0.5, 2.0 ** -40]) == 9                   # condition 2 first: 0.5 * 2^9 = 256 lies in [224, 448)
    assert _n([224.0, 2.0 ** -40]) == 0                 # lower edge of the band belongs to it
    assert _n([223.0, 2.0 ** -40]) == 1
    assert _n([448.0, T / 4]) == 2                      # upper edge does not: only condition 1 can stop it
    assert _n([447.0, T / 4]) == 0
    assert _n([1e-30, 1.0]) == 8                        # a float sum would not see 1e-30 and answer 0
    assert _n([2.0 ** -130]) == 124 and _n([2.0 ** -149]) == pts.N_MAX


def test_pts_thresholds_are_the_papers():
    # eq. 7: S sums 7 * 2^-9 - |w| over the elements under 7 * 2^-9
    mags = pts._magnitudes(np.array([0.0, T / 2, T, 1.0], np.float32))
    unit = Fraction(1, 2 ** 160)
    assert pts.underflow_score(mags, 0) * unit == Fraction(T) + Fraction(T) / 2
    assert pts.underflow_score(mags, 1) * unit == Fraction(T)
    assert pts.underflow_score(mags, 5) == pts.underflow_score(mags, 1)
    # eq. 8 / App. C.1: the band is 1.75 * 2^7 <= delta * |w| < 1.75 * 2^8
    for w, n, hit in [(1.75 * 2 ** 7, 0, True), (1.75 * 2 ** 8, 0, False), (1.75, 7, True), (1.75, 6, False), (1.75, 8, False)]:
        assert pts.overflow_risk(pts._magnitudes(np.array([w], np.float32)), n) is hit


def _pts_by_fractions(values, i_max=330):
    """Def. 3.2 once more, literally, with rationals: condition 1 checked for every i up to i_max."""
    w = [Fraction(float(x)) for x in np.asarray(values, np.float32).ravel()]
    t = Fraction(7, 2 ** 9)

    def S(n):
        return sum((max(Fraction(0), t - abs(x) * 2 ** n) for x in w), Fraction(0))

    for n in range(127):
        sn = S(n)
        if all(S(n + i) == sn for i in range(1, i_max)):
            return n
        if any(Fraction(7 * 2 ** 5, 2 ** n) <= abs(x) < Fraction(7 * 2 ** 6, 2 ** n) for x in w):
            return n
    return 126


def test_pts_matches_a_literal_evaluation_with_rationals():
    rng = np.random.default_rng(9)
    for trial in range(12):
        size = int(rng.integers(1, 7))
        expo = rng.integers(-30, 6, size)
        vals = (rng.uniform(1, 2, size) * 2.0 ** expo * rng.choice([-1, 1], size)).astype(np.float32)
        if trial % 3 == 0:
            vals[0] = 0.0
        assert _n(vals) == _pts_by_fractions(vals, i_max=60), vals       # exponents >= -30: 60 doublings suffice
    assert _n([2.0 ** -100]) == _pts_by_fractions([2.0 ** -100], i_max=330) == 94


def test_pts_then_quantise_underflow_statistics():
    """Lemma B.1 on a whole matrix: a group's FP8 scale is zero exactly when its maximum is under 7 * 2^-9
    after the per-tensor factor, and the factor chosen by condition 1 leaves no such group."""
    rng = np.random.default_rng(10)
    W = trunc_bits((rng.standard_normal((16, 512)) * 0.002).astype(np.float32))
    v = np.abs(oracle.scaled_weights(W).astype(np.float64)).reshape(16, 4, 128).max(axis=2)
    _, gs0 = oracle.quantize_weights(W, n_pts=0)
    assert np.array_equal(gs0 == 0, v < T) and (gs0 == 0).mean() > 0.9   # nearly everything underflows unscaled
    n = oracle.pts_exponent(W)
    assert 0 < n < 20
    _, gs = oracle.quantize_weights(W, n_pts=n)
    assert np.array_equal(gs == 0, v * 2.0 ** n < T)
    assert (gs == 0).sum() == 0
    assert np.abs(oracle.scaled_weights(W)).max() * 2.0 ** n < 448        # and nothing overflows
