"""Per-tensor scaling search of the CPU oracle (Sec. 3.1.2, Def. 3.2; App. C.1), in exact arithmetic.

TEST INFRASTRUCTURE ONLY, like the rest of this package.

Def. 3.2: n is the smallest non-negative integer for which one of these holds:

  1.  S(W * 2^n) = S(W * 2^(n+i)) for every natural i, where
      S(W) = sum over the elements w of max(0, 7 * 2^-9 - |w|)      (cumulative underflow);
  2.  some element satisfies  7 * 2^(5-n) <= |w| < 7 * 2^(6-n)       (one more doubling would overflow).

Every FP32 number is an integer multiple of 2^-149, so with UNIT = 2^-160 every quantity below is
a Python integer and the sums are exact: no rounding can make two different scores look equal.

"For every natural i": S(W * 2^m) never grows with m, and for m >= FAR every non-zero FP32 element
times 2^m lies above the threshold 7 * 2^-9, so S has reached its final value there.  Hence
S(n) = S(n + i) for all i  <=>  S(n) = S(n + FAR); that is the comparison made.

Reading: the search stops at n = 126 (2^n must stay an FP32 number for the quantiser); a matrix that
meets neither condition up to there (all elements non-zero and below 2^-128 or so) gets 126.
"""
from __future__ import annotations

import numpy as np

_UNIT_LOG2 = 160                          # everything in units of 2^-160
_THRESHOLD = 7 << (_UNIT_LOG2 - 9)        # 7 * 2^-9
FAR = 320                                 # 2^-149 * 2^320 is far above the threshold
N_MAX = 126


def _magnitudes(values: np.ndarray) -> list:
    """|v| of FP32 values as exact Python integers in units of 2^-160."""
    v = np.abs(np.ascontiguousarray(values, dtype=np.float32).ravel()).astype(np.float64)
    if not np.all(np.isfinite(v)):
        raise ValueError("weights must be finite")
    mant, expo = np.frexp(v)              # v = mant * 2^expo, mant in [0.5, 1): exact
    mant_i = (mant * 2.0 ** 53).astype(np.int64)
    out = []
    for m, e in zip(mant_i.tolist(), expo.tolist()):
        sh = e - 53 + _UNIT_LOG2          # >= -149 - 53 + 160 - ... : can be negative only by bits that are zero
        out.append(m << sh if sh >= 0 else m >> (-sh))
    return out


def underflow_score(mags: list, n: int) -> int:
    """S(W * 2^n) in units of 2^-160 (eq. 7 of Def. 3.2)."""
    total = 0
    for a in mags:
        d = _THRESHOLD - (a << n)
        if d > 0:
            total += d
    return total


def overflow_risk(mags: list, n: int) -> bool:
    """Condition 2 of Def. 3.2 (eq. 8): an element with 7 * 2^(5-n) <= |w| < 7 * 2^(6-n)."""
    lo = 7 << (_UNIT_LOG2 + 5)            # compare |w| * 2^n with 7 * 2^5 and 7 * 2^6
    hi = 7 << (_UNIT_LOG2 + 6)
    return any(lo <= (a << n) < hi for a in mags)


def pts_exponent(values: np.ndarray) -> int:
    """n of Def. 3.2 for a matrix of FP32 values (the weights after channel scaling)."""
    mags = _magnitudes(values)
    small = [a for a in mags if a < _THRESHOLD]      # only these can ever contribute to S
    for n in range(N_MAX + 1):
        if underflow_score(small, n) == underflow_score(small, n + FAR):
            return n
        if overflow_risk(mags, n):
            return n
    return N_MAX
