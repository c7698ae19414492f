"""Pins for the oracle's table-form GEMM (Sec. 3.1.1 steps 1-2: a 16-entry FP8 table of q * sigma per
group) and the measurement it exists for: what rounding the table entries to E4M3 costs against the
exact scale the library applies.  No GPU here."""
import numpy as np

import oracle
from paper_2505_20839_amd import workloads

ONE = 0x38


def _one_product(qv, gs_code, a_code=ONE):
    A = np.zeros((1, 128), np.uint8); A[0, 9] = a_code
    q = np.zeros((1, 128), np.int8); q[0, 9] = qv
    return A, np.ones(1, np.float32), q, np.array([[gs_code]], np.uint8)


def test_table_entries_hand_values():
    # sigma = 1.125 (code 0x39): 7 * 1.125 = 7.875 lies between the E4M3 neighbours 7.5 and 8 -> 8
    assert oracle.e4m3_decode(0x39) == 1.125
    assert oracle.w4a8_gemm_lut(*_one_product(7, 0x39), 1.0)[0, 0] == 8.0
    assert oracle.w4a8_gemm(*_one_product(7, 0x39), 1.0)[0, 0] == 7.875
    # -8 * 1.125 = -9 is an E4M3 value (step 1 on [8, 16)): no rounding; 3 * 1.125 = 3.375 -> 3.5 (ties to even: 3.25|3.5)
    assert oracle.w4a8_gemm_lut(*_one_product(-8, 0x39), 1.0)[0, 0] == -9.0
    assert oracle.w4a8_gemm_lut(*_one_product(3, 0x39), 1.0)[0, 0] == 3.5
    # saturation: 7 * 448 is far above the largest FP8 value (App. C.1: 448)
    assert oracle.w4a8_gemm_lut(*_one_product(7, 0x7E), 1.0)[0, 0] == 448.0
    # sigma = 0 (Lemma B.1): the whole table is zero
    assert oracle.w4a8_gemm_lut(*_one_product(7, 0x00), 1.0)[0, 0] == 0.0


def test_equals_the_exact_gemm_when_every_entry_is_representable():
    """Power-of-two scales: q * sigma keeps q's four significant bits, so the table rounds nothing."""
    rng = np.random.default_rng(21)
    M, N, K = 4, 6, 256
    A = rng.integers(0, 0x78, (M, K)).astype(np.uint8) | (rng.integers(0, 2, (M, K)).astype(np.uint8) << 7)
    q = rng.integers(-8, 8, (N, K), dtype=np.int8)
    gs = (rng.integers(2, 12, (N, K // 128)).astype(np.uint8) << 3)          # mantissa 0: powers of two
    a = rng.uniform(0.5, 2, M).astype(np.float32)
    exact = oracle.w4a8_gemm(A, a, q, gs, 0.5)
    assert np.allclose(oracle.w4a8_gemm_lut(A, a, q, gs, 0.5), exact, rtol=1e-13, atol=0)


def test_what_the_table_rounding_costs():
    """On workload-like operands the table form differs from the exact-scale result by about 2 % in
    relative Frobenius norm -- ten times the library's whole error budget (2e-3), which is why the exact
    scale is the target here -- and the weights themselves move by 2-3 % RMS."""
    d = workloads.draw(24, 96, 1024, seed=33, outlier_frac=0.01)
    A, s = oracle.quantize_act(d["X_bf16"])
    exact = oracle.w4a8_gemm(A, s, d["q"], d["gscale"], d["w_tscale"])
    table = oracle.w4a8_gemm_lut(A, s, d["q"], d["gscale"], d["w_tscale"])
    rel = np.linalg.norm(table - exact) / np.linalg.norm(exact)
    assert 0.01 < rel < 0.04, rel
    sig = np.array([oracle.e4m3_decode(int(c)) for c in d["gscale"].ravel()]).reshape(d["gscale"].shape).repeat(128, axis=1)
    w_exact = d["q"] * sig
    w_table = np.array([oracle.e4m3_decode(oracle.e4m3_encode_rne(float(x))) for x in w_exact.ravel()[:20000]])
    rms = np.sqrt(np.mean((w_table - w_exact.ravel()[:20000]) ** 2) / np.mean(w_exact.ravel()[:20000] ** 2))
    assert 0.015 < rms < 0.035, rms


def test_bound_is_the_sum_of_absolute_terms():
    """The bound returned beside the table-form result is the same sum with every term's absolute value: equal
    to |Y| when all terms have one sign, and never below |Y|."""
    rng = np.random.default_rng(5)
    M, N, K = 3, 5, 256
    A = rng.integers(0x20, 0x60, (M, K)).astype(np.uint8)                      # positive activations
    q = rng.integers(0, 8, (N, K), dtype=np.int8)                              # non-negative weights
    gs = rng.integers(0x10, 0x40, (N, K // 128)).astype(np.uint8)
    a = rng.uniform(0.5, 2, M).astype(np.float32)
    Y, B = oracle.w4a8_gemm_lut(A, a, q, gs, 0.5, want_bound=True)
    assert np.allclose(Y, B, rtol=1e-14) and np.all(Y > 0)
    q2 = rng.integers(-8, 8, (N, K), dtype=np.int8)
    Y2, B2 = oracle.w4a8_gemm_lut(A, a, q2, gs, -0.5, want_bound=True)
    assert np.all(B2 >= np.abs(Y2)) and np.all(B2 > 0)
    assert np.array_equal(Y2, oracle.w4a8_gemm_lut(A, a, q2, gs, -0.5))
