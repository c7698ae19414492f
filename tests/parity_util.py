"""Shared helpers of the GPU parity tests: the comparison rule and tensor marshalling."""
import numpy as np

import oracle

REL_FROBENIUS_TOL = 2e-3       # against the unrounded FP64 result (bf16 rounding alone costs ~1.7e-3)
BOUND_TOL = 1e-3               # per element: 1 bf16 ulp + 1e-3 * sum of |terms|
FLIP_FRACTION_TOL = 0.15       # share of outputs allowed to land one bf16 step from the once-rounded reference


def to_gpu_bf16(bits: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bf16_bits_from_gpu(t) -> np.ndarray:
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def check_gemm(Y_bits: np.ndarray, Y_ref: np.ndarray, bound: np.ndarray, what: str = "", frobenius: bool = True):
    """Y_bits: uint16 bf16 patterns from the GPU; Y_ref, bound: FP64 from the oracle.
    frobenius=False leaves out the norm-wise criterion (for inputs built so that a handful of outputs carry the
    whole norm: their bf16 rounding alone, up to 2^-9 each, can then exceed the 2e-3 meant for a matrix of like-sized
    outputs); the element-wise criterion, which is the sharper one, always applies."""
    Yg = oracle.bf16_bits_to_f64(Y_bits)
    assert np.all(np.isfinite(Yg)), what + ": non-finite output"
    err = np.abs(Yg - Y_ref)
    tol = oracle.bf16_ulp_array(Y_ref) + BOUND_TOL * bound
    worst = int(np.argmax(err - tol))
    assert np.all(err <= tol), "%s: element %s off by %g (tol %g, ref %g)" % (
        what, np.unravel_index(worst, err.shape), err.flat[worst], tol.flat[worst], Y_ref.flat[worst])
    denom = np.linalg.norm(Y_ref)
    if denom > 0 and frobenius:
        rel = np.linalg.norm(Yg - Y_ref) / denom
        assert rel <= REL_FROBENIUS_TOL, "%s: relative Frobenius error %g" % (what, rel)
    # Against the once-rounded reference: an output differs only where the FP32 result and the exact one
    # lie on opposite sides of a rounding boundary, which FP32 accumulation noise makes happen for a few
    # per cent of the outputs (more where terms cancel); an epilogue that truncated, or rounded twice,
    # would move a quarter to a half of them.  Every difference is a single bf16 step.
    Yb = oracle.bf16_bits_to_f64(oracle.bf16_round_array(Y_ref))
    differs = Yg != Yb
    flips = np.mean(differs)
    assert flips <= FLIP_FRACTION_TOL, "%s: %.1f %% of the outputs differ from the once-rounded reference" % (
        what, 100 * flips)
    return {"flips_vs_rounded_ref": float(flips), "max_err_over_tol": float(np.max(err / tol))}
