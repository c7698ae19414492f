"""Pins for the oracle's activation quantiser (Sec. 2.1 eq. 2: A = FP8(x / beta), one beta per
token) against closed-form rows and an independent path made of library operations
(numpy's IEEE float32 division followed by torch's float8 cast)."""
import numpy as np
import torch

import oracle
from paper_2505_20839_amd import workloads


def _bits(x):
    return workloads.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_closed_form_rows():
    X = _bits([[448.0, -448.0, 224.0, 1.0, 0.0, -0.5, 3.0, 2.0 ** -9],      # absmax 448 -> scale 1
               [1.0, -1.0, 0.5, 0.25, 0.0, 0.0, 0.0, 0.0],                   # absmax 1 -> scale 1/448
               [0.0] * 8,                                                    # all zero -> scale 1
               [-3.0, 1.5, 0.75, 0.0, 0.0, 0.0, 0.0, 0.0]])                  # absmax 3
    A, s = oracle.quantize_act(X)
    assert s.dtype == np.float32
    assert s[0] == 1.0 and s[1] == np.float32(1.0) / np.float32(448.0) and s[2] == 1.0
    assert s[3] == np.float32(3.0) / np.float32(448.0)
    assert A[0].tolist() == [0x7E, 0xFE, 0x76, 0x38, 0x00, 0xB0, 0x44, 0x01]
    assert A[1].tolist()[:5] == [0x7E, 0xFE, 0x76, 0x6E, 0x00]               # 448, -448, 224, 112
    assert A[2].tolist() == [0] * 8
    assert A[3].tolist()[:3] == [0xFE, 0x76, 0x6E]


def test_against_library_division_and_cast():
    rng = np.random.default_rng(21)
    M, K = 40, 768
    X = rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.uniform(-6, 6, (M, 1))).astype(np.float32)
    X[:, rng.choice(K, 8, replace=False)] *= 20
    Xb = _bits(X)
    A, s = oracle.quantize_act(Xb)
    xf = oracle.bf16_bits_to_f64(Xb).astype(np.float32)                      # exact
    amax = np.abs(xf).max(axis=1)
    s_lib = (amax / np.float32(448.0)).astype(np.float32)                    # IEEE float32 division
    assert np.array_equal(s, s_lib)
    quot = (xf / s_lib[:, None]).astype(np.float32)
    assert np.all(np.abs(quot) <= 448.0 * (1 + 2.0 ** -22))
    quot = np.clip(quot, -448.0, 448.0)
    lib = torch.from_numpy(quot).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(A & 0x7F, lib & 0x7F)
    nz = (A & 0x7F) != 0
    assert np.array_equal(A[nz], lib[nz])                                     # signs agree off zero
    assert np.all((A & 0x7F).max(axis=1) == 0x7E)                            # the absmax maps to +-448


def test_all_finite_bf16_inputs():
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = oracle.bf16_bits_to_f64(allbits)
    for amax in (1.0, 448.0, 0.0131, 3.0e4, 2.0 ** -100):
        am = oracle.bf16_bits_to_f64(_bits([amax]))[0]
        keep = allbits[np.isfinite(vals) & (np.abs(vals) <= am)]
        row = np.concatenate([_bits([amax]), keep])
        pad = (-len(row)) % 8
        row = np.concatenate([row, np.zeros(pad, np.uint16)])[None, :]
        A, s = oracle.quantize_act(row)
        xf = oracle.bf16_bits_to_f64(row).astype(np.float32)
        s_lib = np.float32(am) / np.float32(448.0)
        assert s[0] == s_lib
        quot = np.clip((xf / s_lib).astype(np.float32), -448.0, 448.0)
        lib = torch.from_numpy(quot).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(A & 0x7F, lib & 0x7F)


def test_scaled_back_values_are_close():
    # eq. 2: y ~ beta * FP8(y / beta): relative error at most half an E4M3 step (2^-4) for
    # normal results, absolute error at most half the smallest subnormal times beta otherwise.
    d = workloads.draw(64, 8, 1024, seed=33, act="laplace", outlier_frac=0.01)
    A, s = oracle.quantize_act(d["X_bf16"])
    x = oracle.bf16_bits_to_f64(d["X_bf16"])
    deq = np.array([[oracle.e4m3_decode(int(c)) for c in row] for row in A[:4]]) * s[:4, None].astype(np.float64)
    err = np.abs(deq - x[:4])
    assert np.all(err <= np.maximum(np.abs(x[:4]) * 2.0 ** -4, s[:4, None] * 2.0 ** -10) * 1.000001)
