"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integer/byte work (packing, E4M3 codes, row scales) must be bit-exact; the bf16
GEMM output must satisfy  |Y - Y_ref| <= 1 bf16 ulp + 1e-3 * sum|terms|  per element and a relative
Frobenius error of at most 2e-3 against the unrounded FP64 result."""
import ctypes
import os

import numpy as np
import pytest

import oracle
from paper_2505_20839_amd import workloads
from parity_util import bf16_bits_from_gpu, check_gemm, to_gpu_bf16

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def fq():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    from paper_2505_20839_amd import binding
    binding.lib()
    return binding


@pytest.fixture
def kernel_choice(fq):
    yield fq.fq_test_force_kernel
    fq.fq_test_force_kernel(None)


def _gpu(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _run_gemm(fq, A, a_scale, q, gscale, t):
    N = q.shape[0]
    packed = fq.fq_pack_weights(_gpu(q))
    Y = fq.fq_w4a8_gemm(_gpu(A), _gpu(a_scale), packed, _gpu(gscale), t, N)
    torch.cuda.synchronize()
    return bf16_bits_from_gpu(Y)


def _rand_codes(M, N, K, seed, signed_scales=True):
    rng = np.random.default_rng(seed)
    A = rng.integers(0, 0x7F, (M, K)).astype(np.uint8) | (rng.integers(0, 2, (M, K)).astype(np.uint8) << 7)
    q = rng.integers(-8, 8, (N, K), dtype=np.int8)
    gs = rng.integers(0, 0x48, (N, K // 128)).astype(np.uint8)
    if signed_scales:
        gs |= (rng.integers(0, 2, gs.shape).astype(np.uint8) << 7)
    a = rng.uniform(0.01, 2.0, M).astype(np.float32)
    return A, a, q, gs, float(np.float32(rng.uniform(0.1, 3.0)))


# ---- packing: bit-exact round trip ---------------------------------------------------------------

@pytest.mark.parametrize("N,K", [(32, 128), (256, 512), (100, 384), (1, 128), (4096, 1408), (77, 2048)])
def test_pack_unpack_roundtrip(fq, N, K):
    rng = np.random.default_rng(N * 7 + K)
    q = rng.integers(-8, 8, (N, K), dtype=np.int8)
    packed = fq.fq_pack_weights(_gpu(q))
    assert packed.numel() == fq.fq_packed_weight_bytes(N, K)
    back = fq.fq_unpack_weights(packed, N, K).cpu().numpy()
    assert np.array_equal(back, q)


def test_pack_every_code_at_every_position(fq):
    N, K = 64, 256
    base = (np.arange(N)[:, None] * 5 + np.arange(K)[None, :] * 3)
    for shift in range(16):
        q = (((base + shift) % 16) - 8).astype(np.int8)
        packed = fq.fq_pack_weights(_gpu(q))
        assert np.array_equal(fq.fq_unpack_weights(packed, N, K).cpu().numpy(), q)
    # only the low four bits of a code are read
    q = np.random.default_rng(0).integers(-8, 8, (N, K), dtype=np.int8)
    dirty = ((q.astype(np.int16) & 0xF) | 0x50).astype(np.uint8).view(np.int8)
    assert np.array_equal(fq.fq_unpack_weights(fq.fq_pack_weights(_gpu(dirty)), N, K).cpu().numpy(), q)


# ---- activation quantiser: bit-exact --------------------------------------------------------------

def _check_quantize(fq, Xbits):
    A_ref, s_ref = oracle.quantize_act(Xbits)
    A, s = fq.fq_quantize_act(to_gpu_bf16(Xbits))
    torch.cuda.synchronize()
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    A = A.cpu().numpy()
    if not np.array_equal(A, A_ref):                       # -0 and +0 are the same number
        diff = A != A_ref
        assert np.all((A[diff] & 0x7F) == 0) and np.all((A_ref[diff] & 0x7F) == 0)
    return A, s_ref


@pytest.mark.parametrize("M,K,act,frac,seed", [(16, 512, "gauss", 0.0, 0), (300, 4096, "gauss", 0.01, 1),
                                               (64, 11008, "laplace", 0.01, 2), (5, 16512, "gauss", 0.0, 3),
                                               (1, 128, "gauss", 0.0, 4), (3, 8, "gauss", 0.0, 5)])
def test_quantize_matches_oracle(fq, M, K, act, frac, seed):
    if K % 128:
        rng = np.random.default_rng(seed)
        X = workloads.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    else:
        X = workloads.draw(M, 32, K, seed=seed, act=act, outlier_frac=frac)["X_bf16"]
    _check_quantize(fq, X)


def test_quantize_all_finite_bf16_values_and_zero_row(fq):
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = oracle.bf16_bits_to_f64(allbits)
    rows = []
    for amax in (1.0, 448.0, 0.0131, 3.0e4, 2.0 ** -100, 6.0e37):
        ab = workloads.f32_to_bf16_bits(np.array([amax], np.float32))
        am = oracle.bf16_bits_to_f64(ab)[0]
        keep = allbits[np.isfinite(vals) & (np.abs(vals) <= am)]
        row = np.concatenate([ab, keep])
        rows.append(row)
    K = max(len(r) for r in rows)
    K += (-K) % 8
    X = np.zeros((len(rows) + 1, K), np.uint16)           # last row stays all zero
    for i, r in enumerate(rows):
        X[i, :len(r)] = r
    A, s = _check_quantize(fq, X)
    assert s[-1] == 1.0 and not A[-1].any()


# ---- GEMM: element-by-element against the oracle, every kernel ------------------------------------

# small: besides the basics, the M <= 16 kernel's variants -- byte-wise scales (K/128 = 11), a slice
# longer than the ring (K = 14336), 2 and 3 sub-tiles of channels per workgroup, a masked last sub-tile
SMALL_SHAPES = [(16, 256, 512), (1, 32, 128), (33, 100, 384), (64, 96, 1408), (7, 31, 256),
                (8, 100, 1408), (16, 64, 14336), (16, 4120, 512), (3, 9000, 256), (12, 14336, 384),
                # ring depths 12 and 8 with and without a second round, scale rows that are not word-aligned
                (5, 200, 11008), (8, 8192, 5120), (4, 8192, 11008), (16, 300, 1664),
                # 16 < M <= 64 with rows of scales that are whole words (table fetched as words), also beyond the two words a
                # thread fetches up front (K = 16384), ragged channel counts
                (40, 300, 1024), (64, 136, 16384), (17, 8200, 512), (48, 72, 4096)]
# large: ragged M and N, one group only, a second half tile without rows, several zero-point rounds
LARGE_SHAPES = [(16, 256, 512), (300, 200, 640), (257, 513, 384), (512, 256, 1408), (65, 33, 128),
                (129, 136, 256), (130, 64, 16384), (700, 1100, 256)]


@pytest.mark.parametrize("kernel,shape", [("simple", s) for s in SMALL_SHAPES[:3]] +
                         [("small", s) for s in SMALL_SHAPES] + [("large", s) for s in LARGE_SHAPES])
def test_gemm_random_codes(fq, kernel_choice, kernel, shape):
    M, N, K = shape
    A, a, q, gs, t = _rand_codes(M, N, K, seed=M + N + K)
    kernel_choice(kernel)
    Yb = _run_gemm(fq, A, a, q, gs, t)
    Y, B = oracle.w4a8_gemm(A, a, q, gs, t, want_bound=True)
    check_gemm(Yb, Y, B, "%s %s" % (kernel, shape))


@pytest.mark.parametrize("kernel", ["simple", "small", "large"])
def test_gemm_config1(fq, kernel_choice, kernel):
    d = workloads.draw_workload("c1_tiny")
    A, s = _check_quantize(fq, d["X_bf16"])
    kernel_choice(kernel)
    Yb = _run_gemm(fq, A, s, d["q"], d["gscale"], d["w_tscale"])
    Y, B = oracle.w4a8_gemm(A, s, d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(Yb, Y, B, "config 1 " + kernel)


@pytest.mark.parametrize("kernel", ["small", "large"])
def test_gemm_one_hot_activations_read_back_weights(fq, kernel_choice, kernel):
    # A = identity: Y[m,n] = a_scale[m] * t * e4m3(gs[n, m/128]) * q[n,m] -- one product per output, so
    # every packed weight and every scale is read back individually (only bf16 rounding remains).
    K = 256; N = 96
    _, _, q, gs, t = _rand_codes(8, N, K, seed=77)
    a = np.random.default_rng(1).uniform(0.5, 2.0, K).astype(np.float32)
    for m0 in range(0, K, 64):
        M = 64
        A = np.zeros((M, K), np.uint8)
        A[np.arange(M), m0 + np.arange(M)] = 0x38
        kernel_choice(kernel)
        Yb = _run_gemm(fq, A, a[m0:m0 + M], q, gs, t)
        Y = oracle.w4a8_gemm(A, a[m0:m0 + M], q, gs, t)
        assert np.array_equal(Yb, oracle.bf16_round_array(Y)) or \
            np.array_equal(oracle.bf16_bits_to_f64(Yb), oracle.bf16_bits_to_f64(oracle.bf16_round_array(Y)))


@pytest.mark.parametrize("kernel", ["small", "large"])
def test_gemm_special_values(fq, kernel_choice, kernel):
    M, N, K = 48, 64, 512
    kernel_choice(kernel)
    ones = np.ones(M, np.float32)
    # all ones -> K exactly
    Yb = _run_gemm(fq, np.full((M, K), 0x38, np.uint8), ones, np.ones((N, K), np.int8),
                   np.full((N, K // 128), 0x38, np.uint8), 1.0)
    assert np.all(oracle.bf16_bits_to_f64(Yb) == K)
    # extremes: 448 * -8 * K, exactly representable in bf16 (7 * 2^9 * 512 * ... = -7 * 2^18)
    Yb = _run_gemm(fq, np.full((M, K), 0x7E, np.uint8), ones, np.full((N, K), -8, np.int8),
                   np.full((N, K // 128), 0x38, np.uint8), 1.0)
    assert np.all(oracle.bf16_bits_to_f64(Yb) == -3584.0 * K)
    # a zero-scale group contributes nothing (App. B, Lemma B.1); subnormal and negative scales work
    A, a, q, gs, t = _rand_codes(M, N, K, seed=5)
    gs[:, 1] = 0x00
    gs[:, 2] = 0x03
    gs[:, 3] = 0x85
    Yb = _run_gemm(fq, A, a, q, gs, t)
    Y, B = oracle.w4a8_gemm(A, a, q, gs, t, want_bound=True)
    check_gemm(Yb, Y, B, "special scales " + kernel)


def test_gemm_invariants_on_gpu(fq, kernel_choice):
    M, N, K = 300, 256, 1024
    A, a, q, gs, t = _rand_codes(M, N, K, seed=9)
    kernel_choice("large")
    Y1 = _run_gemm(fq, A, a, q, gs, t)
    Y2 = _run_gemm(fq, A, a, q, gs, 2 * t)
    assert np.array_equal(oracle.bf16_bits_to_f64(Y2), 2 * oracle.bf16_bits_to_f64(Y1))   # delta = 2^n is exact
    Yagain = _run_gemm(fq, A, a, q, gs, t)
    assert np.array_equal(Y1, Yagain)                                                     # deterministic
    kernel_choice("small")
    Yrow = _run_gemm(fq, A[5:6], a[5:6], q, gs, t)
    d = np.abs(oracle.bf16_bits_to_f64(Yrow)[0] - oracle.bf16_bits_to_f64(Y1)[5])
    # row independence: another kernel, other rows around it, same row result up to the FP32
    # summation order (a small fraction of the bound on the sum of |terms|) and one rounding step
    _, B = oracle.w4a8_gemm(A[5:6], a[5:6], q, gs, t, want_bound=True)
    assert np.all(d <= oracle.bf16_ulp_array(oracle.bf16_bits_to_f64(Y1)[5]) + 1e-4 * B[0])
    kernel_choice("auto")
    # the kernel chosen by shape (for this one the K-split kernel): the same sums in another FP32 order
    Yauto = _run_gemm(fq, A, a, q, gs, t)
    _, Bf = oracle.w4a8_gemm(A, a, q, gs, t, want_bound=True)
    assert np.all(np.abs(oracle.bf16_bits_to_f64(Yauto) - oracle.bf16_bits_to_f64(Y1))
                  <= oracle.bf16_ulp_array(oracle.bf16_bits_to_f64(Y1)) + 1e-4 * Bf)
    assert np.array_equal(_run_gemm(fq, A, a, q, gs, t), Yauto)


def test_own_workspace_and_callers_workspace_agree(fq):
    """fq_w4a8_gemm (library-owned workspace) and fq_w4a8_gemm_ws (caller's) give the same bits;
    a workspace that is too small is refused before anything is launched."""
    import ctypes
    M, N, K = 300, 256, 1024
    A, a, q, gs, t = _rand_codes(M, N, K, seed=21)
    Ad, ad, gd = _gpu(A), _gpu(a), _gpu(gs)
    packed = fq.fq_pack_weights(_gpu(q))
    need = fq.fq_w4a8_gemm_workspace_bytes(M, N, K)
    assert need > 0
    Y_ws = fq.fq_w4a8_gemm(Ad, ad, packed, gd, t, N, workspace=torch.empty(need + 64, dtype=torch.uint8, device="cuda"))
    Y_own = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    L = fq.lib()
    for _ in range(2):                                   # second call: the library's buffer already exists
        rc = L.fq_w4a8_gemm(Ad.data_ptr(), ad.data_ptr(), packed.data_ptr(), gd.data_ptr(), ctypes.c_float(t),
                            Y_own.data_ptr(), M, N, K, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0
    torch.cuda.synchronize()
    assert torch.equal(Y_own.view(torch.int16), Y_ws.view(torch.int16))
    Y, B = oracle.w4a8_gemm(A, a, q, gs, t, want_bound=True)
    check_gemm(bf16_bits_from_gpu(Y_own), Y, B, "library-owned workspace")
    small = torch.empty(need - 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(fq.FireqError):
        fq.fq_w4a8_gemm(Ad, ad, packed, gd, t, N, workspace=small)


@pytest.mark.parametrize("M,N,K", [(300, 256, 1024), (130, 96, 11008), (257, 160, 128)])
def test_quantiser_prepares_the_gemm_workspace(fq, M, N, K):
    """fq_quantize_act_ws writes the same codes and scales as fq_quantize_act, and the workspace it
    prepares gives the GEMM the oracle's result (and, up to FP32 summation order, the result of the
    GEMM that prepares the workspace itself)."""
    d = workloads.draw(M, N, K, seed=M + K)
    X = to_gpu_bf16(d["X_bf16"])
    A0, s0 = fq.fq_quantize_act(X)
    need = fq.fq_w4a8_gemm_workspace_bytes(M, N, K)
    ws = torch.full((need + 32,), 0xFF, dtype=torch.uint8, device="cuda")    # stale contents must not matter
    A1, s1 = fq.fq_quantize_act(X, workspace=ws)
    assert torch.equal(A0, A1) and torch.equal(s0, s1)
    packed = fq.fq_pack_weights(_gpu(d["q"]))
    gd = _gpu(d["gscale"])
    Y_prep = fq.fq_w4a8_gemm(A1, s1, packed, gd, d["w_tscale"], N, workspace=ws, workspace_prepared=True)
    Y_self = fq.fq_w4a8_gemm(A0, s0, packed, gd, d["w_tscale"], N)
    torch.cuda.synchronize()
    Y, B = oracle.w4a8_gemm(A0.cpu().numpy(), s0.cpu().numpy(), d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(bf16_bits_from_gpu(Y_prep), Y, B, "prepared workspace")
    check_gemm(bf16_bits_from_gpu(Y_self), Y, B, "own pre-pass")
    diff = np.abs(oracle.bf16_bits_to_f64(bf16_bits_from_gpu(Y_prep)) - oracle.bf16_bits_to_f64(bf16_bits_from_gpu(Y_self)))
    assert np.all(diff <= oracle.bf16_ulp_array(Y) + 1e-5 * B)


# ---- fused gate/up epilogue ------------------------------------------------------------------------

SWIGLU_SHAPES = {"simple": [(5, 64, 256), (33, 200, 384)],
                 "small": [(1, 32, 128), (16, 256, 512), (12, 14336, 384), (40, 200, 640), (64, 96, 1408)],
                 "large": [(65, 32, 128), (300, 256, 1024), (257, 528, 384), (512, 1024, 512), (130, 200, 640)]}


@pytest.mark.parametrize("kernel,shape", [(k, s) for k, v in SWIGLU_SHAPES.items() for s in v])
def test_gemm_swiglu_matches_oracle(fq, kernel_choice, kernel, shape):
    """H = SiLU(gate) * up against the oracle, gates of order one so that the nonlinear range is used."""
    M, N, K = shape
    d = workloads.draw(M, N, K, seed=3 * M + N + K, gs_lo=0.01, gs_hi=0.1, w_tscale=0.25, outlier_frac=0.01)
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
    packed = fq.fq_pack_weights(_gpu(d["q"]))
    kernel_choice(kernel)
    Hg = fq.fq_w4a8_gemm_swiglu(A, s, packed, _gpu(d["gscale"]), d["w_tscale"], N)
    torch.cuda.synchronize()
    assert tuple(Hg.shape) == (M, N // 2)
    An, sn = A.cpu().numpy(), s.cpu().numpy()
    H, B = oracle.w4a8_gemm_swiglu(An, sn, d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    Y = oracle.w4a8_gemm(An, sn, d["q"], d["gscale"], d["w_tscale"])
    assert 0.2 < np.median(np.abs(Y[:, 0::2])) < 20            # the gates sit where SiLU bends
    check_gemm(bf16_bits_from_gpu(Hg), H, B, "swiglu %s %s" % (kernel, shape))


def test_gemm_swiglu_pairs_even_gate_with_odd_up(fq, kernel_choice):
    """One-hot activations read back single weights: H[m, j] = SiLU(w[2j, m]) * w[2j+1, m] exactly as the
    oracle pairs them, for every kernel; the plain GEMM on the same buffers gives the two sums."""
    N, K = 64, 256
    rng = np.random.default_rng(4)
    q = rng.integers(-8, 8, (N, K), dtype=np.int8)
    gs = np.full((N, K // 128), 0x30, np.uint8)            # 0.5
    for kernel, M in (("simple", 8), ("small", 48), ("large", 256)):
        A = np.zeros((M, K), np.uint8)
        A[np.arange(M), np.arange(M) % K] = 0x38
        a = np.ones(M, np.float32)
        kernel_choice(kernel)
        packed = fq.fq_pack_weights(_gpu(q))
        Hg = bf16_bits_from_gpu(fq.fq_w4a8_gemm_swiglu(_gpu(A), _gpu(a), packed, _gpu(gs), 1.0, N))
        torch.cuda.synchronize()
        g = 0.5 * q[0::2, :M].T.astype(np.float64)             # [M, N/2]
        u = 0.5 * q[1::2, :M].T.astype(np.float64)
        want = g / (1.0 + np.exp(-g)) * u
        got = oracle.bf16_bits_to_f64(Hg)
        assert np.all(np.abs(got - want) <= oracle.bf16_ulp_array(want) + 1e-6), kernel


def test_ffn_gateup_swiglu_full_size(fq):
    """The fused gate/up layer at its real size (M=2048, 2 x 11008 interleaved rows, K=4096), through the
    fused quantiser, every element against the oracle."""
    name = "ffn_l2_7b_gateup_swiglu"
    w = workloads.WORKLOADS[name]
    d = workloads.draw_workload(name)
    need = fq.fq_w4a8_gemm_workspace_bytes(w.M, w.N, w.K)
    ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]), workspace=ws)
    packed = fq.fq_pack_weights(_gpu(d["q"]))
    Hg = fq.fq_w4a8_gemm_swiglu(A, s, packed, _gpu(d["gscale"]), d["w_tscale"], w.N, workspace=ws, workspace_prepared=True)
    torch.cuda.synchronize()
    An, sn = A.cpu().numpy(), s.cpu().numpy()
    H, B = oracle.w4a8_gemm_swiglu(An, sn, d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(bf16_bits_from_gpu(Hg), H, B, name)


# ---- residual added in the epilogue ---------------------------------------------------------------

ADD_SHAPES = {"simple": [(5, 64, 256), (33, 201, 384)],
              "small": [(1, 32, 128), (16, 256, 512), (12, 14336, 384), (40, 201, 640), (64, 96, 1408)],
              "large": [(65, 32, 128), (300, 256, 1024), (257, 528, 384), (512, 1024, 512), (130, 201, 640),
                        (384, 130, 256)]}


def _residual_bits(M, N, scale, seed):
    return workloads.draw_residual(M, N, scale=scale, seed=seed)


@pytest.mark.parametrize("kernel,shape", [(k, s) for k, v in ADD_SHAPES.items() for s in v])
def test_gemm_add_matches_oracle(fq, kernel_choice, kernel, shape):
    """Y = GEMM + R against the oracle, R of the GEMM's own magnitude; then the same call in place."""
    M, N, K = shape
    d = workloads.draw(M, N, K, seed=5 * M + N + K, outlier_frac=0.01)
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
    packed = fq.fq_pack_weights(_gpu(d["q"]))
    An, sn = A.cpu().numpy(), s.cpu().numpy()
    Y0 = oracle.w4a8_gemm(An, sn, d["q"], d["gscale"], d["w_tscale"])
    Rb = _residual_bits(M, N, float(np.std(Y0)) + 1e-3, seed=M + N)
    kernel_choice(kernel)
    R = to_gpu_bf16(Rb)
    Yg = fq.fq_w4a8_gemm_add(A, s, packed, _gpu(d["gscale"]), d["w_tscale"], N, R)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_bits_from_gpu(R), Rb)           # the residual itself is not written
    Y, B = oracle.w4a8_gemm_add(An, sn, d["q"], d["gscale"], d["w_tscale"], Rb, want_bound=True)
    check_gemm(bf16_bits_from_gpu(Yg), Y, B, "add %s %s" % (kernel, shape))
    Yi = fq.fq_w4a8_gemm_add(A, s, packed, _gpu(d["gscale"]), d["w_tscale"], N, R, out=R)
    torch.cuda.synchronize()
    assert Yi.data_ptr() == R.data_ptr()
    assert np.array_equal(bf16_bits_from_gpu(Yi), bf16_bits_from_gpu(Yg)), "in place differs"


def test_gemm_add_with_zero_activations_returns_the_residual(fq, kernel_choice):
    """All-zero activations: every output is bf16(0 + R[m,n]) = R[m,n] bit for bit, so each element of the
    residual has to arrive at its own place (whole tiles, half tiles and ragged edges of every kernel)."""
    K = 256
    for kernel, M, N in (("simple", 9, 70), ("small", 16, 264), ("small", 50, 1000), ("large", 256, 128),
                         ("large", 384, 392), ("large", 700, 1025)):
        q = np.random.default_rng(M).integers(-8, 8, (N, K), dtype=np.int8)
        gs = np.full((N, K // 128), 0x38, np.uint8)
        A = np.zeros((M, K), np.uint8)
        Rb = np.random.default_rng(N).integers(0, 0x7F80, (M, N)).astype(np.uint16)
        Rb |= np.random.default_rng(N + 1).integers(0, 2, (M, N)).astype(np.uint16) << 15
        Rb[Rb == 0x8000] = 0                                   # 0 + (-0) is +0
        kernel_choice(kernel)
        Yg = fq.fq_w4a8_gemm_add(_gpu(A), _gpu(np.ones(M, np.float32)), fq.fq_pack_weights(_gpu(q)), _gpu(gs), 1.0, N,
                                 to_gpu_bf16(Rb))
        torch.cuda.synchronize()
        got = bf16_bits_from_gpu(Yg)
        bad = np.argwhere(got != Rb)
        assert bad.size == 0, "%s M=%d N=%d: first wrong element %s" % (kernel, M, N, bad[:1])


def test_down_projection_with_residual_full_size(fq):
    """The down projection at its real size (M=2048, N=4096, K=11008) with the residual stream added in
    place, through the fused quantiser, every element against the oracle."""
    name = "ffn_l2_7b_down_residual"
    w = workloads.WORKLOADS[name]
    d = workloads.draw_workload(name)
    need = fq.fq_w4a8_gemm_workspace_bytes(w.M, w.N, w.K)
    ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]), workspace=ws)
    packed = fq.fq_pack_weights(_gpu(d["q"]))
    rows = np.arange(w.M)
    An, sn = A.cpu().numpy()[rows], s.cpu().numpy()[rows]
    Y0 = oracle.w4a8_gemm(An[:64], sn[:64], d["q"], d["gscale"], d["w_tscale"])
    Rb = _residual_bits(w.M, w.N, workloads.RESIDUAL_SCALE, seed=w.seed)
    assert 0.3 < np.std(Y0) / workloads.RESIDUAL_SCALE < 3       # residual and GEMM of like size
    R = to_gpu_bf16(Rb)
    fq.fq_w4a8_gemm_add(A, s, packed, _gpu(d["gscale"]), d["w_tscale"], w.N, R, out=R, workspace=ws, workspace_prepared=True)
    torch.cuda.synchronize()
    Y, B = oracle.w4a8_gemm_add(An, sn, d["q"], d["gscale"], d["w_tscale"], Rb[rows], want_bound=True)
    check_gemm(bf16_bits_from_gpu(R)[rows], Y, B, name + " + residual")


def test_m_zero_is_a_noop(fq):
    packed = torch.zeros(fq.fq_packed_weight_bytes(32, 128), dtype=torch.uint8, device="cuda")
    Y = fq.fq_w4a8_gemm(torch.zeros((0, 128), dtype=torch.uint8, device="cuda"),
                        torch.zeros((0,), dtype=torch.float32, device="cuda"), packed,
                        torch.zeros((32, 1), dtype=torch.uint8, device="cuda"), 1.0, 32)
    assert tuple(Y.shape) == (0, 32)


# ---- the benchmark configurations at full size ----------------------------------------------------

def _full_config(fq, name, sample_rows):
    """GPU on the whole problem, oracle on sampled rows (all N columns of each)."""
    w = workloads.WORKLOADS[name]
    d = workloads.draw_workload(name)
    X = to_gpu_bf16(d["X_bf16"])
    A_gpu, s_gpu = fq.fq_quantize_act(X)
    packed = fq.fq_pack_weights(_gpu(d["q"]))
    Y = fq.fq_w4a8_gemm(A_gpu, s_gpu, packed, _gpu(d["gscale"]), d["w_tscale"], w.N)
    torch.cuda.synchronize()
    rows = np.array(sorted(set(r for r in sample_rows if r < w.M)))
    A_ref, s_ref = oracle.quantize_act(d["X_bf16"][rows])
    assert np.array_equal(A_gpu.cpu().numpy()[rows] & 0x7F | (A_ref & 0x80), A_ref) or \
        np.array_equal(A_gpu.cpu().numpy()[rows], A_ref)
    assert np.array_equal(s_gpu.cpu().numpy()[rows], s_ref)
    Yr, B = oracle.w4a8_gemm(A_ref, s_ref, d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    stats = check_gemm(bf16_bits_from_gpu(Y)[rows], Yr, B, name)
    back = fq.fq_unpack_weights(packed, w.N, w.K)
    assert torch.equal(back.cpu(), torch.from_numpy(d["q"]))
    return stats


@pytest.mark.parametrize("name", ["c5_decode_m1", "c5_decode_m4", "c5_decode_m16", "c5_decode_m64"])
def test_config5_full(fq, name):
    _full_config(fq, name, range(64))


def _every_8th_row(M):
    """One row of every eight, its position inside the eight rotating: every 32-row MFMA tile of every
    256-row workgroup tile is hit, in every accumulator register position over any 8 consecutive tiles."""
    return [8 * i + (5 * i) % 8 for i in range(M // 8)]


@pytest.mark.parametrize("name,rows", [
    ("c2_l2_7b_gateup", None),                                 # every row
    ("c3_l2_7b_down", None),
    ("c4a_l3_8b_qkv", 8),                                      # one row in eight
    ("c4b_l3_8b_up", 8),
])
def test_large_configs_full_size(fq, name, rows):
    """The four large configurations at their real sizes, in the launch configuration bench.py times:
    c2 and c3 on every element, c4a / c4b on one row of every eight (all columns)."""
    M = workloads.WORKLOADS[name].M
    _full_config(fq, name, range(M) if rows is None else _every_8th_row(M))


@pytest.mark.parametrize("name", ["mid_l3_8b_up_m128", "mid_l3_8b_up_m256", "mid_l3_8b_up_m512",
                                  "mid_l2_7b_down_m128", "mid_l2_7b_down_m256", "mid_l2_7b_down_m512"])
def test_mid_m_configs_full_size(fq, name):
    """Batched-decode / chunked-prefill sizes that bench.py times (64 < M <= 512: the K-split kernel with and without
    K slices, and the large-M kernel), every element against the oracle."""
    _full_config(fq, name, range(workloads.WORKLOADS[name].M))


@pytest.mark.parametrize("shape", [(300, 512, 1024), (128, 256, 4096), (64, 8192, 1024)])
def test_ws_entry_points_replay_in_a_hip_graph(fq, shape):
    """The explicit-workspace entry points allocate nothing and keep no state, so a captured graph of
    quantiser + GEMM (plain, with residual, fused gate/up, fused gate/up with quantised output) can be replayed:
    three replays on fresh inputs, eager work and synchronisations between them, each replay equal to the eager
    result bit for bit.  The second shape takes the K-split kernel with four workgroups per tile, whose arrival
    counters must be back at zero after every GEMM of every replay; the third has no workspace at all (the K-split kernel's
    64 x 64 tiles for the plain and the residual form, the M <= 64 kernel for the fused gate/up layer)."""
    M, N, K = shape
    if shape[0] == 128:
        assert fq.fq_w4a8_gemm_plan(M, N, K)["ksplit_slices"] == 4
    if shape[0] == 64:
        assert fq.fq_w4a8_gemm_plan(M, N, K)["kernel"] == "ksplit64x64" and fq.fq_w4a8_gemm_workspace_bytes(M, N, K) == 0
    d = workloads.draw(M, N, K, seed=91, gs_lo=0.01, gs_hi=0.1, outlier_frac=0.01)
    packed = fq.fq_pack_weights(_gpu(d["q"]))
    gs = _gpu(d["gscale"])
    X = to_gpu_bf16(d["X_bf16"]).clone()
    R = to_gpu_bf16(workloads.draw_residual(M, N, scale=4.0, seed=92))
    ws = torch.empty((fq.fq_w4a8_gemm_workspace_bytes(M, N, K),), dtype=torch.uint8, device="cuda")
    A = torch.empty((M, K), dtype=torch.uint8, device="cuda")
    s = torch.empty((M,), dtype=torch.float32, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    Ya = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    H = torch.empty((M, N // 2), dtype=torch.bfloat16, device="cuda")
    Hq = torch.empty((M, N // 2), dtype=torch.bfloat16, device="cuda")
    Cq = torch.empty((M, N // 2), dtype=torch.uint8, device="cuda")
    hq = torch.empty((M,), dtype=torch.float32, device="cuda")
    L = fq.lib()

    def enqueue():
        st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        wsb = ws.numel()
        assert L.fq_quantize_act_ws(X.data_ptr(), A.data_ptr(), s.data_ptr(), M, K, ws.data_ptr(), wsb, st) == 0
        t = ctypes.c_float(d["w_tscale"])
        assert L.fq_w4a8_gemm_ws(A.data_ptr(), s.data_ptr(), packed.data_ptr(), gs.data_ptr(), t, Y.data_ptr(),
                                 M, N, K, ws.data_ptr(), wsb, 1, st) == 0
        assert L.fq_w4a8_gemm_add_ws(A.data_ptr(), s.data_ptr(), packed.data_ptr(), gs.data_ptr(), t, R.data_ptr(),
                                     Ya.data_ptr(), M, N, K, ws.data_ptr(), wsb, 1, st) == 0
        assert L.fq_w4a8_gemm_swiglu_ws(A.data_ptr(), s.data_ptr(), packed.data_ptr(), gs.data_ptr(), t, H.data_ptr(),
                                        M, N, K, ws.data_ptr(), wsb, 1, st) == 0
        assert L.fq_w4a8_gemm_swiglu_quant_ws(A.data_ptr(), s.data_ptr(), packed.data_ptr(), gs.data_ptr(), t, Hq.data_ptr(),
                                              Cq.data_ptr(), hq.data_ptr(), M, N, K, ws.data_ptr(), wsb, 1, None, 0, st) == 0

    enqueue()                                                  # warm-up outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        Xn = to_gpu_bf16(workloads.draw(M, N, K, seed=100 + rep, outlier_frac=0.01)["X_bf16"])
        X.copy_(Xn)
        for out in (Y, Ya, H, A, Hq, Cq, hq):
            out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [bf16_bits_from_gpu(Y).copy(), bf16_bits_from_gpu(Ya).copy(), bf16_bits_from_gpu(H).copy()]
        assert torch.equal(Hq.view(torch.int16), H.view(torch.int16))
        C_e, h_e = fq.fq_quantize_act(H)
        assert torch.equal(Cq, C_e) and torch.equal(hq, h_e), "replay %d: quantised gate/up output" % rep
        A2, s2 = fq.fq_quantize_act(Xn)                        # eager, library-owned paths
        want = [bf16_bits_from_gpu(fq.fq_w4a8_gemm(A2, s2, packed, gs, d["w_tscale"], N)),
                bf16_bits_from_gpu(fq.fq_w4a8_gemm_add(A2, s2, packed, gs, d["w_tscale"], N, R)),
                bf16_bits_from_gpu(fq.fq_w4a8_gemm_swiglu(A2, s2, packed, gs, d["w_tscale"], N))]
        torch.cuda.synchronize()
        assert torch.equal(A, A2)
        for g, w, what in zip(got, want, ("gemm", "add", "swiglu")):
            assert np.array_equal(g, w), "replay %d: %s differs from the eager call" % (rep, what)
    # and the last replay against the oracle
    Yr, B = oracle.w4a8_gemm(A.cpu().numpy(), s.cpu().numpy(), d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(got[0], Yr, B, "graph replay")


# ---- the whole layer from bf16 activations (one kernel for M <= 6, K <= 4096) -------------------

LINEAR_SHAPES = [(6, 256, 512), (1, 32, 128), (5, 100, 384), (6, 4120, 512), (6, 8192, 4096), (4, 4096, 4096),
                 (3, 9000, 256), (6, 14336, 4096), (1, 14336, 4096), (5, 300, 1408), (2, 6144, 3072), (7, 100, 384),
                 # not served by the one-kernel form: long K, more rows, the large-M kernel
                 (16, 200, 8192), (40, 96, 1408), (300, 256, 1024)]


@pytest.mark.parametrize("shape", LINEAR_SHAPES)
def test_linear_matches_oracle_and_the_two_step_path(fq, shape):
    """fq_w4a8_linear against the oracle (quantiser then GEMM), and bit for bit against fq_quantize_act +
    fq_w4a8_gemm on the GPU: the fused kernel must quantise exactly as the quantiser kernel does."""
    M, N, K = shape
    d = workloads.draw(M, N, K, seed=7 * M + N + K, outlier_frac=0.01)
    if M > 2:
        d["X_bf16"][1, :] = 0                                  # an all-zero row takes scale 1
    X = to_gpu_bf16(d["X_bf16"])
    packed = fq.fq_pack_weights(_gpu(d["q"]))
    gs = _gpu(d["gscale"])
    need = fq.fq_w4a8_linear_workspace_bytes(M, N, K)
    assert (need == 0) == (M <= 6 and K <= 4096)
    Yl = fq.fq_w4a8_linear(X, packed, gs, d["w_tscale"], N)
    A, s = fq.fq_quantize_act(X)
    Y2 = fq.fq_w4a8_gemm(A, s, packed, gs, d["w_tscale"], N)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_bits_from_gpu(Yl), bf16_bits_from_gpu(Y2)), "differs from quantiser + GEMM"
    Yr, B = oracle.w4a8_linear(d["X_bf16"], d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(bf16_bits_from_gpu(Yl), Yr, B, "linear %s" % (shape,))


def test_linear_on_every_bf16_magnitude(fq):
    """Rows whose maxima span the whole bf16 range (tiny, huge, subnormal neighbours): the fused kernel's
    codes decide the output, so any difference from the quantiser kernel would show in the comparison."""
    M, N, K = 6, 64, 512
    rng = np.random.default_rng(3)
    X = rng.standard_normal((M, K)).astype(np.float32)
    X *= (2.0 ** np.array([-126, -70, -10, 0, 60, 126]))[:, None].astype(np.float32)
    Xb = workloads.f32_to_bf16_bits(X)
    d = workloads.draw(M, N, K, seed=5)
    packed = fq.fq_pack_weights(_gpu(d["q"]))
    gs = _gpu(d["gscale"])
    Yl = fq.fq_w4a8_linear(to_gpu_bf16(Xb), packed, gs, 1.0, N)
    A, s = fq.fq_quantize_act(to_gpu_bf16(Xb))
    Y2 = fq.fq_w4a8_gemm(A, s, packed, gs, 1.0, N)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_bits_from_gpu(Yl), bf16_bits_from_gpu(Y2))
    An, sn = oracle.quantize_act(Xb)
    assert np.array_equal(A.cpu().numpy() & 0x7F, An & 0x7F) and np.array_equal(s.cpu().numpy(), sn)


# ---- the paper's table mode (Sec. 3.1.1 step 1) ----------------------------------------------------

LUT_SHAPES = [("simple", (5, 64, 256)), ("simple", (33, 100, 384)),
              ("large", (16, 256, 512)), ("large", (65, 33, 128)), ("large", (300, 200, 640)), ("large", (257, 513, 384)),
              ("large", (512, 256, 1408)), ("large", (2048, 8192, 256)), ("large", (2100, 4112, 384))]


@pytest.mark.parametrize("kernel,shape", LUT_SHAPES)
def test_gemm_table_mode_matches_its_oracle(fq, kernel_choice, kernel, shape):
    """fq_w4a8_gemm_lut against the oracle's table-form GEMM (every weight E4M3(q * sigma)), element by element at
    the tolerance of the exact mode (one bf16 step + 1e-3 of the sum of |terms|); the scales span subnormals,
    normals and a few that saturate the table."""
    M, N, K = shape
    A, a, q, gs, t = _rand_codes(M, N, K, seed=2 * M + N + K)
    gs[0, :] = 0x7E                                            # 448: every entry but 0 and +-1 saturates
    gs[N // 2, :] = 0x00                                       # zero scale: an all-zero table (App. B, Lemma B.1)
    kernel_choice(kernel if kernel == "simple" else "auto")
    Yg = fq.fq_w4a8_gemm_lut(_gpu(A), _gpu(a), fq.fq_pack_weights(_gpu(q)), _gpu(gs), t, N)
    torch.cuda.synchronize()
    Y, B = oracle.w4a8_gemm_lut(A, a, q, gs, t, want_bound=True)
    # (channel 0 saturates and carries the whole norm: element-wise criterion only)
    check_gemm(bf16_bits_from_gpu(Yg), Y, B, "table mode %s %s" % (kernel, shape), frobenius=False)


def test_table_mode_equals_exact_mode_for_power_of_two_scales(fq):
    """Power-of-two scales: q * sigma keeps q's four bits, the table rounds nothing, and the two modes compute
    the same sums (each to its own FP32 summation order: equal within a few FP32 steps of the bound)."""
    M, N, K = 300, 256, 1024
    A, a, q, gs, t = _rand_codes(M, N, K, seed=77)
    gs = (np.random.default_rng(3).integers(2, 12, gs.shape).astype(np.uint8) << 3)
    Ad, ad, pk, gd = _gpu(A), _gpu(a), fq.fq_pack_weights(_gpu(q)), _gpu(gs)
    Yl = bf16_bits_from_gpu(fq.fq_w4a8_gemm_lut(Ad, ad, pk, gd, t, N))
    Ye = bf16_bits_from_gpu(fq.fq_w4a8_gemm(Ad, ad, pk, gd, t, N))
    torch.cuda.synchronize()
    Y, B = oracle.w4a8_gemm(A, a, q, gs, t, want_bound=True)
    d = np.abs(oracle.bf16_bits_to_f64(Yl) - oracle.bf16_bits_to_f64(Ye))
    assert np.all(d <= oracle.bf16_ulp_array(Y) + 1e-4 * B)
    check_gemm(Yl, Y, B, "table mode, power-of-two scales, against the exact oracle")


def test_table_mode_full_size_and_what_it_costs(fq):
    """c2 at full size in table mode: every element against the table-form oracle, and the relative Frobenius
    distance of the two modes on the GPU, which must be the oracle's (about 2 %: ten times the error budget)."""
    name = "c2_l2_7b_gateup"
    w = workloads.WORKLOADS[name]
    d = workloads.draw_workload(name)
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
    pk, gd = fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"])
    Yl = bf16_bits_from_gpu(fq.fq_w4a8_gemm_lut(A, s, pk, gd, d["w_tscale"], w.N))
    Ye = bf16_bits_from_gpu(fq.fq_w4a8_gemm(A, s, pk, gd, d["w_tscale"], w.N))
    torch.cuda.synchronize()
    An, sn = A.cpu().numpy(), s.cpu().numpy()
    Y, B = oracle.w4a8_gemm_lut(An, sn, d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(Yl, Y, B, name + " table mode")
    rows = slice(0, 256)
    exact = oracle.w4a8_gemm(An[rows], sn[rows], d["q"], d["gscale"], d["w_tscale"])
    rel_oracle = np.linalg.norm(Y[rows] - exact) / np.linalg.norm(exact)
    yl, ye = oracle.bf16_bits_to_f64(Yl[rows]), oracle.bf16_bits_to_f64(Ye[rows])
    rel_gpu = np.linalg.norm(yl - ye) / np.linalg.norm(ye)
    assert 0.01 < rel_oracle < 0.04 and abs(rel_gpu - rel_oracle) < 0.002, (rel_gpu, rel_oracle)
