"""GPU parity of every path of the large-M kernel: whole tiles (256 rows x 128 channels) and half tiles,
with whole-row stores and with element-wise stores at ragged edges, each as the plain GEMM, with the
residual added (out of place and in place) and with the fused gate/up epilogue -- every output element
against the CPU oracle.  Which path a shape takes depends on the device's compute-unit count, so each
test first asks the library (fq_w4a8_gemm_plan) and asserts that the shape reaches the path it is meant for."""
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
    binding.fq_test_force_kernel(None)
    return binding


def _gpu(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# shape -> the kinds of work item it must contain on this device
WHOLE_EVEN = (2048, 8192, 256)       # 512 whole tiles, nothing ragged
WHOLE_RAGGED = (2100, 4112, 384)     # whole tiles; last row tile has 52 rows, last channel tile 16 channels
MIXED = (2048, 8200, 256)            # whole tiles, half tiles, and a ragged last channel tile of 8 channels


def _plan(fq, shape):
    return fq.fq_w4a8_gemm_plan(*shape)


def test_shapes_reach_the_paths_they_are_meant_for(fq):
    p = _plan(fq, WHOLE_EVEN)
    assert p["kernel"] == "large" and p["whole"] > 0 and p["whole_ragged"] == p["half"] == p["half_ragged"] == 0
    p = _plan(fq, WHOLE_RAGGED)
    assert p["whole"] > 0 and p["whole_ragged"] > 0
    p = _plan(fq, MIXED)
    assert p["whole"] > 0 and p["half"] > 0 and p["whole_ragged"] + p["half_ragged"] > 0
    # the benchmark workloads: c2 mixes whole and half tiles, c4a / c4b are whole tiles throughout
    assert _plan(fq, (2048, 11008, 4096))["whole"] > 0
    assert _plan(fq, (8192, 14336, 4096))["whole"] == 32 * 112
    assert _plan(fq, (8192, 4096, 4096))["whole"] > 0          # attention output projection at prefill, with residual


def _problem(shape, seed, **kw):
    M, N, K = shape
    return workloads.draw(M, N, K, seed=seed, outlier_frac=0.01, **kw)


@pytest.mark.parametrize("shape", [WHOLE_EVEN, WHOLE_RAGGED, MIXED])
def test_plain_gemm_every_element(fq, shape):
    M, N, K = shape
    d = _problem(shape, seed=M + N)
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
    Yg = fq.fq_w4a8_gemm(A, s, fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"]), d["w_tscale"], N)
    torch.cuda.synchronize()
    Y, B = oracle.w4a8_gemm(A.cpu().numpy(), s.cpu().numpy(), d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(bf16_bits_from_gpu(Yg), Y, B, "plain %s" % (shape,))


@pytest.mark.parametrize("shape", [WHOLE_EVEN, WHOLE_RAGGED, MIXED])
def test_residual_every_element_and_in_place(fq, shape):
    M, N, K = shape
    d = _problem(shape, seed=2 * M + N)
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
    packed, gs = fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"])
    An, sn = A.cpu().numpy(), s.cpu().numpy()
    Rb = workloads.draw_residual(M, N, scale=4.0, seed=M + N)
    R = to_gpu_bf16(Rb)
    Yg = fq.fq_w4a8_gemm_add(A, s, packed, gs, d["w_tscale"], N, R)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_bits_from_gpu(R), Rb)           # the residual itself is not written
    Y, B = oracle.w4a8_gemm_add(An, sn, d["q"], d["gscale"], d["w_tscale"], Rb, want_bound=True)
    check_gemm(bf16_bits_from_gpu(Yg), Y, B, "add %s" % (shape,))
    Yi = fq.fq_w4a8_gemm_add(A, s, packed, gs, d["w_tscale"], N, R, out=R)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_bits_from_gpu(Yi), bf16_bits_from_gpu(Yg)), "in place differs"


@pytest.mark.parametrize("shape", [WHOLE_EVEN, WHOLE_RAGGED, MIXED])
def test_swiglu_every_element(fq, shape):
    M, N, K = shape
    d = _problem(shape, seed=3 * M + N, gs_lo=0.01, gs_hi=0.1, w_tscale=0.25)
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
    Hg = fq.fq_w4a8_gemm_swiglu(A, s, fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"]), d["w_tscale"], N)
    torch.cuda.synchronize()
    H, B = oracle.w4a8_gemm_swiglu(A.cpu().numpy(), s.cpu().numpy(), d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(bf16_bits_from_gpu(Hg), H, B, "swiglu %s" % (shape,))


@pytest.mark.parametrize("shape", [WHOLE_EVEN, WHOLE_RAGGED, MIXED])
def test_zero_activations_return_the_residual_bit_for_bit(fq, shape):
    """All-zero activations: every output is bf16(0 + R[m,n]) = R[m,n], so each element of the residual has to
    arrive at its own place in every kind of tile."""
    M, N, K = shape
    q = np.random.default_rng(M).integers(-8, 8, (N, K), dtype=np.int8)
    gs = np.full((N, K // 128), 0x38, np.uint8)
    Rb = np.random.default_rng(N).integers(0, 0x7F80, (M, N)).astype(np.uint16)
    Rb |= np.random.default_rng(N + 1).integers(0, 2, (M, N)).astype(np.uint16) << 15
    Rb[Rb == 0x8000] = 0                                       # 0 + (-0) is +0
    Yg = fq.fq_w4a8_gemm_add(_gpu(np.zeros((M, K), np.uint8)), _gpu(np.ones(M, np.float32)),
                             fq.fq_pack_weights(_gpu(q)), _gpu(gs), 1.0, N, to_gpu_bf16(Rb))
    torch.cuda.synchronize()
    bad = np.argwhere(bf16_bits_from_gpu(Yg) != Rb)
    assert bad.size == 0, "%s: first wrong element %s" % (shape, bad[:1])


def test_exactly_sized_workspace_with_ragged_rows(fq):
    """A workspace of exactly fq_w4a8_gemm_workspace_bytes, placed at the very end of an allocation whose next
    bytes hold a pattern: the result is the oracle's, and the bytes behind the workspace are never written."""
    M, N, K = 300, 256, 1024
    d = workloads.draw(M, N, K, seed=17, outlier_frac=0.01)
    need = fq.fq_w4a8_gemm_workspace_bytes(M, N, K)
    arena = torch.full((need + 4096,), 0xA5, dtype=torch.uint8, device="cuda")
    ws = arena[:need]
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]), workspace=ws)
    Yg = fq.fq_w4a8_gemm(A, s, fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"]), d["w_tscale"], N, workspace=ws,
                         workspace_prepared=True)
    torch.cuda.synchronize()
    assert bool((arena[need:] == 0xA5).all())
    Y, B = oracle.w4a8_gemm(A.cpu().numpy(), s.cpu().numpy(), d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(bf16_bits_from_gpu(Yg), Y, B, "exact workspace")


def test_attention_output_projection_with_residual_at_prefill_size(fq):
    """M = 8192, N = K = 4096 (Llama3-8B attention output projection at prefill) with the residual stream updated
    in place: whole tiles + residual at a real size, one row of every eight against the oracle."""
    M, N, K = 8192, 4096, 4096
    d = workloads.draw(M, N, K, seed=41, act="laplace", outlier_frac=0.01)
    need = fq.fq_w4a8_gemm_workspace_bytes(M, N, K)
    ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]), workspace=ws)
    rows = np.array([8 * i + (5 * i) % 8 for i in range(M // 8)])
    Rb = workloads.draw_residual(M, N, scale=workloads.RESIDUAL_SCALE, seed=42)
    R = to_gpu_bf16(Rb)
    fq.fq_w4a8_gemm_add(A, s, fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"]), d["w_tscale"], N, R, out=R,
                        workspace=ws, workspace_prepared=True)
    torch.cuda.synchronize()
    Y, B = oracle.w4a8_gemm_add(A.cpu().numpy()[rows], s.cpu().numpy()[rows], d["q"], d["gscale"], d["w_tscale"],
                                Rb[rows], want_bound=True)
    check_gemm(bf16_bits_from_gpu(R)[rows], Y, B, "o_proj + residual")


# ---- the K-split kernel (8-wave workgroups that split K inside the workgroup) --------------------------

KSPLIT_SHAPES = [(65, 64, 1024), (128, 128, 1024), (300, 256, 1024), (129, 200, 1408), (512, 520, 2048),
                 (100, 96, 11008), (130, 64, 16384), (257, 513, 1024),
                 # 256 x 128 tiles with K halved
                 (700, 1100, 2048), (1024, 512, 4096), (600, 264, 11008), (513, 130, 1408)]


def test_few_tile_shapes_take_the_k_split_kernel(fq):
    assert _plan(fq, (128, 14336, 4096))["kernel"] == "ksplit128x64"
    assert _plan(fq, (512, 4096, 4096))["kernel"] == "ksplit128x64"
    assert _plan(fq, (512, 14336, 4096))["kernel"] == "large"              # more than one round of 128 x 64 tiles
    assert _plan(fq, (2048, 11008, 4096))["kernel"] == "large"
    # workgroups that share a tile along K: as many as fill the compute units, two groups or more per K split each
    assert _plan(fq, (128, 4096, 4096))["ksplit_slices"] == 4
    assert _plan(fq, (128, 4096, 11008))["ksplit_slices"] == 4
    assert _plan(fq, (256, 4096, 4096))["ksplit_slices"] == 2
    assert _plan(fq, (512, 4096, 4096))["ksplit_slices"] == 1
    assert _plan(fq, (100, 96, 11008))["ksplit_slices"] == 8
    assert _plan(fq, (129, 200, 1408))["ksplit_slices"] == 1
    fq.fq_test_force_kernel("ksplit")
    try:
        for shape in KSPLIT_SHAPES:
            assert _plan(fq, shape)["kernel"] == ("ksplit128x64" if shape[0] <= 512 else "ksplit256x128"), shape
    finally:
        fq.fq_test_force_kernel(None)


@pytest.mark.parametrize("shape", KSPLIT_SHAPES)
def test_k_split_kernel_every_element(fq, shape):
    """Plain GEMM, residual out of place and in place, on the K-split kernel: even and ragged tiles, K splits of
    unequal length (K/128 = 11, 43 + 43), several rounds of zero-point units (K = 16384), against the oracle; and the
    large-M kernel's result on the same operands within the FP32 summation-order margin."""
    M, N, K = shape
    d = _problem(shape, seed=7 * M + N + K)
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
    packed, gs = fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"])
    An, sn = A.cpu().numpy(), s.cpu().numpy()
    Rb = workloads.draw_residual(M, N, scale=4.0, seed=M + N)
    R = to_gpu_bf16(Rb)
    try:
        fq.fq_test_force_kernel("ksplit")
        Yk = fq.fq_w4a8_gemm(A, s, packed, gs, d["w_tscale"], N)
        Ya = fq.fq_w4a8_gemm_add(A, s, packed, gs, d["w_tscale"], N, R)
        torch.cuda.synchronize()
        assert np.array_equal(bf16_bits_from_gpu(R), Rb)
        Yi = fq.fq_w4a8_gemm_add(A, s, packed, gs, d["w_tscale"], N, R, out=R)
        Yk2 = fq.fq_w4a8_gemm(A, s, packed, gs, d["w_tscale"], N)
        fq.fq_test_force_kernel("large")
        Yl = fq.fq_w4a8_gemm(A, s, packed, gs, d["w_tscale"], N)
        torch.cuda.synchronize()
    finally:
        fq.fq_test_force_kernel(None)
    Y, B = oracle.w4a8_gemm(An, sn, d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(bf16_bits_from_gpu(Yk), Y, B, "k-split %s" % (shape,))
    assert np.array_equal(bf16_bits_from_gpu(Yk), bf16_bits_from_gpu(Yk2)), "not deterministic"
    diff = np.abs(oracle.bf16_bits_to_f64(bf16_bits_from_gpu(Yk)) - oracle.bf16_bits_to_f64(bf16_bits_from_gpu(Yl)))
    assert np.all(diff <= oracle.bf16_ulp_array(Y) + 1e-4 * B)
    Yr, Br = oracle.w4a8_gemm_add(An, sn, d["q"], d["gscale"], d["w_tscale"], Rb, want_bound=True)
    check_gemm(bf16_bits_from_gpu(Ya), Yr, Br, "k-split + residual %s" % (shape,))
    assert np.array_equal(bf16_bits_from_gpu(Yi), bf16_bits_from_gpu(Ya)), "in place differs"


# 56 < M <= 64 with at least half a round of 64 x 64 tiles: the K-split kernel without a workspace (zero point through
# the matrix cores); ragged last channel tile (8200), K splits of unequal length (K / 128 = 11), every K split a ghost
# step short of the others (K / 128 = 9)
KSPLIT64_SHAPES = [(64, 8192, 1024), (57, 16384, 1024), (60, 8200, 1408), (64, 8256, 1152)]


@pytest.mark.parametrize("shape", KSPLIT64_SHAPES)
def test_k_split_kernel_without_workspace_every_element(fq, shape):
    """Plain GEMM and residual (out of place, in place) on 64 x 64 tiles against the oracle, and against the M <= 64
    kernel, whose arithmetic it shares (same zero-point instruction, same order inside a group): equal within the FP32
    summation-order margin."""
    M, N, K = shape
    assert _plan(fq, shape)["kernel"] == "ksplit64x64" and fq.fq_w4a8_gemm_workspace_bytes(M, N, K) == 0
    d = _problem(shape, seed=5 * M + N + K)
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
    packed, gs = fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"])
    An, sn = A.cpu().numpy(), s.cpu().numpy()
    Rb = workloads.draw_residual(M, N, scale=4.0, seed=M + N)
    R = to_gpu_bf16(Rb)
    try:
        Yk = fq.fq_w4a8_gemm(A, s, packed, gs, d["w_tscale"], N)
        Ya = fq.fq_w4a8_gemm_add(A, s, packed, gs, d["w_tscale"], N, R)
        torch.cuda.synchronize()
        assert np.array_equal(bf16_bits_from_gpu(R), Rb)
        Yi = fq.fq_w4a8_gemm_add(A, s, packed, gs, d["w_tscale"], N, R, out=R)
        Yk2 = fq.fq_w4a8_gemm(A, s, packed, gs, d["w_tscale"], N)
        fq.fq_test_force_kernel("small")
        assert _plan(fq, shape)["kernel"] == "smallm"
        Ys = fq.fq_w4a8_gemm(A, s, packed, gs, d["w_tscale"], N)
        torch.cuda.synchronize()
    finally:
        fq.fq_test_force_kernel(None)
    Y, B = oracle.w4a8_gemm(An, sn, d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(bf16_bits_from_gpu(Yk), Y, B, "k-split 64 x 64 %s" % (shape,))
    assert np.array_equal(bf16_bits_from_gpu(Yk), bf16_bits_from_gpu(Yk2)), "not deterministic"
    diff = np.abs(oracle.bf16_bits_to_f64(bf16_bits_from_gpu(Yk)) - oracle.bf16_bits_to_f64(bf16_bits_from_gpu(Ys)))
    assert np.all(diff <= oracle.bf16_ulp_array(Y) + 1e-4 * B)
    Yr, Br = oracle.w4a8_gemm_add(An, sn, d["q"], d["gscale"], d["w_tscale"], Rb, want_bound=True)
    check_gemm(bf16_bits_from_gpu(Ya), Yr, Br, "k-split 64 x 64 + residual %s" % (shape,))
    assert np.array_equal(bf16_bits_from_gpu(Yi), bf16_bits_from_gpu(Ya)), "in place differs"


def test_k_split_kernel_without_workspace_keeps_to_its_shapes(fq):
    assert _plan(fq, (64, 14336, 4096))["kernel"] == "ksplit64x64"          # the decode sweep's largest batch
    assert _plan(fq, (56, 14336, 4096))["kernel"] == "smallm"               # below the top of the range
    assert _plan(fq, (64, 4096, 4096))["kernel"] == "smallm"                # a quarter of a round of tiles
    assert _plan(fq, (64, 14336, 11008))["kernel"] == "smallm"              # long K
    assert _plan(fq, (64, 16448, 4096))["kernel"] == "smallm"               # more than one round
    assert _plan(fq, (64, 8192, 512))["kernel"] == "smallm"                 # fewer than two groups per K split
    assert _plan(fq, (65, 14336, 4096))["kernel"] == "ksplit128x64"


def test_k_split_kernel_zero_activations_return_the_residual(fq):
    for shape in [(300, 264, 1024), (1024, 640, 2048), (700, 1032, 2048)]:
        M, N, K = shape
        q = np.random.default_rng(M).integers(-8, 8, (N, K), dtype=np.int8)
        gs = np.full((N, K // 128), 0x38, np.uint8)
        Rb = np.random.default_rng(N).integers(0, 0x7F80, (M, N)).astype(np.uint16)
        Rb |= np.random.default_rng(N + 1).integers(0, 2, (M, N)).astype(np.uint16) << 15
        Rb[Rb == 0x8000] = 0
        try:
            fq.fq_test_force_kernel("ksplit")
            Yg = fq.fq_w4a8_gemm_add(_gpu(np.zeros((M, K), np.uint8)), _gpu(np.ones(M, np.float32)),
                                     fq.fq_pack_weights(_gpu(q)), _gpu(gs), 1.0, N, to_gpu_bf16(Rb))
            torch.cuda.synchronize()
        finally:
            fq.fq_test_force_kernel(None)
        bad = np.argwhere(bf16_bits_from_gpu(Yg) != Rb)
        assert bad.size == 0, "%s: first wrong element %s" % (shape, bad[:1])


def test_a_prepared_workspace_serves_several_sliced_gemms(fq):
    """Projections that share one activation matrix run one after the other on the workspace the quantiser
    prepared: the tiles' arrival counters are back at zero after every call, so each result equals the one a
    freshly prepared workspace gives, bit for bit, and matches the oracle."""
    M, K = 128, 4096
    shapes_n = [1024, 320, 1024]
    ds = [_problem((M, N, K), seed=90 + i) for i, N in enumerate(shapes_n)]
    X = to_gpu_bf16(ds[0]["X_bf16"])
    need = max(fq.fq_w4a8_gemm_workspace_bytes(M, N, K) for N in shapes_n)
    for N in shapes_n:
        assert _plan(fq, (M, N, K))["ksplit_slices"] == 4
    ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
    A, s = fq.fq_quantize_act(X, workspace=ws)
    outs = []
    for d, N in zip(ds, shapes_n):
        packed, gs = fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"])
        outs.append(fq.fq_w4a8_gemm(A, s, packed, gs, d["w_tscale"], N, workspace=ws, workspace_prepared=True))
    torch.cuda.synchronize()
    An, sn = A.cpu().numpy(), s.cpu().numpy()
    for d, N, Yg in zip(ds, shapes_n, outs):
        packed, gs = fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"])
        fresh = fq.fq_w4a8_gemm(A, s, packed, gs, d["w_tscale"], N)
        torch.cuda.synchronize()
        assert np.array_equal(bf16_bits_from_gpu(Yg), bf16_bits_from_gpu(fresh)), N
        Y, B = oracle.w4a8_gemm(An, sn, d["q"], d["gscale"], d["w_tscale"], want_bound=True)
        check_gemm(bf16_bits_from_gpu(Yg), Y, B, "shared workspace, N = %d" % N)
