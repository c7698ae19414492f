"""fq_w4a8_gemm_swiglu_quant_ws -- the fused gate/up layer whose output also leaves as the FP8 input of the next
layer (Sec. 3.1.1 step 3, Fig. 1) -- on the GPU: H_bf16 equals what fq_w4a8_gemm_swiglu_ws gives, the codes and
scales equal what the oracle's quantiser (Sec. 2.1 eq. 2) makes of that H, bit for bit, and a workspace prepared
on the way serves the next GEMM."""
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
    binding.fq_test_force_kernel(None)
    return binding


def _gpu(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _same_codes(got, want):
    """E4M3 codes equal, the sign of a zero aside."""
    return np.array_equal(got & 0x7F, want & 0x7F) and np.array_equal((got & 0x80)[(want & 0x7F) != 0],
                                                                     (want & 0x80)[(want & 0x7F) != 0])


# whole 256-row tiles (64 per XCD), whole tiles with ragged edges, half tiles, a ragged small problem, M <= 64
SHAPES = [(2048, 8192, 256), (2100, 4112, 384), (300, 512, 1024), (65, 48, 128), (130, 272, 256), (16, 256, 512),
          (40, 208, 640)]


@pytest.mark.parametrize("shape", SHAPES)
def test_codes_and_scales_are_those_of_the_quantiser_on_the_same_h(fq, shape):
    M, N, K = shape
    d = workloads.draw(M, N, K, seed=3 * M + N + K, gs_lo=0.01, gs_hi=0.1, outlier_frac=0.01)
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
    packed, gs = fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"])
    H_ref = fq.fq_w4a8_gemm_swiglu(A, s, packed, gs, d["w_tscale"], N)
    H, C, hs = fq.fq_w4a8_gemm_swiglu_quant(A, s, packed, gs, d["w_tscale"], N)
    C2, hs2 = fq.fq_quantize_act(H_ref)
    torch.cuda.synchronize()
    Hb = bf16_bits_from_gpu(H)
    assert np.array_equal(Hb, bf16_bits_from_gpu(H_ref))
    assert torch.equal(C, C2) and torch.equal(hs, hs2)
    # the oracle's quantiser on the very same bf16 numbers
    C_or, s_or = oracle.quantize_act(Hb)
    assert np.array_equal(hs.cpu().numpy(), s_or)
    assert _same_codes(C.cpu().numpy(), C_or)
    # and H itself against the oracle's fused layer
    Ho, B = oracle.w4a8_gemm_swiglu(A.cpu().numpy(), s.cpu().numpy(), d["q"], d["gscale"], d["w_tscale"], want_bound=True)
    check_gemm(Hb, Ho, B, "gate/up + quantised output %s" % (shape,))


def test_two_calls_in_a_row_leave_nothing_behind(fq):
    """The row maxima live in the scale array between the two kernels of a call: a second call with other operands
    (smaller magnitudes) into the same arrays must not see the first call's maxima."""
    M, N, K = 512, 1024, 512
    L = fq.lib()
    import ctypes
    outs = []
    H = torch.empty((M, N // 2), dtype=torch.bfloat16, device="cuda")
    C = torch.empty((M, N // 2), dtype=torch.uint8, device="cuda")
    hs = torch.empty((M,), dtype=torch.float32, device="cuda")
    for seed, tscale in ((5, 4.0), (6, 0.03125)):
        d = workloads.draw(M, N, K, seed=seed, gs_lo=0.01, gs_hi=0.1, outlier_frac=0.01)
        A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
        packed, gs = fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"])
        need = fq.fq_w4a8_gemm_workspace_bytes(M, N, K)
        ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
        rc = L.fq_w4a8_gemm_swiglu_quant_ws(A.data_ptr(), s.data_ptr(), packed.data_ptr(), gs.data_ptr(),
                                            ctypes.c_float(tscale), H.data_ptr(), C.data_ptr(), hs.data_ptr(), M, N, K,
                                            ws.data_ptr(), need, 0, None, 0,
                                            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0
        torch.cuda.synchronize()
        C_or, s_or = oracle.quantize_act(bf16_bits_from_gpu(H))
        assert np.array_equal(hs.cpu().numpy(), s_or), seed
        assert _same_codes(C.cpu().numpy(), C_or), seed
        outs.append(float(hs.max()))
    assert outs[1] < outs[0] / 16                             # the second problem really is smaller


def test_feed_forward_chain_at_full_size(fq):
    """Llama2-7B feed-forward block, 2048 tokens: gate/up with the fused epilogue and quantised output, its prepared
    workspace, then the down projection on the codes -- equal, bit for bit, to the chain through the separate
    quantiser; codes and scales against the oracle's quantiser on sampled rows."""
    name = "ffn_l2_7b_gateup_swiglu"
    w = workloads.WORKLOADS[name]
    d = workloads.draw_workload(name)
    NH, ND = w.N // 2, 4096
    dd = workloads.draw(8, ND, NH, seed=77, gs_lo=0.005, gs_hi=0.05, outlier_frac=0.0)      # weights of the down projection
    need = fq.fq_w4a8_gemm_workspace_bytes(w.M, w.N, w.K)
    ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
    A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]), workspace=ws)
    packed, gs = fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"])
    pd, gd = fq.fq_pack_weights(_gpu(dd["q"])), _gpu(dd["gscale"])
    need_d = fq.fq_w4a8_gemm_workspace_bytes(w.M, ND, NH)
    ws_d = torch.empty((need_d,), dtype=torch.uint8, device="cuda")
    H, C, hs = fq.fq_w4a8_gemm_swiglu_quant(A, s, packed, gs, d["w_tscale"], w.N, workspace=ws, workspace_prepared=True,
                                            next_workspace=ws_d)
    Y = fq.fq_w4a8_gemm(C, hs, pd, gd, 1.0, ND, workspace=ws_d, workspace_prepared=True)
    # the same chain through the separate quantiser
    H2 = fq.fq_w4a8_gemm_swiglu(A, s, packed, gs, d["w_tscale"], w.N, workspace=ws, workspace_prepared=True)
    ws_d2 = torch.empty((need_d,), dtype=torch.uint8, device="cuda")
    C2, hs2 = fq.fq_quantize_act(H2, workspace=ws_d2)
    Y2 = fq.fq_w4a8_gemm(C2, hs2, pd, gd, 1.0, ND, workspace=ws_d2, workspace_prepared=True)
    torch.cuda.synchronize()
    assert torch.equal(H.view(torch.int16), H2.view(torch.int16))
    assert torch.equal(C, C2) and torch.equal(hs, hs2)
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16))
    rows = np.arange(0, w.M, 37)
    C_or, s_or = oracle.quantize_act(bf16_bits_from_gpu(H)[rows])
    assert np.array_equal(hs.cpu().numpy()[rows], s_or)
    assert _same_codes(C.cpu().numpy()[rows], C_or)
    Yo, B = oracle.w4a8_gemm(C.cpu().numpy()[rows], hs.cpu().numpy()[rows], dd["q"], dd["gscale"], 1.0, want_bound=True)
    check_gemm(bf16_bits_from_gpu(Y)[rows], Yo, B, "down projection on the fused layer's codes")
