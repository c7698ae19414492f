"""fq_w4a8_gemm_static -- the GEMM entry point that allocates nothing and takes no workspace (its
scratch is a fixed array inside the library) -- against fq_w4a8_gemm_ws on the same operands, bit for
bit, on two calls in a row, the second with a smaller input, and against the CPU oracle."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2505_20839_amd import workloads
from parity_util import bf16_bits_from_gpu, check_gemm, to_gpu_bf16

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _gpu(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_static_scratch_entry_point_matches_the_workspace_one():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    from paper_2505_20839_amd import binding as fq
    L = fq.lib()
    fq.fq_test_force_kernel(None)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # first a problem whose scratch is large (K = 11008: 12 units per plane), then a smaller one that
    # leaves most of the first call's contents in place behind its own
    for M, N, K, seed in [(700, 520, 11008, 3), (300, 256, 1024, 4), (16, 256, 512, 5)]:
        d = workloads.draw(M, N, K, seed=seed, outlier_frac=0.01)
        A, s = fq.fq_quantize_act(to_gpu_bf16(d["X_bf16"]))
        packed, gs = fq.fq_pack_weights(_gpu(d["q"])), _gpu(d["gscale"])
        Y_ws = fq.fq_w4a8_gemm(A, s, packed, gs, d["w_tscale"], N)           # fq_w4a8_gemm_ws on a torch workspace
        Y_st = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = L.fq_w4a8_gemm_static(A.data_ptr(), s.data_ptr(), packed.data_ptr(), gs.data_ptr(),
                                   ctypes.c_float(d["w_tscale"]), Y_st.data_ptr(), M, N, K, stream)
        assert rc == 0, fq.status_string(rc)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(Y_st.view(torch.int16), Y_ws.view(torch.int16)), (M, N, K)
        Y, B = oracle.w4a8_gemm(A.cpu().numpy(), s.cpu().numpy(), d["q"], d["gscale"], d["w_tscale"], want_bound=True)
        check_gemm(bf16_bits_from_gpu(Y_st), Y, B, "static scratch %dx%dx%d" % (M, N, K))
    # a problem that needs more than the built-in scratch is refused before anything is enqueued
    cap = L.fq_w4a8_gemm_static_max_workspace()
    M, N, K = 32768 + 256, 128, 16384
    assert fq.fq_w4a8_gemm_workspace_bytes(M, N, K) > cap
    p = ctypes.c_void_p(0x1000)                               # never dereferenced: the size check comes first
    assert L.fq_w4a8_gemm_static(p, p, p, p, ctypes.c_float(1.0), p, M, N, K, stream) == -5
    assert fq.fq_w4a8_gemm_workspace_bytes(32768, 128, 16384) == cap
