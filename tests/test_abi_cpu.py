"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments before touching the GPU (no kernel is launched here)."""
import ctypes
import os
import re

import pytest

from paper_2505_20839_amd import binding, build

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "fireq.h")


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(fq_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = _declared_functions()
    assert names == sorted(["fq_w4a8_gemm", "fq_w4a8_gemm_ws", "fq_w4a8_gemm_swiglu_ws", "fq_w4a8_gemm_swiglu_quant_ws", "fq_w4a8_gemm_add_ws", "fq_w4a8_gemm_workspace_bytes", "fq_quantize_act", "fq_quantize_act_ws", "fq_packed_weight_bytes", "fq_pack_weights",
                            "fq_unpack_weights", "fq_layout_version", "fq_status_string",
                            "fq_cas_scales", "fq_pts_exponent", "fq_quantize_weights",
                            "fq_w4a8_linear_ws", "fq_w4a8_linear_workspace_bytes",
                            "fq_w4a8_gemm_plan", "fq_test_force_kernel",
                            "fq_w4a8_gemm_static", "fq_w4a8_gemm_static_max_workspace",
                            "fq_diag_stream_read", "fq_diag_stream_read_sink_bytes", "fq_w4a8_gemm_lut",
                            "fq_kv4_packed_bytes", "fq_kv4_pack", "fq_kv4_unpack", "fq_kv4_scores", "fq_kv4_output"])
    for name in names:
        assert hasattr(L, name), name
    assert os.path.samefile(L._name, build.LIB_PATH)


def test_sizes_version_and_status_strings():
    assert binding.fq_packed_weight_bytes(256, 512) == 256 * 512 // 2
    assert binding.fq_packed_weight_bytes(33, 128) == 64 * 128 // 2      # rows padded to 32
    assert binding.fq_packed_weight_bytes(14336, 4096) == 14336 * 4096 // 2
    assert binding.fq_packed_weight_bytes(16, 100) == 0                  # K not a multiple of 128
    assert binding.fq_packed_weight_bytes(0, 128) == 0
    assert binding.fq_layout_version() >= 1
    seen = {binding.status_string(s) for s in (0, -1, -2, -3, -4, -5)}
    assert len(seen) == 6 and binding.status_string(0) == "ok"
    # workspace: none for the small-M kernels, two fp16 planes of [M][16 * ceil(K / 2048)] for the rest
    assert binding.fq_w4a8_gemm_workspace_bytes(64, 256, 4096) == 0
    # zero-point planes, arrival counters, and 4 K slices x 4 tiles of 128 x 64 FP32 partial sums (256 compute units assumed without a GPU)
    assert binding.fq_w4a8_gemm_workspace_bytes(65, 256, 4096) == 2 * 4 * 65 * 16 + 4096 + 4 * 4 * 32768
    assert binding.fq_w4a8_gemm_workspace_bytes(513, 256, 4096) == 2 * 4 * 513 * 16
    assert binding.fq_w4a8_gemm_workspace_bytes(2048, 4096, 11008) == 2 * 12 * 2048 * 16
    assert binding.fq_w4a8_gemm_workspace_bytes(128, 256, 100) == 0      # invalid shape
    assert binding.status_string(-99) == "unknown status"


def test_bad_arguments_are_rejected_without_a_launch():
    L = binding.lib()
    p = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1008)
    null = ctypes.c_void_p(0)
    f1 = ctypes.c_float(1.0)
    # shape errors
    assert L.fq_w4a8_gemm(p, p, p, p, f1, p, 4, 32, 100, null) == -2
    assert L.fq_w4a8_gemm(p, p, p, p, f1, p, -1, 32, 128, null) == -2
    assert L.fq_w4a8_gemm(p, p, p, p, f1, p, 4, 0, 128, null) == -2
    assert L.fq_w4a8_gemm(p, p, p, p, f1, p, 4, 32, 0, null) == -2
    # operands of 4 GiB or more are not addressable by the kernels
    assert L.fq_w4a8_gemm(p, p, p, p, f1, p, 1 << 20, 32, 1 << 12, null) == -2      # A: 4 GiB
    assert L.fq_w4a8_gemm(p, p, p, p, f1, p, 4, 1 << 20, 1 << 13, null) == -2       # packed W: 4 GiB
    # M == 0 is a successful no-op even with NULL pointers
    assert L.fq_w4a8_gemm(null, null, null, null, f1, null, 0, 32, 128, null) == 0
    # NULL and misaligned pointers
    assert L.fq_w4a8_gemm(null, p, p, p, f1, p, 4, 32, 128, null) == -1
    assert L.fq_w4a8_gemm(p, p, p, p, f1, null, 4, 32, 128, null) == -1
    assert L.fq_w4a8_gemm(odd, p, p, p, f1, p, 4, 32, 128, null) == -3
    assert L.fq_w4a8_gemm(p, p, odd, p, f1, p, 4, 32, 128, null) == -3
    # the explicit-workspace variant: same checks, plus the workspace itself
    ws = (p, ctypes.c_size_t(1 << 30), 0)
    assert L.fq_w4a8_gemm_ws(p, p, p, p, f1, p, 4, 32, 100, *ws, null) == -2
    assert L.fq_w4a8_gemm_ws(null, null, null, null, f1, null, 0, 32, 128, null, ctypes.c_size_t(0), 0, null) == 0
    assert L.fq_w4a8_gemm_ws(null, p, p, p, f1, p, 128, 32, 128, *ws, null) == -1
    assert L.fq_w4a8_gemm_ws(p, p, p, odd, f1, p, 128, 32, 128, *ws, null) == -3
    assert L.fq_w4a8_gemm_ws(p, p, p, p, f1, p, 128, 32, 128, null, ctypes.c_size_t(0), 0, null) == -5
    assert L.fq_w4a8_gemm_ws(p, p, p, p, f1, p, 128, 32, 128, p, ctypes.c_size_t(100), 1, null) == -5
    assert L.fq_w4a8_gemm_ws(p, p, p, p, f1, p, 128, 32, 128, odd, ctypes.c_size_t(1 << 30), 0, null) == -3
    assert L.fq_w4a8_gemm_swiglu_ws(p, p, p, p, f1, p, 128, 33, 128, *ws, null) == -2          # N odd
    assert L.fq_w4a8_gemm_swiglu_ws(p, p, p, p, f1, null, 128, 32, 128, *ws, null) == -1
    assert L.fq_w4a8_gemm_swiglu_ws(p, p, p, p, f1, p, 128, 32, 128, null, ctypes.c_size_t(0), 0, null) == -5
    # the residual variant: the residual is required, aligned, and either the output itself or disjoint
    p2 = ctypes.c_void_p(p.value + 16)
    far = ctypes.c_void_p(p.value + (1 << 20))
    assert L.fq_w4a8_gemm_add_ws(p, p, p, p, f1, null, far, 128, 32, 128, *ws, null) == -1
    assert L.fq_w4a8_gemm_add_ws(p, p, p, p, f1, odd, far, 128, 32, 128, *ws, null) == -3
    assert L.fq_w4a8_gemm_add_ws(p, p, p, p, f1, p2, p, 128, 32, 128, *ws, null) == -2          # shifted overlap
    assert L.fq_w4a8_gemm_add_ws(p, p, p, p, f1, p, p2, 128, 32, 128, *ws, null) == -2
    assert L.fq_w4a8_gemm_add_ws(p, p, p, p, f1, p, p, 128, 32, 100, *ws, null) == -2           # K % 128
    assert L.fq_w4a8_gemm_add_ws(p, p, p, p, f1, p, p, 128, 32, 128, null, ctypes.c_size_t(0), 0, null) == -5
    assert L.fq_w4a8_gemm_add_ws(null, null, null, null, f1, null, null, 0, 32, 128, null, ctypes.c_size_t(0), 0, null) == 0
    assert L.fq_quantize_act_ws(p, p, p, 4, 100, p, ctypes.c_size_t(1 << 30), null) == -2      # K % 128
    assert L.fq_quantize_act_ws(p, p, p, 0, 128, null, ctypes.c_size_t(0), null) == 0
    assert L.fq_quantize_act_ws(null, p, p, 4, 128, p, ctypes.c_size_t(1 << 30), null) == -1
    assert L.fq_quantize_act_ws(p, p, p, 128, 128, null, ctypes.c_size_t(0), null) == -5
    assert L.fq_quantize_act_ws(p, p, p, 128, 128, p, ctypes.c_size_t(8), null) == -5
    assert L.fq_quantize_act_ws(p, p, p, 128, 128, odd, ctypes.c_size_t(1 << 30), null) == -3
    assert L.fq_quantize_act(p, p, p, 4, 12, null) == -2
    assert L.fq_quantize_act(p, p, p, 0, 128, null) == 0
    assert L.fq_quantize_act(null, p, p, 4, 128, null) == -1
    assert L.fq_quantize_act(p, odd, p, 4, 128, null) == -3
    # the whole layer from bf16 activations: no workspace for the one-kernel case, else codes + scales + GEMM scratch
    assert L.fq_w4a8_linear_workspace_bytes(6, 256, 4096) == 0
    assert L.fq_w4a8_linear_workspace_bytes(7, 256, 4096) == 7 * 4096 + 32
    assert L.fq_w4a8_linear_workspace_bytes(16, 256, 8192) == 16 * 8192 + 64
    assert L.fq_w4a8_linear_workspace_bytes(17, 256, 512) == 17 * 512 + 80
    assert L.fq_w4a8_linear_workspace_bytes(100, 256, 512) == 100 * 512 + 400 + L.fq_w4a8_gemm_workspace_bytes(100, 256, 512)
    lin = (ctypes.c_size_t(1 << 30), null)
    assert L.fq_w4a8_linear_ws(p, p, p, f1, p, 4, 32, 100, p, *lin) == -2
    assert L.fq_w4a8_linear_ws(null, p, p, f1, p, 4, 32, 128, p, *lin) == -1
    assert L.fq_w4a8_linear_ws(odd, p, p, f1, p, 4, 32, 128, p, *lin) == -3
    assert L.fq_w4a8_linear_ws(p, p, p, f1, p, 100, 32, 128, null, ctypes.c_size_t(0), null) == -5
    assert L.fq_w4a8_linear_ws(p, p, p, f1, p, 100, 32, 128, p, ctypes.c_size_t(64), null) == -5
    assert L.fq_w4a8_linear_ws(null, null, null, f1, null, 0, 32, 128, null, ctypes.c_size_t(0), null) == 0
    # offline weight quantiser
    assert L.fq_cas_scales(p, f1, p, 0, 128, null) == -2
    assert L.fq_cas_scales(p, ctypes.c_float(0.0), p, 4, 128, null) == -2
    assert L.fq_cas_scales(null, f1, p, 4, 128, null) == -1
    assert L.fq_pts_exponent(p, null, p, 4, 100, null) == -2
    assert L.fq_pts_exponent(p, null, null, 4, 128, null) == -1
    assert L.fq_pts_exponent(p, null, odd, 4, 128, null) == -3
    assert L.fq_quantize_weights(p, null, 0, 0, p, p, 4, 100, null) == -2
    assert L.fq_quantize_weights(p, null, 127, 0, p, p, 4, 128, null) == -2
    assert L.fq_quantize_weights(p, null, -1, 0, p, p, 4, 128, null) == -2
    assert L.fq_quantize_weights(p, null, 0, 0, null, p, 4, 128, null) == -1
    assert L.fq_quantize_weights(p, null, 0, 0, odd, p, 4, 128, null) == -3
    assert L.fq_quantize_weights(null, null, 0, 0, null, null, 0, 128, null) == 0
    assert L.fq_pack_weights(p, p, 8, 100, null) == -2
    assert L.fq_pack_weights(null, p, 8, 128, null) == -1
    assert L.fq_pack_weights(p, odd, 8, 128, null) == -3
    assert L.fq_pack_weights(null, null, 0, 128, null) == 0
    assert L.fq_unpack_weights(p, null, 8, 128, null) == -1
    assert L.fq_unpack_weights(p, p, 8, 64, null) == -2
