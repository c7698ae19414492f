// Host-side launchers implemented by the kernel translation units (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

// ---- per-device host state (fq_device.hip) ----
// Compute units of the current device, read once per device (256 if the runtime cannot say).
int fq_device_cus();
// One-time set-up that has to happen on every device the library is used on (kernel attributes): `f`
// has run on the current device when fq_once_per_device returns.  Threads that race on a device's
// first call may both run `f`, so it must be idempotent (hipFuncSetAttribute is).
#define FQ_MAX_DEVICES 64
struct fq_device_once {
    std::atomic<unsigned char> done[FQ_MAX_DEVICES];
};
int fq_current_device_slot();                             // current device id, 0 if out of range or unknown
template <class F>
inline void fq_once_per_device(fq_device_once& st, F&& f) {
    const int d = fq_current_device_slot();
    if (st.done[d].load(std::memory_order_acquire)) return;
    f();
    st.done[d].store(1, std::memory_order_release);
}

// Each launcher validates nothing: arguments were checked by the C entry point.  They enqueue on
// `stream` and return; the caller reads hipGetLastError().
void fq_launch_pack(const int8_t* q, uint8_t* wp, int N, int K, hipStream_t stream);
void fq_launch_unpack(const uint8_t* wp, int8_t* q, int N, int K, hipStream_t stream);
void fq_launch_quantize(const uint16_t* X, uint8_t* A, float* a_scale, int M, int K, hipStream_t stream);
// The same, also filling the large-M GEMM's workspace (fq_gemm_large_workspace_bytes(M, K)) with the
// zero-point terms of A; only for shapes fq_quantize_can_write_zero_point(K) accepts.
bool fq_quantize_can_write_zero_point(int K);
// fq_launch_quantize_known: the same quantiser for rows whose largest magnitude is already known: a_scale[m] holds
// it on entry (the bits of the number as FP32, as the fused gate/up epilogue leaves it) and the scale on return;
// workspace may be null (no zero-point terms written).
void fq_launch_quantize_known(const uint16_t* X, uint8_t* A, float* a_scale, int M, int K, void* workspace,
                              hipStream_t stream);
void fq_launch_fill_zero(unsigned* p, int n, hipStream_t stream);
void fq_launch_quantize_zp(const uint16_t* X, uint8_t* A, float* a_scale, int M, int K, void* workspace,
                           hipStream_t stream);

// GEMM kernels.  `which` selects the kernel: see fq_api.hip.
// `swiglu` (all three launchers): channels 2j / 2j+1 are the gate / up rows of a feed-forward block and
// the output is H[M, N/2] = bf16(SiLU(gate) * up) instead of Y[M, N] (N even).
// `lut` (the simple and the large-M launcher): the paper's table mode, weights rounded to E4M3(q * sigma)
// before the products (Sec. 3.1.1 step 1); workspace and `prepared` are ignored then.
// `R` (all three; NULL = none; not together with swiglu): residual [M, N] in bf16 added to the result
// before its one rounding; may be the output array itself.
void fq_launch_gemm_simple(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                           float tscale, uint16_t* Y, int M, int N, int K, bool swiglu, const uint16_t* R,
                           hipStream_t stream, bool lut = false);
// The large-M kernel needs fq_gemm_large_workspace_bytes(M, K) bytes of device scratch (16-byte aligned)
// holding the zero-point term of every (row, group) of A: fq_launch_zero_point writes it, and
// fq_launch_gemm_large calls that first unless `prepared` says the workspace already holds it.
// For M <= FQ_KSPLIT_MAX_M the planes are followed by FQ_KSPLIT_COUNTERS arrival counters (32-bit), which whatever
// writes the planes also sets to zero; the K-split kernel's partial tiles come after those.
#define FQ_KSPLIT_COUNTERS 1024
#define FQ_KSPLIT_MAX_M 512
size_t fq_gemm_plane_bytes(int M, int K);
size_t fq_gemm_large_workspace_bytes(int M, int K);
// How the large-M kernel cuts an M x N problem on `cus` compute units: out[0] whole tiles (256 rows x
// 128 channels) stored with whole-row vector stores, out[1] whole tiles stored element by element (rows
// past M, channels past N, or N not a multiple of 8), out[2] / out[3] the same for the 128-row halves of
// the tail round.
void fq_gemm_large_plan(int M, int N, int cus, int out[4]);
void fq_launch_zero_point(const uint8_t* A, void* workspace, int M, int K, hipStream_t stream);
void fq_launch_gemm_large(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                          float tscale, uint16_t* Y, int M, int N, int K, void* workspace, bool prepared,
                          bool swiglu, const uint16_t* R, hipStream_t stream, bool lut = false,
                          unsigned* rowmax = nullptr);   // (fused gate/up only: row maxima of |H|, see the kernel)
// M <= 64 only; returns false (nothing enqueued) for a shape it does not serve.
bool fq_launch_gemm_small(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                          float tscale, uint16_t* Y, int M, int N, int K, bool swiglu, const uint16_t* R,
                           hipStream_t stream);
// M <= 16: quantiser and GEMM in one kernel, from bf16 activations X [M,K]; a_scale_out (may be NULL) receives
// the row scales.  Serves M <= 6 with K <= 4096 (fq_linear_small_serves); returns false (nothing enqueued) otherwise.
bool fq_linear_small_serves(int M, int K);
bool fq_launch_linear_small(const uint16_t* X, float* a_scale_out, const uint8_t* wp, const uint8_t* gs, float tscale,
                            uint16_t* Y, int M, int N, int K, hipStream_t stream);

// Offline weight quantisation (fq_wquant.hip).  W is [N,K] bf16; lambda (may be NULL) is [K] FP32.
void fq_launch_cas_scales(const uint16_t* W, float target, float* lambda, int N, int K, hipStream_t stream);
// n_out: 64 bytes of device memory; int 0 receives n, ints 8..12 are scratch for the statistics.
void fq_launch_pts_exponent(const uint16_t* W, const float* lambda, int* n_out, int N, int K, hipStream_t stream);
void fq_launch_quantize_weights(const uint16_t* W, const float* lambda, int n_pts, bool sigma_rne, int8_t* q,
                                uint8_t* gs, int N, int K, hipStream_t stream);


// Measurement aid (fq_diag.hip): reads `bytes` (a multiple of 16) from src and writes one word per workgroup
// to sink (fq_stream_read_blocks() words).
unsigned fq_stream_read_blocks();
void fq_launch_stream_read(const void* src, size_t bytes, unsigned* sink, hipStream_t stream);

// Attention operands with an INT4 key/value cache (fq_kv4.hip).  codes: [H][T][128] int8; packed: per head
// fq_kv4_key_bytes(T) / fq_kv4_value_bytes(T) bytes; scales: [H][T] E4M3 codes.
size_t fq_kv4_key_bytes(int T);
size_t fq_kv4_value_bytes(int T);
void fq_launch_kv4_pack(const int8_t* codes, uint8_t* packed, int H, int T, bool values, hipStream_t stream);
void fq_launch_kv4_unpack(const uint8_t* packed, int8_t* codes, int H, int T, bool values, hipStream_t stream);
void fq_launch_kv4_scores(const uint8_t* Q, const float* q_scale, const uint8_t* kp, const uint8_t* ks, float out_scale,
                          uint16_t* S, int H, int R, int T, hipStream_t stream);
void fq_launch_kv4_output(const uint8_t* P, const float* p_scale, const uint8_t* vp, const uint8_t* vs, uint16_t* O,
                          int H, int R, int T, int ldp, hipStream_t stream);

// K-split kernel (fq_gemm_ksplit.hip): 8-wave workgroups that split K inside the workgroup, for problems with
// too few tiles for the large-M kernel.  fq_gemm_ksplit_choice: 0 = not used for this shape, 1 = 256 x 128 tiles
// with K halved, 2 = 128 x 64 tiles with K quartered.  Workspace and `prepared` as for fq_launch_gemm_large; no
// fused gate/up epilogue.
int fq_gemm_ksplit_choice(int M, int N, int K, int cus);
// K slices per tile (workgroups that share a tile and add their partial tiles through the workspace) and the
// bytes of partial tiles, which follow the arrival counters in the workspace; 1 and 0 when there are none.
int fq_gemm_ksplit_slices(int choice, int M, int N, int K, int cus);
size_t fq_gemm_ksplit_partial_bytes(int choice, int M, int N, int K, int cus);
// The same kernel on 64 x 64 tiles for the top of 16 < M <= 64, which has no workspace (zero point through the matrix cores).
#ifndef FQ_KSPLIT64_MIN_M
#define FQ_KSPLIT64_MIN_M 56
#endif
bool fq_gemm_ksplit64_serves(int M, int N, int K, int cus);
void fq_launch_gemm_ksplit64(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs, float tscale,
                             uint16_t* Y, int M, int N, int K, const uint16_t* R, hipStream_t stream);
void fq_launch_gemm_ksplit(int choice, const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                           float tscale, uint16_t* Y, int M, int N, int K, void* workspace, bool prepared,
                           const uint16_t* R, hipStream_t stream);
