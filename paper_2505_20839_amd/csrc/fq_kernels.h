// Host-side launchers implemented by the kernel translation units (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Each launcher validates nothing: arguments were checked by the C entry point.  They enqueue on
// `stream` and return; the caller reads hipGetLastError().
void fq_launch_pack(const int8_t* q, uint8_t* wp, int N, int K, hipStream_t stream);
void fq_launch_unpack(const uint8_t* wp, int8_t* q, int N, int K, hipStream_t stream);
void fq_launch_quantize(const uint16_t* X, uint8_t* A, float* a_scale, int M, int K, hipStream_t stream);

// GEMM kernels.  `which` selects the kernel: see fq_api.hip.
void fq_launch_gemm_simple(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                           float tscale, uint16_t* Y, int M, int N, int K, hipStream_t stream);
// The large-M launcher keeps a grow-only device scratch buffer (3 * 2 * ceil(K / 2048) * M * 16 bytes) that
// all calls of the process share: calls on different streams that overlap would race on it.  It
// returns non-zero when that buffer cannot be allocated (nothing is enqueued then).
int fq_launch_gemm_large(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                         float tscale, uint16_t* Y, int M, int N, int K, hipStream_t stream);
void fq_launch_gemm_small(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                          float tscale, uint16_t* Y, int M, int N, int K, hipStream_t stream);
