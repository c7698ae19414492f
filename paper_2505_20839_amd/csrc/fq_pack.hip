// Offline weight packing and its inverse (Sec. 3.1: INT4 weights, groups of 128 along K).
// The byte order is described in fq_common.h.
#include "fq_common.h"
#include "fq_kernels.h"

// One thread per packed byte: gathers the two codes that share it.
__global__ __launch_bounds__(256) void fq_pack_kernel(const int8_t* __restrict__ q, uint8_t* __restrict__ wp,
                                                      int N, int K, size_t total) {
    size_t idx = (size_t)blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    const int G = K / FQ_GROUP;
    size_t blk = idx >> 11;
    int in = (int)(idx & 2047u);
    int nt = (int)(blk / (size_t)G), g = (int)(blk % (size_t)G);
    int h = in >> 10, lane = (in >> 4) & 63, ij = in & 15;
    int kh = lane >> 5, n = nt * 32 + (lane & 31);
    int k_lo = g * FQ_GROUP + 64 * h + 32 * kh + ij;
    int k_hi = k_lo + 16;
    unsigned lo = 0, hi = 0;
    if (n < N) {
        lo = fq_code_from_q(q[(size_t)n * K + k_lo]);
        hi = fq_code_from_q(q[(size_t)n * K + k_hi]);
    }
    wp[idx] = (uint8_t)(lo | (hi << 4));
}

// One thread per weight.
__global__ __launch_bounds__(256) void fq_unpack_kernel(const uint8_t* __restrict__ wp, int8_t* __restrict__ q,
                                                        int N, int K, size_t total) {
    size_t idx = (size_t)blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    int n = (int)(idx / (size_t)K), k = (int)(idx % (size_t)K);
    int hi;
    size_t off = fq_weight_byte(n, k, K / FQ_GROUP, &hi);
    unsigned byte = wp[off];
    q[idx] = (int8_t)fq_q_from_code(hi ? (byte >> 4) : (byte & 0xFu));
}

void fq_launch_pack(const int8_t* q, uint8_t* wp, int N, int K, hipStream_t stream) {
    size_t total = (size_t)((N + 31) / 32) * 32u * (size_t)K / 2u;
    unsigned blocks = (unsigned)((total + 255u) / 256u);
    hipLaunchKernelGGL(fq_pack_kernel, dim3(blocks), dim3(256), 0, stream, q, wp, N, K, total);
}

void fq_launch_unpack(const uint8_t* wp, int8_t* q, int N, int K, hipStream_t stream) {
    size_t total = (size_t)N * (size_t)K;
    unsigned blocks = (unsigned)((total + 255u) / 256u);
    hipLaunchKernelGGL(fq_unpack_kernel, dim3(blocks), dim3(256), 0, stream, wp, q, N, K, total);
}
