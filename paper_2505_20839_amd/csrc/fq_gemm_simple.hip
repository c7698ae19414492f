// Plain W4A8-FP GEMM: one thread per output element, no matrix cores.  It reads the same packed
// weights as the tuned kernels and exists for shapes they do not cover and as an in-library
// cross-check (selected with FQ_FORCE_KERNEL=simple).  Computes, in FP32,
//   Y[m,n] = bf16( a_scale[m] * w_tscale * sum_g e4m3(gs[n,g]) * sum_{k in g} e4m3(A[m,k]) * q[n,k] )
// (Sec. 2.2 eq. 3 with the operands of Sec. 3.1 and the output factor of Def. 3.2).
// With `swiglu` a thread computes the two sums of channels 2j (gate) and 2j + 1 (up) and stores
// H[m,j] = bf16(SiLU(gate) * up) (the fused epilogue of Sec. 3.1.1 step 3), H being [M, N/2].
// With a residual R [M,N] (bf16; may be Y itself) the plain result is Y = bf16(sum + R), rounded once.
// With `lut` the weights enter as the paper's table entries E4M3(q * sigma) (Sec. 3.1.1 step 1: nearest
// even, saturating at +-448) and the sum runs over all of K without a separate group scale.
#include "fq_common.h"
#include "fq_kernels.h"

__device__ float fq_simple_dot(const uint8_t* __restrict__ A, const uint8_t* __restrict__ wp,
                               const uint8_t* __restrict__ gs, int m, int n, int K, int lut) {
    const int G = K / FQ_GROUP;
    float acc = 0.f;
    for (int g = 0; g < G; ++g) {
        float p = 0.f;
        if (lut) {
            const float sigma = fq_e4m3_to_float(gs[(size_t)n * G + g]);
            for (int kk = 0; kk < FQ_GROUP; ++kk) {
                int k = g * FQ_GROUP + kk, hi;
                size_t off = fq_weight_byte(n, k, G, &hi);
                unsigned byte = wp[off];
                int qv = fq_q_from_code(hi ? (byte >> 4) : (byte & 0xFu));
                const float e = fminf(fmaxf((float)qv * sigma, -448.f), 448.f);
                const unsigned code = (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(e, 0.f, 0, false) & 0xFFu;
                acc = fmaf(fq_e4m3_to_float(A[(size_t)m * K + k]), fq_e4m3_to_float(code), acc);
            }
            continue;
        }
        for (int kk = 0; kk < FQ_GROUP; ++kk) {
            int k = g * FQ_GROUP + kk, hi;
            size_t off = fq_weight_byte(n, k, G, &hi);
            unsigned byte = wp[off];
            int qv = fq_q_from_code(hi ? (byte >> 4) : (byte & 0xFu));
            p = fmaf(fq_e4m3_to_float(A[(size_t)m * K + k]), (float)qv, p);
        }
        acc = fmaf(fq_e4m3_to_float(gs[(size_t)n * G + g]), p, acc);
    }
    return acc;
}

__global__ __launch_bounds__(256) void fq_gemm_simple_kernel(const uint8_t* __restrict__ A,
                                                             const float* __restrict__ a_scale,
                                                             const uint8_t* __restrict__ wp,
                                                             const uint8_t* __restrict__ gs, float tscale,
                                                             uint16_t* Y, int M, int N, int K,
                                                             int swiglu, const uint16_t* R, int lut) {
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);   // output column
    const int m = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int NO = swiglu ? N / 2 : N;
    if (c >= NO || m >= M) return;
    const float outer = a_scale[m] * tscale;
    float v;
    if (swiglu) v = fq_silu_mul(outer * fq_simple_dot(A, wp, gs, m, 2 * c, K, lut), outer * fq_simple_dot(A, wp, gs, m, 2 * c + 1, K, lut));
    else if (R) v = fmaf(outer, fq_simple_dot(A, wp, gs, m, c, K, lut), __uint_as_float((unsigned)R[(size_t)m * N + c] << 16));
    else        v = outer * fq_simple_dot(A, wp, gs, m, c, K, lut);
    Y[(size_t)m * NO + c] = (uint16_t)fq_float_to_bf16(v);
}

void fq_launch_gemm_simple(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                           float tscale, uint16_t* Y, int M, int N, int K, bool swiglu, const uint16_t* R,
                           hipStream_t stream, bool lut) {
    const int NO = swiglu ? N / 2 : N;
    dim3 grid((unsigned)((NO + 63) / 64), (unsigned)((M + 3) / 4));
    hipLaunchKernelGGL(fq_gemm_simple_kernel, grid, dim3(256), 0, stream, A, a_scale, wp, gs, tscale, Y, M, N, K,
                       swiglu ? 1 : 0, R, lut ? 1 : 0);
}
