// Per-token FP8 quantisation of activations (Sec. 2.1 eq. 2):  A = FP8(x / beta), beta per row.
//   beta = absmax / 448 in FP32 (1 for an all-zero row); quotient in IEEE FP32 division;
//   conversion to OCP E4M3 round-to-nearest-even by the hardware converter, after clamping to
//   +-448 so that the result saturates instead of becoming NaN.
#include "fq_common.h"
#include "fq_kernels.h"

#define FQ_Q_THREADS 256
#define FQ_Q_MAXCHUNK 8        // 16-byte chunks (8 bf16) a thread keeps in registers: K <= 16384

__device__ __forceinline__ float fq_bf16_hi(unsigned w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ float fq_bf16_lo(unsigned w) { return __uint_as_float(w << 16); }

__device__ __forceinline__ float fq_block_max(float v, float* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < FQ_Q_THREADS / 64; ++i) r = fmaxf(r, red[i]);
    return r;
}

__device__ __forceinline__ unsigned fq_quant4(float a, float b, float c, float d, float s) {
    a = fminf(fmaxf(a / s, -448.f), 448.f);
    b = fminf(fmaxf(b / s, -448.f), 448.f);
    c = fminf(fmaxf(c / s, -448.f), 448.f);
    d = fminf(fmaxf(d / s, -448.f), 448.f);
    int r = 0;
    r = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, r, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, r, true);
    return (unsigned)r;
}

// One workgroup per row.  The row is read once into registers when it fits (K <= 16384),
// otherwise it is read a second time for the conversion pass.
__global__ __launch_bounds__(FQ_Q_THREADS) void fq_quantize_kernel(const uint16_t* __restrict__ X,
                                                                   uint8_t* __restrict__ A,
                                                                   float* __restrict__ a_scale, int K) {
    __shared__ float red[FQ_Q_THREADS / 64];
    const int m = blockIdx.x;
    const fq_v4i* x = reinterpret_cast<const fq_v4i*>(X + (size_t)m * K);
    fq_v2i* a = reinterpret_cast<fq_v2i*>(A + (size_t)m * K);
    const int nchunk = K >> 3;
    const bool in_regs = nchunk <= FQ_Q_THREADS * FQ_Q_MAXCHUNK;
    fq_v4i keep[FQ_Q_MAXCHUNK];
    float amax = 0.f;
    if (in_regs) {
#pragma unroll
        for (int i = 0; i < FQ_Q_MAXCHUNK; ++i) {
            int c = threadIdx.x + i * FQ_Q_THREADS;
            keep[i] = (fq_v4i){0, 0, 0, 0};
            if (c < nchunk) keep[i] = x[c];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                unsigned w = (unsigned)keep[i][j];
                amax = fmaxf(amax, fmaxf(fabsf(fq_bf16_lo(w)), fabsf(fq_bf16_hi(w))));
            }
        }
    } else {
        for (int c = threadIdx.x; c < nchunk; c += FQ_Q_THREADS) {
            fq_v4i v = x[c];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                unsigned w = (unsigned)v[j];
                amax = fmaxf(amax, fmaxf(fabsf(fq_bf16_lo(w)), fabsf(fq_bf16_hi(w))));
            }
        }
    }
    amax = fq_block_max(amax, red);
    const float s = (amax == 0.f) ? 1.0f : amax / 448.0f;
    if (threadIdx.x == 0) a_scale[m] = s;
    if (in_regs) {
#pragma unroll
        for (int i = 0; i < FQ_Q_MAXCHUNK; ++i) {
            int c = threadIdx.x + i * FQ_Q_THREADS;
            if (c < nchunk) {
                fq_v4i v = keep[i];
                fq_v2i o;
                o[0] = (int)fq_quant4(fq_bf16_lo(v[0]), fq_bf16_hi(v[0]), fq_bf16_lo(v[1]), fq_bf16_hi(v[1]), s);
                o[1] = (int)fq_quant4(fq_bf16_lo(v[2]), fq_bf16_hi(v[2]), fq_bf16_lo(v[3]), fq_bf16_hi(v[3]), s);
                a[c] = o;
            }
        }
    } else {
        for (int c = threadIdx.x; c < nchunk; c += FQ_Q_THREADS) {
            fq_v4i v = x[c];
            fq_v2i o;
            o[0] = (int)fq_quant4(fq_bf16_lo(v[0]), fq_bf16_hi(v[0]), fq_bf16_lo(v[1]), fq_bf16_hi(v[1]), s);
            o[1] = (int)fq_quant4(fq_bf16_lo(v[2]), fq_bf16_hi(v[2]), fq_bf16_lo(v[3]), fq_bf16_hi(v[3]), s);
            a[c] = o;
        }
    }
}

void fq_launch_quantize(const uint16_t* X, uint8_t* A, float* a_scale, int M, int K, hipStream_t stream) {
    hipLaunchKernelGGL(fq_quantize_kernel, dim3((unsigned)M), dim3(FQ_Q_THREADS), 0, stream, X, A, a_scale, K);
}
