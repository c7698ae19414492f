// Per-token FP8 quantisation of activations (Sec. 2.1 eq. 2):  A = FP8(x / beta), beta per row.
//   beta = absmax / 448 in FP32 (1 for an all-zero row); quotient as IEEE FP32 division would give
//   it; conversion to OCP E4M3 round-to-nearest-even by the hardware converter, after clamping to
//   +-448 so that the result saturates instead of becoming NaN.
// The quotient.  A full IEEE division is about eleven instructions per element.  With r = 1 / beta
// (one IEEE division per row), q = x * r, the residual e = fma(-q, beta, x) (exact) and
// q' = fma(e, r, q), then the sign of x put on q' (beta > 0), the stored E4M3 code equals that of
// the IEEE quotient for every finite bf16 x with |x| <= absmax and every beta = absmax / 448 in
// [2^-60, 2^60]: checked exhaustively on the host (5.3e8 pairs; the few quotients that differ in
// their last bit all come from subnormal x and round to zero).  Rows with beta outside that range
// take the full division.
#include <type_traits>
#include "fq_common.h"
#include "fq_kernels.h"

#define FQ_Q_THREADS 256
#define FQ_Q_MAXCHUNK 8        // 16-byte chunks (8 bf16) a thread keeps in registers: K <= 16384

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

// Sum of the eight E4M3 values of two words of codes.
__device__ __forceinline__ float fq_sum8(fq_v2i o) {
    const fq_v2f a = __builtin_amdgcn_cvt_pk_f32_fp8(o[0], false), b = __builtin_amdgcn_cvt_pk_f32_fp8(o[0], true);
    const fq_v2f c = __builtin_amdgcn_cvt_pk_f32_fp8(o[1], false), d = __builtin_amdgcn_cvt_pk_f32_fp8(o[1], true);
    return ((a[0] + a[1]) + (b[0] + b[1])) + ((c[0] + c[1]) + (d[0] + d[1]));
}

// One workgroup per row.  The row is read once into registers when it fits (K <= 16384),
// otherwise it is read a second time for the conversion pass.
// ZP: also write, for every group of 128 codes of the row, the zero-point term the large-M GEMM
// kernels take from their workspace: -2^-6 * (sum of the group's E4M3 values) as two fp16 terms,
// laid out as that kernel reads it ([plane][group / 8][M rows][group % 8]; groups up to the next
// multiple of 16 are zero).  Needs K % 128 == 0 and the row in registers.
// KNOWN: the row's largest magnitude is not searched for but taken from a_scale[m], where the kernel that
// produced X left it (the fused gate/up epilogue); the scale replaces it there.
template <bool ZP, bool KNOWN = false>
__global__ __launch_bounds__(FQ_Q_THREADS) void fq_quantize_kernel(const uint16_t* __restrict__ X,
                                                                   uint8_t* __restrict__ A,
                                                                   float* __restrict__ a_scale, int K,
                                                                   uint16_t* __restrict__ planes, int M) {
    __shared__ float red[FQ_Q_THREADS / 64];
    __shared__ __attribute__((aligned(16))) uint16_t zrow[2][FQ_Q_THREADS * FQ_Q_MAXCHUNK / 16 + 16];   // [plane][group]
    const int m = blockIdx.x;
    const fq_v4i* x = reinterpret_cast<const fq_v4i*>(X + (size_t)m * K);
    fq_v2i* a = reinterpret_cast<fq_v2i*>(A + (size_t)m * K);
    if (ZP && M <= FQ_KSPLIT_MAX_M) {                     // the arrival counters behind the planes start at zero
        const int G = K >> 7, C2 = 2 * ((G + 15) >> 4);
        unsigned* counters = reinterpret_cast<unsigned*>(planes + (size_t)2 * C2 * M * 8);
        for (int i = blockIdx.x * FQ_Q_THREADS + threadIdx.x; i < FQ_KSPLIT_COUNTERS; i += gridDim.x * FQ_Q_THREADS)
            counters[i] = 0u;
    }
    const int nchunk = K >> 3;
    const bool in_regs = nchunk <= FQ_Q_THREADS * FQ_Q_MAXCHUNK;
    fq_v4i keep[FQ_Q_MAXCHUNK];
    float amax = 0.f;
    if (in_regs) {
#pragma unroll
        for (int i = 0; i < FQ_Q_MAXCHUNK; ++i) {
            int c = threadIdx.x + i * FQ_Q_THREADS;
            keep[i] = (fq_v4i){0, 0, 0, 0};
            if (c < nchunk) {
                keep[i] = x[c];
                if (!KNOWN) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        unsigned w = (unsigned)keep[i][j];
                        amax = fmaxf(amax, fmaxf(fabsf(fq_bf16_lo(w)), fabsf(fq_bf16_hi(w))));
                    }
                }
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
    if (KNOWN) {                                          // (read by one thread before anyone overwrites it below)
        if (threadIdx.x == 0) red[0] = a_scale[m];
        __syncthreads();
        amax = red[0];
    } else {
        amax = fq_block_max(amax, red);
    }
    const float s = (amax == 0.f) ? 1.0f : amax / 448.0f;
    if (threadIdx.x == 0) a_scale[m] = s;
    const float rcp = 1.0f / s;
    // One choice of quotient per row (s is the same in every thread of the workgroup): the range the
    // short quotient was checked on, else the full division; straight-line code either way.
    auto convert = [&](auto fast_tag) __attribute__((always_inline)) {
    constexpr bool FAST = decltype(fast_tag)::value;
    if (in_regs) {
#pragma unroll
        for (int i = 0; i < FQ_Q_MAXCHUNK; ++i) {
            int c = threadIdx.x + i * FQ_Q_THREADS;
            if (c < nchunk) {
                const fq_v2i o = fq_quant8<FAST>(keep[i], s, rcp);
                a[c] = o;
                if (ZP) {
                    // a group is 16 consecutive chunks = 16 consecutive lanes (nchunk is a multiple of 16,
                    // so a group's lanes are all here or all absent)
                    float z = fq_sum8(o);
                    z += __shfl_xor(z, 1, 64);
                    z += __shfl_xor(z, 2, 64);
                    z += __shfl_xor(z, 4, 64);
                    z += __shfl_xor(z, 8, 64);
                    if ((threadIdx.x & 15) == 0) {
                        z *= -0.015625f;
                        const _Float16 hi = (_Float16)z;                  // round to nearest even
                        const _Float16 lo = (_Float16)(z - (float)hi);    // the difference is exact in FP32
                        zrow[0][c >> 4] = __builtin_bit_cast(uint16_t, hi);
                        zrow[1][c >> 4] = __builtin_bit_cast(uint16_t, lo);
                    }
                }
            }
        }
        if (ZP) {
            // padding groups are zero; then one 16-byte store per (plane, 8 groups) of this row
            const int G = K >> 7, C2 = 2 * ((G + 15) >> 4);
            for (int g = G + threadIdx.x; g < 8 * C2; g += FQ_Q_THREADS) zrow[0][g] = zrow[1][g] = 0;
            __syncthreads();
            for (int t = threadIdx.x; t < 2 * C2; t += FQ_Q_THREADS) {
                const int plane = t / C2, unit = t - plane * C2;
                const fq_v4i v = *reinterpret_cast<const fq_v4i*>(&zrow[plane][8 * unit]);
                *reinterpret_cast<fq_v4i*>(planes + (((size_t)plane * C2 + unit) * M + m) * 8) = v;
            }
        }
    } else {
        for (int c = threadIdx.x; c < nchunk; c += FQ_Q_THREADS) a[c] = fq_quant8<FAST>(x[c], s, rcp);
    }
    };
    if (__builtin_amdgcn_readfirstlane((int)fq_scale_is_fast(s))) convert(std::true_type());
    else convert(std::false_type());
}

void fq_launch_quantize(const uint16_t* X, uint8_t* A, float* a_scale, int M, int K, hipStream_t stream) {
    hipLaunchKernelGGL(fq_quantize_kernel<false>, dim3((unsigned)M), dim3(FQ_Q_THREADS), 0, stream, X, A, a_scale, K,
                       static_cast<uint16_t*>(nullptr), M);
}

bool fq_quantize_can_write_zero_point(int K) {
    return (K % FQ_GROUP) == 0 && (K >> 3) <= FQ_Q_THREADS * FQ_Q_MAXCHUNK;
}

void fq_launch_quantize_known(const uint16_t* X, uint8_t* A, float* a_scale, int M, int K, void* workspace,
                              hipStream_t stream) {
    if (workspace)
        hipLaunchKernelGGL((fq_quantize_kernel<true, true>), dim3((unsigned)M), dim3(FQ_Q_THREADS), 0, stream, X, A, a_scale,
                           K, static_cast<uint16_t*>(workspace), M);
    else
        hipLaunchKernelGGL((fq_quantize_kernel<false, true>), dim3((unsigned)M), dim3(FQ_Q_THREADS), 0, stream, X, A, a_scale,
                           K, static_cast<uint16_t*>(nullptr), M);
}

__global__ void fq_fill_zero_kernel(unsigned* __restrict__ p, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0u;
}

void fq_launch_fill_zero(unsigned* p, int n, hipStream_t stream) {
    hipLaunchKernelGGL(fq_fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n);
}

void fq_launch_quantize_zp(const uint16_t* X, uint8_t* A, float* a_scale, int M, int K, void* workspace,
                           hipStream_t stream) {
    hipLaunchKernelGGL(fq_quantize_kernel<true>, dim3((unsigned)M), dim3(FQ_Q_THREADS), 0, stream, X, A, a_scale, K,
                       static_cast<uint16_t*>(workspace), M);
}
