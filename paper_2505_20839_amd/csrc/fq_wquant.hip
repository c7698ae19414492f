// Offline weight quantisation: the step that produces the GEMM's weight operands from a bf16 matrix
// W [N,K] (output channel n, input channel k; Y = X W^T).
//
//   channel-wise absmean scaling (Sec. 3.1.2, Def. 3.1)   lambda[k] = target / mean_n |W[n,k]|
//   per-tensor scaling (Def. 3.2, App. C.1)                delta = 2^n, n the smallest non-negative integer
//       for which the cumulative underflow S(W * 2^n) has reached its final value, or an element lies in
//       7 * 2^(5-n) <= |w| < 7 * 2^(6-n)
//   group-wise INT4 with an FP8 scale (Sec. 2.1 eq. 1, Sec. 3.1; App. B Lemma B.1)
//       sigma = max_group |v| / 7,  sigma8 = E4M3(sigma),  q = clamp(round(v / sigma8), -8, 7)
//
// Everywhere the weight that is worked on is v = fp32(W[n,k] * lambda[k]) (lambda may be absent),
// and the quantiser multiplies it by 2^n (exact).
#include "fq_common.h"
#include "fq_kernels.h"

namespace {

__device__ __forceinline__ float fqw_bf16(unsigned short b) { return __uint_as_float((unsigned)b << 16); }

// floor(log2(v / 7)) of a positive finite FP32 number given by its bits: v = 1.m * 2^E lies at or
// above 7 * 2^(E-2) = 1.75 * 2^E exactly when its fraction is at least 0.75.
__device__ __forceinline__ int fqw_log2_over_7(unsigned bits) {
    int e = (int)(bits >> 23);
    unsigned frac = bits & 0x7FFFFFu;
    if (e == 0) {                                         // subnormal: normalise by hand
        const int p = 31 - __builtin_clz(frac);           // frac != 0 for a positive number
        e = p - 22;                                       // value = frac * 2^-149 = 1.x * 2^(p-149); biased: p - 149 + 127
        frac = (frac << (23 - p)) & 0x7FFFFFu;
    }
    const int E = e - 127;
    return frac >= 0x600000u ? E - 2 : E - 3;
}

}  // namespace

// ---- channel-wise absmean scaling ------------------------------------------------------------------
// One workgroup per 32 input channels.  16 lanes cover the 32 channels of a row (a dword = two channels
// each), so a wave reads 4 rows per instruction and the 4 waves 16; FQW_CAS_UNROLL such loads are in flight
// per lane.  FP64 sums, combined in a fixed order: the result does not depend on timing.
#define FQW_CAS_UNROLL 8
__global__ __launch_bounds__(256) void fq_cas_scales_kernel(const uint16_t* __restrict__ W, float target,
                                                            float* __restrict__ lambda, int N, int K) {
    __shared__ double part[16][32];
    const int sub = threadIdx.x >> 4;                     // which of the 16 rows of a pass
    const int k = blockIdx.x * 32 + 2 * (threadIdx.x & 15);
    const bool two = k + 1 < K, one = k < K;              // K may be odd: the last channel then loads 2 bytes
    double s0 = 0.0, s1 = 0.0;
    for (int n0 = sub; n0 < N; n0 += 16 * FQW_CAS_UNROLL) {
        unsigned w[FQW_CAS_UNROLL];
#pragma unroll
        for (int u = 0; u < FQW_CAS_UNROLL; ++u) {
            const int n = n0 + 16 * u;
            w[u] = 0u;
            if (n < N && one) {
                const uint16_t* src = W + (size_t)n * K + k;
                // a dword load needs 4-byte alignment, which an odd row length breaks on every other row
                if (two && ((reinterpret_cast<uintptr_t>(src) & 3u) == 0)) w[u] = *reinterpret_cast<const unsigned*>(src);
                else w[u] = (unsigned)src[0] | (two ? (unsigned)src[1] << 16 : 0u);
            }
        }
#pragma unroll
        for (int u = 0; u < FQW_CAS_UNROLL; ++u) {
            s0 += (double)fabsf(fqw_bf16((unsigned short)(w[u] & 0xFFFFu)));
            s1 += (double)fabsf(fqw_bf16((unsigned short)(w[u] >> 16)));
        }
    }
    part[sub][2 * (threadIdx.x & 15)] = s0;
    part[sub][2 * (threadIdx.x & 15) + 1] = s1;
    __syncthreads();
    if (threadIdx.x < 32 && blockIdx.x * 32 + (int)threadIdx.x < K) {
        double t = 0.0;
#pragma unroll
        for (int r = 0; r < 16; ++r) t += part[r][threadIdx.x];
        lambda[blockIdx.x * 32 + threadIdx.x] =
            t == 0.0 ? 1.0f : (float)((double)target / (t / (double)N));            // an all-zero channel keeps 1
    }
}

// ---- per-tensor scaling: statistics, then the choice of n --------------------------------------------
// stats[0]: bits of the smallest non-zero |v| (0xFFFFFFFF: none); stats[1..4]: bit n of this 128-bit mask
// is set when some element lies in the band of condition 2 for that n.
__global__ void fq_pts_init_kernel(unsigned* __restrict__ stats) {
    if (threadIdx.x < 8) stats[threadIdx.x] = threadIdx.x == 0 ? 0xFFFFFFFFu : 0u;
}

__global__ __launch_bounds__(256) void fq_pts_stats_kernel(const uint16_t* __restrict__ W,
                                                           const float* __restrict__ lambda,
                                                           unsigned* __restrict__ stats, size_t chunks, int K) {
    unsigned vmin = 0xFFFFFFFFu;
    unsigned long long mlo = 0ull, mhi = 0ull;            // bands 0..63 and 64..127
    const size_t stride = (size_t)gridDim.x * 256u;
    for (size_t c = (size_t)blockIdx.x * 256u + threadIdx.x; c < chunks; c += stride) {   // 8 weights per chunk
        const fq_v4i w = *reinterpret_cast<const fq_v4i*>(W + c * 8);
        const int k0 = (int)((c * 8) % (size_t)K);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const unsigned word = (unsigned)w[i >> 1];
            float v = fqw_bf16((unsigned short)((i & 1) ? (word >> 16) : (word & 0xFFFFu)));
            if (lambda) v *= lambda[k0 + i];
            const unsigned b = __float_as_uint(v) & 0x7FFFFFFFu;
            if (b != 0u) {
                vmin = b < vmin ? b : vmin;
                const int n = 5 - fqw_log2_over_7(b);     // the n whose band holds this element
                const unsigned long long bit = 1ull << (n & 63);
                mlo |= (n >= 0 && n < 64) ? bit : 0ull;
                mhi |= (n >= 64 && n <= 126) ? bit : 0ull;
            }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned other = (unsigned)__shfl_xor((int)vmin, o, 64);
        vmin = other < vmin ? other : vmin;
        mlo |= (unsigned long long)__shfl_xor((long long)mlo, o, 64);
        mhi |= (unsigned long long)__shfl_xor((long long)mhi, o, 64);
    }
    // one set of atomics per workgroup, and only those that would change the statistics (the plain reads
    // may be stale: that costs at most an atomic that changes nothing): thousands of atomics on five
    // addresses would otherwise take longer than reading the matrix
    __shared__ unsigned red[4][5];
    if ((threadIdx.x & 63) == 0) {
        unsigned* r = red[threadIdx.x >> 6];
        r[0] = vmin;
        r[1] = (unsigned)mlo; r[2] = (unsigned)(mlo >> 32); r[3] = (unsigned)mhi; r[4] = (unsigned)(mhi >> 32);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned m0 = red[0][0];
#pragma unroll
        for (int w = 1; w < 4; ++w) m0 = red[w][0] < m0 ? red[w][0] : m0;
        const volatile unsigned* seen = stats;
        if (m0 < seen[0]) atomicMin(&stats[0], m0);
#pragma unroll
        for (int j = 1; j < 5; ++j) {
            const unsigned m = red[0][j] | red[1][j] | red[2][j] | red[3][j];
            if (m & ~seen[j]) atomicOr(&stats[j], m);
        }
    }
}

// Condition 1 holds from the n at which the smallest non-zero element reaches 7 * 2^-9 (then no
// non-zero element adds to S any more, and zeros add the same for every n); condition 2 at the
// lowest band that holds an element.  n is the smaller of the two, at most 126.
__global__ void fq_pts_resolve_kernel(const unsigned* __restrict__ stats, int* __restrict__ n_out) {
    if (threadIdx.x != 0) return;
    int n1 = 0;
    if (stats[0] != 0xFFFFFFFFu) {
        n1 = -9 - fqw_log2_over_7(stats[0]);
        n1 = n1 < 0 ? 0 : n1;
    }
    int n2 = 127;
    for (int j = 3; j >= 0; --j)
        if (stats[1 + j]) n2 = 32 * j + __builtin_ctz(stats[1 + j]);
    int n = n1 < n2 ? n1 : n2;
    n_out[0] = n > 126 ? 126 : n;
}

// ---- group-wise INT4 quantisation ------------------------------------------------------------------
// 16 lanes per group of 128 weights (8 neighbouring weights = 16 bytes per lane): a wave quantises four
// groups, a workgroup sixteen.
__global__ __launch_bounds__(256) void fq_quantize_weights_kernel(const uint16_t* __restrict__ W,
                                                                  const float* __restrict__ lambda, int n_pts,
                                                                  int sigma_rne, int8_t* __restrict__ q,
                                                                  uint8_t* __restrict__ gs, size_t groups, int K) {
    const size_t grp = (size_t)blockIdx.x * 16u + (threadIdx.x >> 4);
    if (grp >= groups) return;                            // whole 16-lane teams leave together
    const size_t e0 = grp * FQ_GROUP + 8 * (threadIdx.x & 15);   // K is a multiple of 128: a group never straddles rows
    const fq_v4i w = *reinterpret_cast<const fq_v4i*>(W + e0);
    const float p2n = __uint_as_float((unsigned)(n_pts + 127) << 23);    // 2^n, 0 <= n <= 126
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned word = (unsigned)w[i >> 1];
        v[i] = fqw_bf16((unsigned short)((i & 1) ? (word >> 16) : (word & 0xFFFFu)));
    }
    if (lambda) {
        const int k = (int)(e0 % (size_t)K);
        const fq_v4f l0 = *reinterpret_cast<const fq_v4f*>(lambda + k), l1 = *reinterpret_cast<const fq_v4f*>(lambda + k + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[i] *= l0[i];
            v[4 + i] *= l1[i];
        }
    }
    float vmax = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v[i] *= p2n;
        vmax = fmaxf(vmax, fabsf(v[i]));
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) vmax = fmaxf(vmax, __shfl_xor(vmax, o, 64));
    const float sigma = fminf(vmax / 7.0f, 448.0f);
    unsigned code = (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(sigma, sigma, 0, false) & 0xFFu;   // nearest even
    float s8 = __builtin_amdgcn_cvt_f32_fp8((int)code, 0);
    if (!sigma_rne && s8 > sigma) {                       // toward zero: one code down (positive codes are ordered)
        code -= 1u;
        s8 = __builtin_amdgcn_cvt_f32_fp8((int)code, 0);
    }
    unsigned out[2] = {0u, 0u};
    if (s8 > 0.f) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = (int)fminf(fmaxf(rintf(v[i] / s8), -8.f), 7.f);
            out[i >> 2] |= (unsigned)(c & 0xFF) << (8 * (i & 3));
        }
    }
    *reinterpret_cast<fq_v2i*>(q + e0) = (fq_v2i){(int)out[0], (int)out[1]};
    if ((threadIdx.x & 15) == 0) gs[grp] = (uint8_t)code;
}

void fq_launch_cas_scales(const uint16_t* W, float target, float* lambda, int N, int K, hipStream_t stream) {
    hipLaunchKernelGGL(fq_cas_scales_kernel, dim3((unsigned)((K + 31) / 32)), dim3(256), 0, stream, W, target, lambda, N, K);
}

void fq_launch_pts_exponent(const uint16_t* W, const float* lambda, int* n_out, int N, int K, hipStream_t stream) {
    unsigned* stats = reinterpret_cast<unsigned*>(n_out) + 8;     // the caller's 64 bytes: [0] = n, [8..12] statistics
    const size_t chunks = (size_t)N * (size_t)K / 8u;
    size_t blocks = (chunks + 255u) / 256u;
    if (blocks > 2048u) blocks = 2048u;
    hipLaunchKernelGGL(fq_pts_init_kernel, dim3(1), dim3(64), 0, stream, stats);
    hipLaunchKernelGGL(fq_pts_stats_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, W, lambda, stats, chunks, K);
    hipLaunchKernelGGL(fq_pts_resolve_kernel, dim3(1), dim3(64), 0, stream, stats, n_out);
}

void fq_launch_quantize_weights(const uint16_t* W, const float* lambda, int n_pts, bool sigma_rne, int8_t* q,
                                uint8_t* gs, int N, int K, hipStream_t stream) {
    const size_t groups = (size_t)N * (size_t)(K / FQ_GROUP);
    hipLaunchKernelGGL(fq_quantize_weights_kernel, dim3((unsigned)((groups + 15u) / 16u)), dim3(256), 0, stream, W, lambda,
                       n_pts, sigma_rne ? 1 : 0, q, gs, groups, K);
}
