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
// One workgroup of 16 waves per 32 input channels (a column sum has to stay inside one workgroup to keep its
// order fixed without a scratch buffer, so the bytes in flight come from the workgroup's size).  16 lanes cover
// the 32 channels of a row (a dword = two channels each), so a wave reads 4 rows per instruction and the 16
// waves 64; FQW_CAS_UNROLL such loads are in flight per lane.  FP64 sums, combined in a fixed order: the result
// does not depend on timing.
#define FQW_CAS_UNROLL 16
#define FQW_CAS_THREADS 1024
// LPR lanes per row (2 channels each): 16 -> 32 channels per workgroup.  (8 -> 16 channels and twice the workgroups
// is slower, 57 against 35 us on 11008 x 4096: four workgroups then fetch every 128-byte line.)
template <int LPR>
__global__ __launch_bounds__(FQW_CAS_THREADS) void fq_cas_scales_kernel(const uint16_t* __restrict__ W, float target,
                                                            float* __restrict__ lambda, int N, int K) {
    constexpr int FQW_CAS_ROWS = FQW_CAS_THREADS / LPR, CH = 2 * LPR;
    __shared__ double part[FQW_CAS_ROWS][CH];
    const int sub = threadIdx.x / LPR;                    // which of the rows of a pass
    const int k = blockIdx.x * CH + 2 * (threadIdx.x % LPR);
    const bool two = k + 1 < K, one = k < K;              // K may be odd: the last channel then loads 2 bytes
    double s0 = 0.0, s1 = 0.0;
    for (int n0 = sub; n0 < N; n0 += FQW_CAS_ROWS * FQW_CAS_UNROLL) {
        unsigned w[FQW_CAS_UNROLL];
#pragma unroll
        for (int u = 0; u < FQW_CAS_UNROLL; ++u) {
            const int n = n0 + FQW_CAS_ROWS * u;
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
    part[sub][2 * (threadIdx.x % LPR)] = s0;
    part[sub][2 * (threadIdx.x % LPR) + 1] = s1;
    __syncthreads();
    if (threadIdx.x < CH && blockIdx.x * CH + (int)threadIdx.x < K) {
        double t = 0.0;
#pragma unroll 16
        for (int r = 0; r < FQW_CAS_ROWS; ++r) t += part[r][threadIdx.x];
        lambda[blockIdx.x * CH + threadIdx.x] =
            t == 0.0 ? 1.0f : (float)((double)target / (t / (double)N));            // an all-zero channel keeps 1
    }
}

// The same for rows in 16-byte steps (K a multiple of 8, W 16-byte aligned), 64 channels per workgroup: a workgroup
// then reads whole 128-byte lines (with 32 channels two workgroups fetch each line, and the memory side moved the
// matrix twice: 35 us; with 16 channels four times: 57 us), 8 lanes x 16 bytes per row, 8 rows per wave-level load,
// and keeps FQW_CASW_UNROLL of them in flight per lane -- with K / 64 workgroups (64 for K = 4096) it is the bytes in
// flight per workgroup that set the rate.  The 8 rows of a wave are added by shuffles, the 16 waves through LDS, both
// in a fixed order.
#define FQW_CASW_UNROLL 8
#define FQW_CASW_ROWS 128
__global__ __launch_bounds__(8 * FQW_CASW_ROWS) void fq_cas_scales_wide_kernel(const uint16_t* __restrict__ W, float target,
                                                                              float* __restrict__ lambda, int N, int K) {
    __shared__ double part[16][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sub = threadIdx.x >> 3;                     // which of the 128 rows of a pass
    const int k = blockIdx.x * 64 + 8 * (lane & 7);
    const bool on = k < K;                                // (K % 8 == 0: the 8 channels are inside or outside together)
    double s[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) s[i] = 0.0;
    for (int n0 = sub; n0 < N; n0 += FQW_CASW_ROWS * FQW_CASW_UNROLL) {
        fq_v4i w[FQW_CASW_UNROLL];
#pragma unroll
        for (int u = 0; u < FQW_CASW_UNROLL; ++u) {
            const int n = n0 + FQW_CASW_ROWS * u;
            w[u] = (fq_v4i){0, 0, 0, 0};
            if (n < N && on) w[u] = __builtin_nontemporal_load(reinterpret_cast<const fq_v4i*>(W + (size_t)n * K + k));
        }
#pragma unroll
        for (int u = 0; u < FQW_CASW_UNROLL; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned word = (unsigned)w[u][i];
                s[2 * i] += (double)__uint_as_float((word << 16) & 0x7FFF0000u);     // |bf16| as FP32, exact in FP64
                s[2 * i + 1] += (double)__uint_as_float(word & 0x7FFF0000u);
            }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int m = 8; m < 64; m <<= 1) s[i] += __shfl_xor(s[i], m, 64);
    if (lane < 8) {
#pragma unroll
        for (int i = 0; i < 8; ++i) part[wave][8 * lane + i] = s[i];
    }
    __syncthreads();
    if (threadIdx.x < 64 && blockIdx.x * 64 + (int)threadIdx.x < K) {
        double t = 0.0;
#pragma unroll
        for (int r = 0; r < 16; ++r) t += part[r][threadIdx.x];
        lambda[blockIdx.x * 64 + threadIdx.x] =
            t == 0.0 ? 1.0f : (float)((double)target / (t / (double)N));            // an all-zero channel keeps 1
    }
}

// ---- per-tensor scaling: statistics, then the choice of n --------------------------------------------
// stats[0]: bits of the smallest non-zero |v| (0xFFFFFFFF: none); stats[1]: bits of the largest |v| below
// 7 * 2^6 (0: none) -- the bands of condition 2 are ordered by magnitude, so the lowest band n >= 0 that holds an
// element is the band of that element.
#define FQW_BAND0_END 0x43E00000u                         // bits of 448 = 7 * 2^6: at or above it the band index is negative
__global__ void fq_pts_init_kernel(unsigned* __restrict__ stats) {
    if (threadIdx.x < 8) stats[threadIdx.x] = threadIdx.x == 0 ? 0xFFFFFFFFu : 0u;
}

// Condition 1 holds from the n at which the smallest non-zero element reaches 7 * 2^-9 (then no
// non-zero element adds to S any more, and zeros add the same for every n); condition 2 at the
// lowest band that holds an element.  n is the smaller of the two, at most 126.
__device__ __forceinline__ int fqw_pts_resolve(unsigned vmin, unsigned vmax) {
    int n1 = 0;
    if (vmin != 0xFFFFFFFFu) {
        n1 = -9 - fqw_log2_over_7(vmin);
        n1 = n1 < 0 ? 0 : n1;
    }
    int n2 = 127;
    if (vmax != 0u) {
        n2 = 5 - fqw_log2_over_7(vmax);                   // >= 0 by the choice of vmax
        n2 = n2 > 126 ? 127 : n2;
    }
    const int n = n1 < n2 ? n1 : n2;
    return n > 126 ? 126 : n;
}

// Thread t works on the 16-byte chunk (8 weights) t % (K / 8) of the rows t / (K / 8), + rows_par, ...: its 8
// input channels never change, so their lambda sit in registers, and neighbouring threads read neighbouring
// chunks.  FQW_PTS_UNROLL rows are in flight per thread.
#ifndef FQW_PTS_UNROLL
#define FQW_PTS_UNROLL 4
#endif
__global__ __launch_bounds__(256) void fq_pts_stats_kernel(const uint16_t* __restrict__ W,
                                                           const float* __restrict__ lambda,
                                                           unsigned* __restrict__ stats,
                                                           int N, int K, int rows_par) {
    unsigned vmin = 0xFFFFFFFFu, vmax = 0u;
    const int KC = K / 8;
    const unsigned t = blockIdx.x * 256u + threadIdx.x;
    const int r0 = (int)(t / (unsigned)KC), cc = (int)(t % (unsigned)KC);
    float lam[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) lam[i] = lambda ? lambda[8 * cc + i] : 1.0f;
    for (int n0 = r0; n0 < N && r0 < rows_par; n0 += FQW_PTS_UNROLL * rows_par) {
        fq_v4i w[FQW_PTS_UNROLL];
#pragma unroll
        for (int u = 0; u < FQW_PTS_UNROLL; ++u) {
            const int n = n0 + u * rows_par;
            w[u] = (fq_v4i){0, 0, 0, 0};                  // zeros change neither statistic
            if (n < N) w[u] = *reinterpret_cast<const fq_v4i*>(W + ((size_t)n * KC + cc) * 8);
        }
#pragma unroll
        for (int u = 0; u < FQW_PTS_UNROLL; ++u)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const unsigned word = (unsigned)w[u][i >> 1];
                float v = fqw_bf16((unsigned short)((i & 1) ? (word >> 16) : (word & 0xFFFFu)));
                if (lambda) v *= lam[i];
                const unsigned b = __float_as_uint(v) & 0x7FFFFFFFu;
                vmin = (b != 0u && b < vmin) ? b : vmin;
                vmax = (b < FQW_BAND0_END && b > vmax) ? b : vmax;
            }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned lo = (unsigned)__shfl_xor((int)vmin, o, 64), hi = (unsigned)__shfl_xor((int)vmax, o, 64);
        vmin = lo < vmin ? lo : vmin;
        vmax = hi > vmax ? hi : vmax;
    }
    __shared__ unsigned red[4][2];
    if ((threadIdx.x & 63) == 0) {
        red[threadIdx.x >> 6][0] = vmin;
        red[threadIdx.x >> 6][1] = vmax;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned m0 = red[0][0], m1 = red[0][1];
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            m0 = red[w][0] < m0 ? red[w][0] : m0;
            m1 = red[w][1] > m1 ? red[w][1] : m1;
        }
        // only the atomics that would change a statistic (the plain reads may be stale: that costs at most an
        // atomic that changes nothing): thousands of atomics on two addresses would otherwise take longer than
        // reading the matrix
        const volatile unsigned* seen = stats;
        if (m0 < seen[0]) atomicMin(&stats[0], m0);
        if (m1 > seen[1]) atomicMax(&stats[1], m1);
    }
}

__global__ void fq_pts_resolve_kernel(const unsigned* __restrict__ stats, int* __restrict__ n_out) {
    if (threadIdx.x == 0) n_out[0] = fqw_pts_resolve(stats[0], stats[1]);
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
#ifndef FQW_CAS_LPR
#define FQW_CAS_LPR 16
#endif
    // whole lines per workgroup where K / 64 workgroups are enough to cover half the chip (measured, N x K: 4096 x 11008
    // 34.3 -> 19.1 us; 11008 x 4096, 64 workgroups: 35.1 -> 42.3, where the conversions to FP64 bound a compute unit)
    if ((K % 8) == 0 && (reinterpret_cast<uintptr_t>(W) % 16) == 0 && 2 * ((K + 63) / 64) >= fq_device_cus()) {
        hipLaunchKernelGGL(fq_cas_scales_wide_kernel, dim3((unsigned)((K + 63) / 64)), dim3(8 * FQW_CASW_ROWS), 0, stream, W, target, lambda, N, K);
        return;
    }
    constexpr int CH = 2 * FQW_CAS_LPR;
    hipLaunchKernelGGL(fq_cas_scales_kernel<FQW_CAS_LPR>, dim3((unsigned)((K + CH - 1) / CH)), dim3(FQW_CAS_THREADS), 0, stream, W, target, lambda, N, K);
}

void fq_launch_pts_exponent(const uint16_t* W, const float* lambda, int* n_out, int N, int K, hipStream_t stream) {
    unsigned* stats = reinterpret_cast<unsigned*>(n_out) + 8;     // the caller's 64 bytes: [0] = n, [8..9] statistics
    // about 512 workgroups' worth of threads (two per compute unit: few enough that their closing atomics stay cheap),
    // as whole rows of K / 8 chunk columns
    const int KC = K / 8;
    int rows_par = (512 * 256 + KC - 1) / KC;
    if (rows_par > N) rows_par = N;
    const size_t blocks = ((size_t)KC * (size_t)rows_par + 255u) / 256u;
    hipLaunchKernelGGL(fq_pts_init_kernel, dim3(1), dim3(64), 0, stream, stats);
    hipLaunchKernelGGL(fq_pts_stats_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, W, lambda, stats, N, K, rows_par);
    hipLaunchKernelGGL(fq_pts_resolve_kernel, dim3(1), dim3(64), 0, stream, stats, n_out);
}

void fq_launch_quantize_weights(const uint16_t* W, const float* lambda, int n_pts, bool sigma_rne, int8_t* q,
                                uint8_t* gs, int N, int K, hipStream_t stream) {
    const size_t groups = (size_t)N * (size_t)(K / FQ_GROUP);
    hipLaunchKernelGGL(fq_quantize_weights_kernel, dim3((unsigned)((groups + 15u) / 16u)), dim3(256), 0, stream, W, lambda,
                       n_pts, sigma_rne ? 1 : 0, q, gs, groups, K);
}
