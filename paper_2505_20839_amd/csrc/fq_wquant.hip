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
// One workgroup per 64 input channels: lane = channel (128-byte row segments), the four waves take
// every fourth row; FP64 sums, combined in a fixed order.
__global__ __launch_bounds__(256) void fq_cas_scales_kernel(const uint16_t* __restrict__ W, float target,
                                                            float* __restrict__ lambda, int N, int K) {
    __shared__ double part[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + lane;
    double s = 0.0;
    if (k < K)
        for (int n = wave; n < N; n += 4) s += (double)fabsf(fqw_bf16(W[(size_t)n * K + k]));
    part[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && k < K) {
        const double t = ((part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]));
        lambda[k] = t == 0.0 ? 1.0f : (float)((double)target / (t / (double)N));   // an all-zero channel keeps 1
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
    unsigned vmin = 0xFFFFFFFFu, mask[4] = {0u, 0u, 0u, 0u};
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
                if (n >= 0 && n <= 126) mask[n >> 5] |= 1u << (n & 31);
            }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned other = (unsigned)__shfl_xor((int)vmin, o, 64);
        vmin = other < vmin ? other : vmin;
#pragma unroll
        for (int j = 0; j < 4; ++j) mask[j] |= (unsigned)__shfl_xor((int)mask[j], o, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        if (vmin != 0xFFFFFFFFu) atomicMin(&stats[0], vmin);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (mask[j]) atomicOr(&stats[1 + j], mask[j]);
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
// One wave per group of 128 weights: a lane holds two neighbouring ones.
__global__ __launch_bounds__(256) void fq_quantize_weights_kernel(const uint16_t* __restrict__ W,
                                                                  const float* __restrict__ lambda, int n_pts,
                                                                  int sigma_rne, int8_t* __restrict__ q,
                                                                  uint8_t* __restrict__ gs, size_t groups, int K) {
    const int lane = threadIdx.x & 63;
    const size_t grp = (size_t)blockIdx.x * 4u + (threadIdx.x >> 6);
    if (grp >= groups) return;
    const size_t e0 = grp * FQ_GROUP + 2 * lane;          // K is a multiple of 128: a group never straddles rows
    const unsigned word = *reinterpret_cast<const unsigned*>(W + e0);
    float v0 = fqw_bf16((unsigned short)(word & 0xFFFFu)), v1 = fqw_bf16((unsigned short)(word >> 16));
    if (lambda) {
        const int k = (int)(e0 % (size_t)K);
        v0 *= lambda[k];
        v1 *= lambda[k + 1];
    }
    const float p2n = __uint_as_float((unsigned)(n_pts + 127) << 23);    // 2^n, 0 <= n <= 126
    v0 *= p2n;
    v1 *= p2n;
    float vmax = fmaxf(fabsf(v0), fabsf(v1));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) vmax = fmaxf(vmax, __shfl_xor(vmax, o, 64));
    const float sigma = fminf(vmax / 7.0f, 448.0f);
    unsigned code = (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(sigma, sigma, 0, false) & 0xFFu;   // nearest even
    float s8 = __builtin_amdgcn_cvt_f32_fp8((int)code, 0);
    if (!sigma_rne && s8 > sigma) {                       // toward zero: one code down (positive codes are ordered)
        code -= 1u;
        s8 = __builtin_amdgcn_cvt_f32_fp8((int)code, 0);
    }
    int c0 = 0, c1 = 0;
    if (s8 > 0.f) {
        c0 = (int)fminf(fmaxf(rintf(v0 / s8), -8.f), 7.f);
        c1 = (int)fminf(fmaxf(rintf(v1 / s8), -8.f), 7.f);
    }
    *reinterpret_cast<unsigned short*>(q + e0) = (unsigned short)((c0 & 0xFF) | ((c1 & 0xFF) << 8));
    if (lane == 0) gs[grp] = (uint8_t)code;
}

void fq_launch_cas_scales(const uint16_t* W, float target, float* lambda, int N, int K, hipStream_t stream) {
    hipLaunchKernelGGL(fq_cas_scales_kernel, dim3((unsigned)((K + 63) / 64)), dim3(256), 0, stream, W, target, lambda, N, K);
}

void fq_launch_pts_exponent(const uint16_t* W, const float* lambda, int* n_out, int N, int K, hipStream_t stream) {
    unsigned* stats = reinterpret_cast<unsigned*>(n_out) + 8;     // the caller's 64 bytes: [0] = n, [8..12] statistics
    const size_t chunks = (size_t)N * (size_t)K / 8u;
    size_t blocks = (chunks + 255u) / 256u;
    if (blocks > 4096u) blocks = 4096u;
    hipLaunchKernelGGL(fq_pts_init_kernel, dim3(1), dim3(64), 0, stream, stats);
    hipLaunchKernelGGL(fq_pts_stats_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, W, lambda, stats, chunks, K);
    hipLaunchKernelGGL(fq_pts_resolve_kernel, dim3(1), dim3(64), 0, stream, stats, n_out);
}

void fq_launch_quantize_weights(const uint16_t* W, const float* lambda, int n_pts, bool sigma_rne, int8_t* q,
                                uint8_t* gs, int N, int K, hipStream_t stream) {
    const size_t groups = (size_t)N * (size_t)(K / FQ_GROUP);
    hipLaunchKernelGGL(fq_quantize_weights_kernel, dim3((unsigned)((groups + 3u) / 4u)), dim3(256), 0, stream, W, lambda,
                       n_pts, sigma_rne ? 1 : 0, q, gs, groups, K);
}
