// W4A8-FP GEMM for large M (compute bound): INT4 weights x E4M3 activations on the gfx950 FP8
// matrix cores (Sec. 3.1.1: unpack INT4 to FP8 in registers, FP8 MMA with FP32 accumulation,
// scale and write bf16).  Differences from the paper's H100 kernel: the group scale is not folded
// into a rounded FP8 table but applied exactly, in FP32, to each group's partial sum; all output
// scaling is FP32 with a single rounding to bf16.
//
// Work split.  A workgroup of 8 waves owns a 256 x (32*NW*...) output tile; wave w owns 32
// output channels and all 256 rows (8 MFMA tiles of 32x32), so every weight is unpacked exactly
// once per workgroup and each unpacked operand is reused by 8 row tiles.  Per 128-wide group g:
//     P   = A[:, g, first 64] * Wq[g, first 64]            v_mfma_f32_32x32x64_f8f6f4, C = 0
//     P  += A[:, g, last 64]  * Wq[g, last 64]             same, C = P
//     acc += e4m3(gscale[n, g]) * P                        16 v_fma_f32 per 32x32 tile
// A tiles go global -> registers -> LDS (three stages of 32 KiB), packed weights go global ->
// registers directly (each wave reads only its own 32 channels).
#include "fq_common.h"
#include "fq_kernels.h"

#define FQL_THREADS 512
#define FQL_BM 256
#define FQL_STAGE_BYTES (FQL_BM * FQ_GROUP)          // 32 KiB: 256 rows x 128 E4M3 bytes
#define FQL_STAGES 3

#define FQ_MFMA(a, b, c) __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4((a), (b), (c), 0, 0, 0, 0, 0, 0)

namespace {

// LDS layout of one A stage: 16-byte chunks ordered [row tile mt (8)][half h (2)][part (2)][lane (64)],
// lane = 32*kh + (row % 32), holding A[row][64*h + 32*kh + 16*part .. +16] of the current group.
// A wave reads the two parts of (mt, h) with two ds_read_b128 whose addresses are linear in the lane.
__device__ __forceinline__ int fql_lds_chunk(int row, int kc) {
    int h = kc >> 2, kh = (kc >> 1) & 1, part = kc & 1;
    return ((((row >> 5) * 2 + h) * 2 + part) << 6) + (kh << 5) + (row & 31);
}

struct AStage { fq_v4i v[4]; };

__device__ __forceinline__ void fql_load_a(AStage& st, const uint8_t* __restrict__ A, int M, int K,
                                           int m0, int g) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int c = threadIdx.x + i * FQL_THREADS;            // 2048 chunks: row = c / 8, kc = c % 8
        int row = m0 + (c >> 3);
        row = row < M ? row : M - 1;
        st.v[i] = *reinterpret_cast<const fq_v4i*>(A + (size_t)row * K + (size_t)g * FQ_GROUP + (c & 7) * 16);
    }
}

__device__ __forceinline__ void fql_store_a(const AStage& st, fq_v4i* lds_stage) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int c = threadIdx.x + i * FQL_THREADS;
        lds_stage[fql_lds_chunk(c >> 3, c & 7)] = st.v[i];
    }
}

}  // namespace

__global__ __launch_bounds__(FQL_THREADS) void fq_gemm_large_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* __restrict__ Y, int M, int N, int K) {
    extern __shared__ fq_v4i lds[];                       // FQL_STAGES stages of 2048 chunks
    const int G = K / FQ_GROUP;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m0 = blockIdx.y * FQL_BM;
    const int nw0 = blockIdx.x * 256 + wave * 32;         // first output channel of this wave
    const bool wave_on = nw0 < N;                         // waves past N only help moving A
    const int n = nw0 + (lane & 31);                      // this lane's output channel
    const bool n_ok = n < N;
    const uint8_t* wblk = wp + fq_block_offset(nw0 >> 5, 0, G) + (size_t)lane * 16u;
    const uint8_t* gsrow = gs + (size_t)(n_ok ? n : 0) * G;

    fq_v16f acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    fq_v16f zero;
#pragma unroll
    for (int r = 0; r < 16; ++r) zero[r] = 0.f;

    // ---- prologue: A stages 0 and 1, packed weights and scale of group 0 ----
    AStage st;
    fql_load_a(st, A, M, K, m0, 0);
    fql_store_a(st, lds);
    if (G > 1) {
        fql_load_a(st, A, M, K, m0, 1);
        fql_store_a(st, lds + 2048);
    }
    fq_v4i bp0 = {0, 0, 0, 0}, bp1 = {0, 0, 0, 0};
    unsigned sbyte = 0;
    if (wave_on) {
        bp0 = *reinterpret_cast<const fq_v4i*>(wblk);
        bp1 = *reinterpret_cast<const fq_v4i*>(wblk + 1024);
        sbyte = gsrow[0];
    }
    __syncthreads();

    fq_v16f pprev = zero;                                 // partial sums of the previous row tile
    float sprev = 0.f;                                    // and their group scale
    for (int g = 0; g < G; ++g) {
        const fq_v4i* cur = lds + (g % FQL_STAGES) * 2048;
        const bool more2 = g + 2 < G;
        if (more2) fql_load_a(st, A, M, K, m0, g + 2);
        fq_v8i b0 = fq_unpack_chunk(bp0);
        fq_v8i b1 = fq_unpack_chunk(bp1);
        float s = __builtin_amdgcn_cvt_f32_fp8((int)sbyte, 0);
        if (wave_on && g + 1 < G) {
            const uint8_t* nb = wblk + (size_t)(g + 1) * 2048u;
            bp0 = *reinterpret_cast<const fq_v4i*>(nb);
            bp1 = *reinterpret_cast<const fq_v4i*>(nb + 1024);
            sbyte = gsrow[g + 1];
        }
        if (wave_on) {
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) {
                const fq_v4i* ap = cur + mt * 256 + lane;
                fq_v8i a0, a1;
                fq_v4i t0 = ap[0], t1 = ap[64], t2 = ap[128], t3 = ap[192];
                a0[0] = t0[0]; a0[1] = t0[1]; a0[2] = t0[2]; a0[3] = t0[3];
                a0[4] = t1[0]; a0[5] = t1[1]; a0[6] = t1[2]; a0[7] = t1[3];
                a1[0] = t2[0]; a1[1] = t2[1]; a1[2] = t2[2]; a1[3] = t2[3];
                a1[4] = t3[0]; a1[5] = t3[1]; a1[6] = t3[2]; a1[7] = t3[3];
                fq_v16f p = FQ_MFMA(a0, b0, zero);
                p = FQ_MFMA(a1, b1, p);
                // scale-accumulate the previous tile while these two MFMAs run
                const int tp = (mt + 7) & 7;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[tp][r] = fmaf(sprev, pprev[r], acc[tp][r]);
                pprev = p;
                if (mt == 0) sprev = s;                   // tiles 0..7 of this group use s; tile 7 of the previous group used the old value
            }
        }
        if (more2) fql_store_a(st, lds + ((g + 2) % FQL_STAGES) * 2048);
        __syncthreads();
    }
    // last pending tile (row tile 7 of the last group)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[7][r] = fmaf(sprev, pprev[r], acc[7][r]);

    // ---- epilogue: per-token and per-tensor factors (x 2^9: weights were fed as q * 2^-9), bf16 ----
    if (!wave_on || !n_ok) return;
    const float outer = tscale * 512.0f;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int m = m0 + mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (m < M) Y[(size_t)m * N + n] = (uint16_t)fq_float_to_bf16(acc[mt][r] * (a_scale[m] * outer));
        }
    }
}

void fq_launch_gemm_large(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                          float tscale, uint16_t* Y, int M, int N, int K, hipStream_t stream) {
    static bool attr_set = false;
    const int lds_bytes = FQL_STAGES * FQL_STAGE_BYTES;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fq_gemm_large_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        attr_set = true;
    }
    dim3 grid((unsigned)((N + 255) / 256), (unsigned)((M + FQL_BM - 1) / FQL_BM));
    hipLaunchKernelGGL(fq_gemm_large_kernel, grid, dim3(FQL_THREADS), lds_bytes, stream,
                       A, a_scale, wp, gs, tscale, Y, M, N, K);
}
