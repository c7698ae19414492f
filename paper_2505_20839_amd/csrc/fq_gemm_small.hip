// W4A8-FP GEMM for small M (decode, M <= 64): bound by streaming the packed INT4 weights from HBM
// once (Sec. 1: memory bandwidth is what motivates 4-bit weights).  Same arithmetic as the
// large-M kernel (Sec. 3.1.1): unpack INT4 to E4M3 in registers, FP8 MFMA with FP32 accumulation,
// exact FP32 group scale, one rounding to bf16.
//
// Work split.  One workgroup per 32 output channels; its waves split K: wave w takes a contiguous
// range of 128-wide groups, keeps up to FQS_DEPTH groups of packed weights (2 KiB each) in flight,
// and accumulates a 32 x 32 (x MT row tiles) partial result.  The partial results of the waves are
// summed through LDS and written as bf16.  Activations are tiny (M x K bytes) and are read straight
// from L2 in MFMA operand order.
#include "fq_common.h"
#include "fq_kernels.h"

#define FQS_THREADS 256
#define FQS_WAVES (FQS_THREADS / 64)
#define FQS_DEPTH 8

#define FQ_MFMA(a, b, c) __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4((a), (b), (c), 0, 0, 0, 0, 0, 0)

namespace {

__device__ __forceinline__ fq_v8i fqs_join(fq_v4i lo, fq_v4i hi) {
    fq_v8i r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return r;
}

}  // namespace

template <int MT>
__global__ __launch_bounds__(FQS_THREADS) void fq_gemm_small_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* __restrict__ Y, int M, int N, int K) {
    __shared__ float red[FQS_WAVES][MT][16][64];
    const int G = K / FQ_GROUP;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nt = blockIdx.x;
    const int n = nt * 32 + (lane & 31);
    const bool n_ok = n < N;
    const int per = (G + FQS_WAVES - 1) / FQS_WAVES;
    const int g_begin = wave * per;
    const int g_end = (g_begin + per < G) ? g_begin + per : G;
    const uint8_t* wblk = wp + fq_block_offset(nt, 0, G) + (size_t)lane * 16u;
    const uint8_t* gsrow = gs + (size_t)(n_ok ? n : 0) * G;
    // this lane's activation rows (clamped: rows past M are computed and dropped)
    const uint8_t* arow[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        int m = t * 32 + (lane & 31);
        m = m < M ? m : M - 1;
        arow[t] = A + (size_t)m * K + (lane >> 5) * 32;
    }

    fq_v16f acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    fq_v16f zero;
#pragma unroll
    for (int r = 0; r < 16; ++r) zero[r] = 0.f;

    fq_v4i bq[FQS_DEPTH][2];
    unsigned sq[FQS_DEPTH];
#pragma unroll
    for (int i = 0; i < FQS_DEPTH; ++i) {
        bq[i][0] = (fq_v4i){0, 0, 0, 0};
        bq[i][1] = (fq_v4i){0, 0, 0, 0};
        sq[i] = 0;
        int g = g_begin + i;
        if (g < g_end) {
            const uint8_t* p = wblk + (size_t)g * 2048u;
            bq[i][0] = __builtin_nontemporal_load(reinterpret_cast<const fq_v4i*>(p));
            bq[i][1] = __builtin_nontemporal_load(reinterpret_cast<const fq_v4i*>(p + 1024));
            sq[i] = gsrow[g];
        }
    }

    for (int gb = g_begin; gb < g_end; gb += FQS_DEPTH) {
#pragma unroll
        for (int i = 0; i < FQS_DEPTH; ++i) {
            const int g = gb + i;
            if (g < g_end) {
                // activations of this group, in operand order: lane (row, kh) holds 32 consecutive k per half
                fq_v8i a[MT][2];
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const fq_v4i* ap = reinterpret_cast<const fq_v4i*>(arow[t] + (size_t)g * FQ_GROUP);
                    a[t][0] = fqs_join(ap[0], ap[1]);
                    a[t][1] = fqs_join(ap[4], ap[5]);
                }
                fq_v8i b0 = fq_unpack_chunk(bq[i][0]);
                fq_v8i b1 = fq_unpack_chunk(bq[i][1]);
                float s = __builtin_amdgcn_cvt_f32_fp8((int)sq[i], 0);
                const int gn = g + FQS_DEPTH;
                if (gn < g_end) {                         // refill this slot
                    const uint8_t* p = wblk + (size_t)gn * 2048u;
                    bq[i][0] = __builtin_nontemporal_load(reinterpret_cast<const fq_v4i*>(p));
                    bq[i][1] = __builtin_nontemporal_load(reinterpret_cast<const fq_v4i*>(p + 1024));
                    sq[i] = gsrow[gn];
                }
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    fq_v16f p = FQ_MFMA(a[t][0], b0, zero);
                    p = FQ_MFMA(a[t][1], b1, p);
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[t][r] = fmaf(s, p[r], acc[t][r]);
                }
            }
        }
    }

    // ---- sum the K-slices of the waves through LDS, scale, write bf16 ----
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave][t][r][lane] = acc[t][r];
    __syncthreads();
    const float outer = tscale * 512.0f;                  // weights were fed as q * 2^-9
    for (int idx = threadIdx.x; idx < MT * 16 * 64; idx += FQS_THREADS) {
        int l = idx & 63, r = (idx >> 6) & 15, t = idx >> 10;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < FQS_WAVES; ++w) v += red[w][t][r][l];
        int m = t * 32 + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
        int nn = nt * 32 + (l & 31);
        if (m < M && nn < N) Y[(size_t)m * N + nn] = (uint16_t)fq_float_to_bf16(v * (a_scale[m] * outer));
    }
}

// ---------------------------------------------------------------------------------------------
// M <= 16: one 16-row MFMA tile (v_mfma_f32_16x16x128_f8f6f4 = exactly one group per instruction).
// The output channels are dealt out evenly, in multiples of 8, to one workgroup per compute unit
// (N = 14336 on 256 units: 56 channels each), so that every unit streams the same number of weight
// bytes and the whole matrix is requested at once.  A workgroup of 8 waves covers its channels with
// up to four 16-channel sub-tiles (the last one may be partly masked); the waves split K into eight
// contiguous slices, so each activation byte is read once per workgroup and each weight byte once
// overall.  A wave requests all packed weights of a batch of four groups before it computes
// anything; with K = 4096 that is its whole share.
// The 16x16x128 operand of lane l = 16*kq + r holds 32 consecutive k (32*kq ..) of row/channel r,
// which is one 16-byte chunk of the packed block: chunk (h = kq/2, kh = kq%2, channel % 32).
// ---------------------------------------------------------------------------------------------
#define FQS16_THREADS 512
#define FQS16_WAVES 8
#define FQS16_BATCH 4
#define FQS16_NSUB 4
#define FQ_MFMA16(a, b, c) __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4((a), (b), (c), 0, 0, 0, 0, 0, 0)

__global__ __launch_bounds__(FQS16_THREADS) void fq_gemm_small16_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* __restrict__ Y, int M, int N, int K, int cols) {
    __shared__ float red[FQS16_WAVES][FQS16_NSUB][4][64];
    const int G = K / FQ_GROUP;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kq = lane >> 4;
    const int n_first = blockIdx.x * cols;                // this workgroup owns channels [n_first, n_first + cols)
    const int per = (G + FQS16_WAVES - 1) / FQS16_WAVES;
    const int g_begin = wave * per;
    const int g_end = (g_begin + per < G) ? g_begin + per : G;

    // per sub-tile: this lane's channel, its chunk in group 0 of the packed block, its scale row
    const uint8_t* wsub[FQS16_NSUB];
    const uint8_t* gsub[FQS16_NSUB];
    bool on[FQS16_NSUB];
#pragma unroll
    for (int j = 0; j < FQS16_NSUB; ++j) {
        const int c = 16 * j + r16;
        int n = n_first + c;
        on[j] = (c < cols) && (n < N);                    // masked lanes request nothing and store nothing
        n = on[j] ? n : 0;
        wsub[j] = wp + fq_block_offset(n >> 5, 0, G) + (size_t)(kq >> 1) * 1024u +
                  (size_t)((kq & 1) * 32 + (n & 31)) * 16u;
        gsub[j] = gs + (size_t)n * G;
    }
    const uint8_t* arow = A + (size_t)(r16 < M ? r16 : M - 1) * K + kq * 32;
    // output factor of the (at most two) elements this thread writes at the end, fetched up front
    float osc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int idx = threadIdx.x + i * FQS16_THREADS;
        const int m = 4 * ((idx & 63) >> 4) + ((idx >> 6) & 3);
        osc[i] = a_scale[m < M ? m : M - 1];
    }

    fq_v4f acc[FQS16_NSUB];
#pragma unroll
    for (int j = 0; j < FQS16_NSUB; ++j) acc[j] = (fq_v4f){0.f, 0.f, 0.f, 0.f};
    const fq_v4f zero4 = {0.f, 0.f, 0.f, 0.f};

    for (int gb = g_begin; gb < g_end; gb += FQS16_BATCH) {
        fq_v4i bq[FQS16_BATCH][FQS16_NSUB];
        fq_v4i aq[FQS16_BATCH][2];
        unsigned sq[FQS16_BATCH][FQS16_NSUB];
        // requests in the order they are consumed, so the first group can start while the rest lands
#pragma unroll
        for (int i = 0; i < FQS16_BATCH; ++i) {
            int g = gb + i;
            g = g < g_end ? g : g_end - 1;                // short last batch: duplicates, skipped below
            const fq_v4i* ap = reinterpret_cast<const fq_v4i*>(arow + (size_t)g * FQ_GROUP);
            aq[i][0] = ap[0];
            aq[i][1] = ap[1];
#pragma unroll
            for (int j = 0; j < FQS16_NSUB; ++j) sq[i][j] = gsub[j][g];
#pragma unroll
            for (int j = 0; j < FQS16_NSUB; ++j) {
                bq[i][j] = (fq_v4i){0, 0, 0, 0};
                if (on[j])
                    bq[i][j] = __builtin_nontemporal_load(reinterpret_cast<const fq_v4i*>(wsub[j] + (size_t)g * 2048u));
            }
        }
#pragma unroll
        for (int i = 0; i < FQS16_BATCH; ++i) {
            if (gb + i < g_end) {
                fq_v8i a = fqs_join(aq[i][0], aq[i][1]);
#pragma unroll
                for (int j = 0; j < FQS16_NSUB; ++j) {
                    if (16 * j < cols) {                  // uniform: sub-tiles past the share are skipped
                        fq_v8i b = fq_unpack_chunk(bq[i][j]);
                        float s = __builtin_amdgcn_cvt_f32_fp8((int)sq[i][j], 0);
                        fq_v4f p = FQ_MFMA16(a, b, zero4);
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[j][r] = fmaf(s, p[r], acc[j][r]);
                    }
                }
            }
        }
    }

    // ---- sum the K-slices of the 8 waves through LDS, scale, write bf16 ----
#pragma unroll
    for (int j = 0; j < FQS16_NSUB; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][j][r][lane] = acc[j][r];
    __syncthreads();
    const float outer = tscale * 512.0f;                  // weights were fed as q * 2^-9
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int idx = threadIdx.x + i * FQS16_THREADS;  // 1024 outputs: [sub-tile][reg][lane]
        const int l = idx & 63, r = (idx >> 6) & 3, j = idx >> 8;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < FQS16_WAVES; ++w) v += red[w][j][r][l];
        const int m = 4 * (l >> 4) + r;
        const int c = 16 * j + (l & 15);
        const int n = n_first + c;
        if (m < M && c < cols && n < N) {
            fq_v2f pr = {v * (osc[i] * outer), 0.f};
            fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
            Y[(size_t)m * N + n] = __builtin_bit_cast(unsigned short, pk[0]);
        }
    }
}

void fq_launch_gemm_small(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                          float tscale, uint16_t* Y, int M, int N, int K, hipStream_t stream) {
    if (M <= 16) {
        // channels per workgroup: an even share of N over the compute units, a multiple of 8, at most 64
        int dev = 0, cus = 256;
        if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        int cols = ((N + cus - 1) / cus + 7) & ~7;
        cols = cols < 8 ? 8 : (cols > 64 ? 64 : cols);
        hipLaunchKernelGGL(fq_gemm_small16_kernel, dim3((unsigned)((N + cols - 1) / cols)), dim3(FQS16_THREADS), 0, stream,
                           A, a_scale, wp, gs, tscale, Y, M, N, K, cols);
        return;
    }
    dim3 grid((unsigned)((N + 31) / 32));
    for (int m0 = 0; m0 < M; m0 += 64) {                  // M > 64 is served in slabs of 64 rows
        int mm = (M - m0 < 64) ? M - m0 : 64;
        const uint8_t* Ab = A + (size_t)m0 * K;
        uint16_t* Yb = Y + (size_t)m0 * N;
        if (mm <= 32)
            hipLaunchKernelGGL(fq_gemm_small_kernel<1>, grid, dim3(FQS_THREADS), 0, stream,
                               Ab, a_scale + m0, wp, gs, tscale, Yb, mm, N, K);
        else
            hipLaunchKernelGGL(fq_gemm_small_kernel<2>, grid, dim3(FQS_THREADS), 0, stream,
                               Ab, a_scale + m0, wp, gs, tscale, Yb, mm, N, K);
    }
}
