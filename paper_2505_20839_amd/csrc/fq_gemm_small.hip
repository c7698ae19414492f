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

    fq_v8i zp;
#pragma unroll
    for (int r = 0; r < 8; ++r) zp[r] = (int)FQ_ZP_BYTES;

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
                    fq_v16f p = FQ_MFMA(a[t][0], zp, zero);   // zero point: -2^-6 * sum_k a_k in every column
                    p = FQ_MFMA(a[t][1], zp, p);
                    p = FQ_MFMA(a[t][0], b0, p);
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
    const float outer = tscale * 512.0f;                  // weights were fed in units of 2^-9
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
// NSUB <= 4 sub-tiles of 16 channels (the last one may be partly masked); the waves split K into
// eight contiguous slices, so each activation byte is read once per workgroup and each weight byte
// once overall.  A wave requests all packed weights of a batch of four groups before it computes
// anything; with K = 4096 that is its whole share.
// Every load is a raw buffer load: masked lanes carry an out-of-range offset (they fetch nothing
// and read zero), group steps travel in the scalar offset, and the code has no branches between
// the first request and the last MFMA.
// The 16x16x128 operand of lane l = 16*kq + r holds 32 consecutive k (32*kq ..) of row/channel r,
// which is one 16-byte chunk of the packed block: chunk (h = kq/2, kh = kq%2, channel % 32).
// ---------------------------------------------------------------------------------------------
#define FQS16_THREADS 512
#define FQS16_WAVES 8
#define FQS16_OOB 0xFFFFFF00u                             // beyond any 32-bit buffer size
// byte `i` (0..3, compile-time) of a word of E4M3 codes -> float
__device__ __forceinline__ float fq_e4m3_byte_to_float(unsigned w, int i) {
    return i == 0 ? __builtin_amdgcn_cvt_f32_fp8((int)w, 0) : i == 1 ? __builtin_amdgcn_cvt_f32_fp8((int)w, 1)
         : i == 2 ? __builtin_amdgcn_cvt_f32_fp8((int)w, 2) : __builtin_amdgcn_cvt_f32_fp8((int)w, 3);
}
#define FQ_MFMA16(a, b, c) __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4((a), (b), (c), 0, 0, 0, 0, 0, 0)

// WORDS: every wave's slice starts at a multiple of 4 groups and the scale rows are word-aligned,
// so four consecutive scale bytes of a channel are one aligned word.
// A wave keeps a ring of BATCH groups in flight (NSUB * BATCH = 16, 12 or 8 weight chunks per lane):
// it requests the first BATCH groups of its slice at once and re-requests each slot, for the group
// BATCH further on, as soon as it has used it.  Loads return in order, so the ring is consumed in
// the order it was requested.
template <int NSUB, bool WORDS>
struct fqs16_ring {
    static constexpr int BATCH = NSUB <= 2 ? 8 : 4;
    fq_v4i bq[BATCH][NSUB];
    fq_v4i aq[BATCH][2];
    unsigned sq[WORDS ? BATCH / 4 : BATCH][NSUB];         // scale bytes, or words of four

    // request group g into slot i; groups at or past g_end request nothing and read as zeros
    __device__ __forceinline__ void issue(int i, __amdgpu_buffer_rsrc_t rsA, __amdgpu_buffer_rsrc_t rsW,
                                          __amdgpu_buffer_rsrc_t rsG, unsigned aoff, const unsigned (&woff)[NSUB],
                                          const unsigned (&goff)[NSUB], int g, int g_end) {
        const unsigned dead = g < g_end ? 0u : FQS16_OOB;
        if (WORDS) {
            if (i % 4 == 0) {
#pragma unroll
                for (int j = 0; j < NSUB; ++j)
                    sq[i / 4][j] = __builtin_amdgcn_raw_buffer_load_b32(rsG, goff[j] | dead, g, 0);
            }
        } else {
#pragma unroll
            for (int j = 0; j < NSUB; ++j) sq[i][j] = __builtin_amdgcn_raw_buffer_load_b8(rsG, goff[j] | dead, g, 0);
        }
        aq[i][0] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsA, aoff | dead, g * FQ_GROUP, 0));
        aq[i][1] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsA, (aoff + 16u) | dead, g * FQ_GROUP, 0));
#pragma unroll
        for (int j = 0; j < NSUB; ++j)                    // streamed once: non-temporal
            bq[i][j] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsW, woff[j] | dead, g * 2048, 2));
    }

    // slot i -> accumulators (a dead group is all zeros and adds nothing); `sw` is the slot's scale
    // word, read before the slot group's first slot may be re-requested
    __device__ __forceinline__ void compute(int i, fq_v4f (&acc)[NSUB], const unsigned (&sw)[NSUB]) const {
        const fq_v4f zero4 = {0.f, 0.f, 0.f, 0.f};
        const fq_v8i a = fqs_join(aq[i][0], aq[i][1]);
        fq_v8i zp;
#pragma unroll
        for (int r = 0; r < 8; ++r) zp[r] = (int)FQ_ZP_BYTES;
        const fq_v4f c0 = FQ_MFMA16(a, zp, zero4);        // zero point: -2^-6 * sum_k a_k in every column
#pragma unroll
        for (int j = 0; j < NSUB; ++j) {
            const fq_v8i b = fq_unpack_chunk(bq[i][j]);
            const float s = WORDS ? fq_e4m3_byte_to_float(sw[j], i % 4) : __builtin_amdgcn_cvt_f32_fp8((int)sq[i][j], 0);
            const fq_v4f p = FQ_MFMA16(a, b, c0);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[j][r] = fmaf(s, p[r], acc[j][r]);
        }
    }
};

template <int NSUB, bool WORDS, bool ROUNDS>
__global__ __launch_bounds__(FQS16_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void fq_gemm_small16_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* __restrict__ Y, int M, int N, int K, int cols) {
    typedef fqs16_ring<NSUB, WORDS> ring_t;
    constexpr int BATCH = ring_t::BATCH;
    __shared__ float red[FQS16_WAVES][NSUB][4][64];
    const int G = K / FQ_GROUP;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int r16 = lane & 15, kq = lane >> 4;
    const int n_first = blockIdx.x * cols;                // this workgroup owns channels [n_first, n_first + cols)
    const int per = (G + FQS16_WAVES - 1) / FQS16_WAVES;
    const int g_begin = wave * per;
    const int g_end = (g_begin + per < G) ? g_begin + per : G;

    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(A), 0, (int)((unsigned)M * (unsigned)K), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(wp), 0, (int)((unsigned)((N + 31) >> 5) * (unsigned)G * 2048u), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsG = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(gs), 0, (int)((unsigned)N * (unsigned)G), 0x00020000);
    // per sub-tile: byte offset of this lane's chunk in group 0 of its packed block, and of its scale row
    unsigned woff[NSUB], goff[NSUB];
#pragma unroll
    for (int j = 0; j < NSUB; ++j) {
        const int c = 16 * j + r16;
        const int n = n_first + c;
        const bool on = (c < cols) && (n < N);            // masked lanes request nothing and store nothing
        woff[j] = on ? (unsigned)(n >> 5) * (unsigned)G * 2048u + (unsigned)(kq >> 1) * 1024u +
                       (unsigned)((kq & 1) * 32 + (n & 31)) * 16u
                     : FQS16_OOB;
        goff[j] = on ? (unsigned)n * (unsigned)G : FQS16_OOB;
    }
    const unsigned aoff = (unsigned)(r16 < M ? r16 : M - 1) * (unsigned)K + (unsigned)kq * 32u;
    // output factor of the (at most two) elements this thread writes at the end, fetched up front
    constexpr int NOUT = (NSUB * 256 + FQS16_THREADS - 1) / FQS16_THREADS;
    float osc[NOUT];
#pragma unroll
    for (int i = 0; i < NOUT; ++i) {
        const int idx = threadIdx.x + i * FQS16_THREADS;
        const int m = 4 * ((idx & 63) >> 4) + ((idx >> 6) & 3);
        osc[i] = a_scale[m < M ? m : M - 1];
    }

    fq_v4f acc[NSUB];
#pragma unroll
    for (int j = 0; j < NSUB; ++j) acc[j] = (fq_v4f){0.f, 0.f, 0.f, 0.f};

    ring_t ring;
#pragma unroll
    for (int i = 0; i < BATCH; ++i) ring.issue(i, rsA, rsW, rsG, aoff, woff, goff, g_begin + i, g_end);
    __builtin_amdgcn_sched_barrier(0);                    // all requests go out before any arithmetic
    // ROUNDS == false: no slice is longer than BATCH groups, the ring is used once and never refilled
    for (int gb = g_begin; gb < g_end; gb += BATCH) {
        unsigned sw[NSUB];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            if (WORDS && i % 4 == 0) {                    // keep the word: its slot may be re-requested below
#pragma unroll
                for (int j = 0; j < NSUB; ++j) sw[j] = ring.sq[i / 4][j];
            }
            ring.compute(i, acc, sw);
            __builtin_amdgcn_sched_barrier(0);            // slot by slot, as the data lands
            if (ROUNDS) {
                ring.issue(i, rsA, rsW, rsG, aoff, woff, goff, gb + BATCH + i, g_end);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (!ROUNDS) break;
    }

    // ---- sum the K-slices of the 8 waves through LDS, scale, write bf16 ----
#pragma unroll
    for (int j = 0; j < NSUB; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][j][r][lane] = acc[j][r];
    __syncthreads();
    const float outer = tscale * 512.0f;                  // weights were fed in units of 2^-9
#pragma unroll
    for (int i = 0; i < NOUT; ++i) {
        const int idx = threadIdx.x + i * FQS16_THREADS;  // NSUB * 256 outputs: [sub-tile][reg][lane]
        const int l = idx & 63, r = (idx >> 6) & 3, j = idx >> 8;
        if (j < NSUB) {
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
}

namespace {

template <int NSUB, bool WORDS>
void fq_launch_small16w(bool rounds, unsigned grid, hipStream_t stream, const uint8_t* A, const float* a_scale,
                        const uint8_t* wp, const uint8_t* gs, float tscale, uint16_t* Y, int M, int N, int K, int cols) {
    if (rounds)
        hipLaunchKernelGGL((fq_gemm_small16_kernel<NSUB, WORDS, true>), dim3(grid), dim3(FQS16_THREADS), 0, stream,
                           A, a_scale, wp, gs, tscale, Y, M, N, K, cols);
    else
        hipLaunchKernelGGL((fq_gemm_small16_kernel<NSUB, WORDS, false>), dim3(grid), dim3(FQS16_THREADS), 0, stream,
                           A, a_scale, wp, gs, tscale, Y, M, N, K, cols);
}

template <int NSUB>
void fq_launch_small16(bool words, int per, unsigned grid, hipStream_t stream, const uint8_t* A, const float* a_scale,
                       const uint8_t* wp, const uint8_t* gs, float tscale, uint16_t* Y, int M, int N, int K, int cols) {
    const bool rounds = per > fqs16_ring<NSUB, true>::BATCH;      // some slice needs the ring more than once
    if (words) fq_launch_small16w<NSUB, true>(rounds, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols);
    else       fq_launch_small16w<NSUB, false>(rounds, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols);
}

}  // namespace

void fq_launch_gemm_small(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                          float tscale, uint16_t* Y, int M, int N, int K, hipStream_t stream) {
    if (M <= 16) {
        // channels per workgroup: an even share of N over the compute units, a multiple of 8, at most 64
        static int cus = 0;
        if (cus == 0) {
            int dev = 0, v = 0;
            if (hipGetDevice(&dev) == hipSuccess &&
                hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
            else cus = 256;
        }
        int cols = ((N + cus - 1) / cus + 7) & ~7;
        cols = cols < 8 ? 8 : (cols > 64 ? 64 : cols);
        const unsigned grid = (unsigned)((N + cols - 1) / cols);
        const int G = K / FQ_GROUP, per = (G + FQS16_WAVES - 1) / FQS16_WAVES;
        const bool words = (per % 4 == 0) && (G % 4 == 0) && ((reinterpret_cast<uintptr_t>(gs) & 3) == 0);
        switch ((cols + 15) / 16) {
            case 1: fq_launch_small16<1>(words, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols); break;
            case 2: fq_launch_small16<2>(words, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols); break;
            case 3: fq_launch_small16<3>(words, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols); break;
            default: fq_launch_small16<4>(words, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols); break;
        }
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
