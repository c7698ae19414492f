// W4A8-FP GEMM for small M (decode, M <= 64): bound by streaming the packed INT4 weights from HBM
// once (Sec. 1: memory bandwidth is what motivates 4-bit weights).  Same arithmetic as the
// large-M kernel (Sec. 3.1.1): unpack INT4 to E4M3 in registers, FP8 MFMA with FP32 accumulation,
// exact FP32 group scale, one rounding to bf16.  The packed codes carry a zero point of 8; each
// group's MFMA chain starts from -2^-6 * sum_k a_k, which one more MFMA against a constant operand
// delivers (the matrix cores are idle at these sizes).
//
// Work split (both kernels).  The output channels are dealt out evenly to one workgroup per compute
// unit; its 8 waves split K into contiguous slices of groups, so every weight byte is read once
// overall and every activation byte once per workgroup; the partial sums of the waves are added
// through LDS.  Activations are tiny (M x K bytes) and come straight from L2 in MFMA operand order.
#include <cstdlib>
#include <type_traits>
#include "fq_common.h"
#include "fq_kernels.h"

namespace {

__device__ __forceinline__ fq_v8i fqs_join(fq_v4i lo, fq_v4i hi) {
    fq_v8i r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return r;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// M <= 16: one 16-row MFMA tile (v_mfma_f32_16x16x128_f8f6f4 = exactly one group per instruction).
// The output channels are dealt out evenly, in multiples of 8, to one workgroup per compute unit
// (N = 14336 on 256 units: 56 channels each), so that every unit streams the same number of weight
// bytes and the whole matrix is requested at once.  A workgroup of 8 waves covers its channels with
// NSUB <= 4 sub-tiles of 16 channels (the last one may be partly masked); the waves split K into
// eight contiguous slices, so each activation byte is read once per workgroup and each weight byte
// once overall.  A wave requests the packed weights of its first 4, 8 or 12 groups before it computes
// anything; with K = 4096 that is its whole share.
// Every load is a raw buffer load: masked lanes carry an out-of-range offset (they fetch nothing
// and read zero), group steps travel in the scalar offset, and the code has no branches between
// the first request and the last MFMA.
// The 16x16x128 operand of lane l = 16*kq + r holds 32 consecutive k (32*kq ..) of row/channel r,
// which is one 16-byte chunk of the packed block: chunk (h = kq/2, kh = kq%2, channel % 32).
// ---------------------------------------------------------------------------------------------
#define FQS16_THREADS 512
#define FQS16_WAVES 8
#define FQS16_FUSED_MAX_M 6                               // rows up to which quantising inside the GEMM kernel pays (<= waves)
#define FQS16_OOB 0xFFFFFF00u                             // beyond any 32-bit buffer size
// byte `i` (0..3, compile-time) of a word of E4M3 codes -> float
__device__ __forceinline__ float fq_e4m3_byte_to_float(unsigned w, int i) {
    return i == 0 ? __builtin_amdgcn_cvt_f32_fp8((int)w, 0) : i == 1 ? __builtin_amdgcn_cvt_f32_fp8((int)w, 1)
         : i == 2 ? __builtin_amdgcn_cvt_f32_fp8((int)w, 2) : __builtin_amdgcn_cvt_f32_fp8((int)w, 3);
}
#define FQ_MFMA16(a, b, c) __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4((a), (b), (c), 0, 0, 0, 0, 0, 0)

// The four scale bytes of a channel that go with four consecutive slots are fetched as words.
// WORDS: every wave's slice starts at a multiple of 4 groups and the scale rows are word-aligned, so
// they are one aligned word; otherwise the two aligned words around them are fetched and shifted
// into place when they are used.
// A wave keeps a ring of BATCH groups in flight (4, 8 or 12: the shortest that holds a wave's slice,
// at most 48 bytes of packed weights per lane): it requests the first BATCH groups of its slice at
// once and re-requests each slot, for the group BATCH further on, as soon as it has used it.  Loads
// return in order, so the ring is consumed in the order it was requested.
template <int NSUB, bool WORDS, int BATCH_>
struct fqs16_ring {
    static constexpr int BATCH = BATCH_;
    static_assert(BATCH % 4 == 0, "scale words cover four slots");
    fq_v4i bq[BATCH][NSUB];
    fq_v4i aq[BATCH][2];
    unsigned sq[BATCH / 4][NSUB][WORDS ? 1 : 2];          // scale words of four slots

    // request group g into slot i; groups at or past g_end request nothing and read as zeros
    // (LOAD_A = false: the activations of the slot come from elsewhere)
    template <bool LOAD_A = true>
    __device__ __forceinline__ void issue(int i, __amdgpu_buffer_rsrc_t rsA, __amdgpu_buffer_rsrc_t rsW,
                                          __amdgpu_buffer_rsrc_t rsG, unsigned aoff, const unsigned (&woff)[NSUB],
                                          const unsigned (&goff)[NSUB], int g, int g_end) {
        const unsigned dead = g < g_end ? 0u : FQS16_OOB;
        if (i % 4 == 0) {
#pragma unroll
            for (int j = 0; j < NSUB; ++j) {
                if (WORDS) {
                    sq[i / 4][j][0] = __builtin_amdgcn_raw_buffer_load_b32(rsG, goff[j] | dead, g, 0);
                } else {
                    const unsigned base = ((goff[j] + (unsigned)g) & ~3u) | dead;
                    sq[i / 4][j][0] = __builtin_amdgcn_raw_buffer_load_b32(rsG, base, 0, 0);
                    sq[i / 4][j][WORDS ? 0 : 1] = __builtin_amdgcn_raw_buffer_load_b32(rsG, base, 4, 0);
                }
            }
        }
        if (LOAD_A) {
            aq[i][0] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsA, aoff | dead, g * FQ_GROUP, 0));
            aq[i][1] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsA, (aoff + 16u) | dead, g * FQ_GROUP, 0));
        }
#pragma unroll
        for (int j = 0; j < NSUB; ++j)                    // streamed once: non-temporal
            bq[i][j] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsW, woff[j] | dead, g * 2048, 2));
    }

    // the scale word of slots i .. i + 3 (i a multiple of 4) of sub-tile j, whose first slot holds group g
    __device__ __forceinline__ unsigned scale_word(int i, int j, unsigned goff_j, int g) const {
        if (WORDS) return sq[i / 4][j][0];
        return __builtin_amdgcn_alignbyte(sq[i / 4][j][WORDS ? 0 : 1], sq[i / 4][j][0], (goff_j + (unsigned)g) & 3u);
    }

    // slot i -> accumulators (a dead group is all zeros and adds nothing: `live` also keeps whatever
    // byte sits where its scale would be out of the sum); `sw` is the slot's scale word, read before
    // the slot group's first slot may be re-requested
    __device__ __forceinline__ void compute(int i, fq_v4f (&acc)[NSUB], const unsigned (&sw)[NSUB], bool live) const {
        const fq_v4f zero4 = {0.f, 0.f, 0.f, 0.f};
        const fq_v8i a = fqs_join(aq[i][0], aq[i][1]);
        fq_v8i zp;
#pragma unroll
        for (int r = 0; r < 8; ++r) zp[r] = (int)FQ_ZP_BYTES;
        const fq_v4f c0 = FQ_MFMA16(a, zp, zero4);        // zero point: -2^-6 * sum_k a_k in every column
#pragma unroll
        for (int j = 0; j < NSUB; ++j) {
            const fq_v8i b = fq_unpack_chunk(bq[i][j]);
            // (WORDS: a dead slot's word was not fetched at all and reads as zero)
            const float s = (WORDS || live) ? fq_e4m3_byte_to_float(sw[j], i % 4) : 0.f;
            const fq_v4f p = FQ_MFMA16(a, b, c0);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[j][r] = fmaf(s, p[r], acc[j][r]);
        }
    }
};

// FUSEDQ (M <= 6, K <= 4096): `A` holds the bf16 activations X [M,K] instead of E4M3 codes, and the
// kernel quantises them itself (Sec. 2.1 eq. 2, the arithmetic of the quantiser kernel): wave w reads
// row w of X whole (coalesced 16-byte loads into registers), takes its maximum, converts it and
// leaves the codes in LDS ([M rows][K + 16 bytes]: the pad spreads the rows over the banks); after one
// barrier every wave fetches the operands of its K slice from there.  All of that happens while the
// weights are on their way.  Every workgroup repeats it for all of X, which for a few rows costs
// less than a second kernel (measured at N = 14336, K = 4096: 8.4 against 10.0 us at M = 1, 8.8 against
// 10.1 at M = 4, 10.5 against 10.3 at M = 8: the conversion is some ten instructions per element, on
// every compute unit).  `a_scale` is not read;
// `a_scale_out` (may be NULL) receives the row scales.  Dynamic LDS: 8 * (K + 16) bytes.
template <int NSUB, bool WORDS, bool ROUNDS, int BATCH_, bool FUSEDQ = false>
__global__ __launch_bounds__(FQS16_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void fq_gemm_small16_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* Y, int M, int N, int K, int cols,
    int swiglu, const uint16_t* R, float* __restrict__ a_scale_out) {
    static_assert(!(FUSEDQ && ROUNDS), "the fused form serves K <= 4096: a slice is at most four groups");
    typedef fqs16_ring<NSUB, WORDS, BATCH_> ring_t;
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
        const_cast<uint8_t*>(A), 0, (int)((unsigned)M * (unsigned)K * (FUSEDQ ? 2u : 1u)), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(wp), 0, (int)((unsigned)((N + 31) >> 5) * (unsigned)G * 2048u), 0x00020000);
    // (range rounded up to whole words, so that the array's last word is readable when it holds fewer
    // than four scales; the array is 16-byte aligned and the surplus bytes never enter a sum)
    const __amdgpu_buffer_rsrc_t rsG = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(gs), 0, (int)(((unsigned)N * (unsigned)G + 3u) & ~3u), 0x00020000);
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
    if (!FUSEDQ) {
#pragma unroll
        for (int i = 0; i < NOUT; ++i) {
            const int idx = threadIdx.x + i * FQS16_THREADS;
            const int m = 4 * ((idx & 63) >> 4) + ((idx >> 6) & 3);
            osc[i] = a_scale[m < M ? m : M - 1];
        }
    }

    fq_v4f acc[NSUB];
#pragma unroll
    for (int j = 0; j < NSUB; ++j) acc[j] = (fq_v4f){0.f, 0.f, 0.f, 0.f};

    ring_t ring;
    extern __shared__ __attribute__((aligned(16))) uint8_t codes[];   // FUSEDQ: [8][K + 16] E4M3 codes
    __shared__ float srow[FQS16_WAVES];                   // FUSEDQ: row scales
    constexpr int XCH = 8;                                // 16-byte chunks of a row per lane: K <= 4096
    fq_v4i xr[FUSEDQ ? XCH : 1];
    const bool my_row = FUSEDQ && wave < M;               // wave w quantises row w (M <= 6 < number of waves)
    if (FUSEDQ) {                                         // first in the queue: they are needed first
#pragma unroll
        for (int c = 0; c < XCH; ++c) {
            const int chunk = lane + 64 * c;
            const unsigned off = (my_row && chunk < (K >> 3)) ? ((unsigned)wave * (unsigned)K * 2u + (unsigned)chunk * 16u) : FQS16_OOB;
            xr[c] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsA, off, 0, 0));
        }
    }
#pragma unroll
    for (int i = 0; i < BATCH; ++i) ring.template issue<!FUSEDQ>(i, rsA, rsW, rsG, aoff, woff, goff, g_begin + i, g_end);
    __builtin_amdgcn_sched_barrier(0);                    // all requests go out before any arithmetic
    if (FUSEDQ) {
        const int stride = K + 16;
        if (my_row) {
            float amax = 0.f;
#pragma unroll
            for (int c = 0; c < XCH; ++c)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const unsigned w = (unsigned)xr[c][e];
                    amax = fmaxf(amax, fmaxf(fabsf(fq_bf16_lo(w)), fabsf(fq_bf16_hi(w))));
                }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
            const float s = amax == 0.f ? 1.0f : amax / 448.0f;   // the quantiser's scale (an all-zero row: 1)
            const float rcp = 1.0f / s;
            if (lane == 0) {
                srow[wave] = s;
                if (a_scale_out != nullptr && blockIdx.x == 0) a_scale_out[wave] = s;
            }
            // one choice of quotient per row (s is the same in every lane), then straight-line code
            auto convert = [&](auto fast_tag) __attribute__((always_inline)) {
                constexpr bool FAST = decltype(fast_tag)::value;
#pragma unroll
                for (int c = 0; c < XCH; ++c) {
                    const int chunk = lane + 64 * c;
                    if (chunk < (K >> 3))
                        *reinterpret_cast<fq_v2i*>(codes + wave * stride + chunk * 8) = fq_quant8<FAST>(xr[c], s, rcp);
                }
            };
            if (__builtin_amdgcn_readfirstlane((int)fq_scale_is_fast(s))) convert(std::true_type());
            else convert(std::false_type());
        }
        __syncthreads();
        // operands of this wave's slice: row r16 (rows past M repeat the last one, as the unfused form does)
        const uint8_t* arow = codes + (r16 < M ? r16 : M - 1) * stride + kq * 32;
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const int g = g_begin + i;
            if (g < g_end) {
                ring.aq[i][0] = *reinterpret_cast<const fq_v4i*>(arow + g * FQ_GROUP);
                ring.aq[i][1] = *reinterpret_cast<const fq_v4i*>(arow + g * FQ_GROUP + 16);
            } else {
                ring.aq[i][0] = ring.aq[i][1] = (fq_v4i){0, 0, 0, 0};
            }
        }
#pragma unroll
        for (int i = 0; i < NOUT; ++i) {
            const int idx = threadIdx.x + i * FQS16_THREADS;
            const int m = 4 * ((idx & 63) >> 4) + ((idx >> 6) & 3);
            osc[i] = srow[m < M ? m : M - 1];
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    // ROUNDS == false: no slice is longer than BATCH groups, the ring is used once and never refilled
    for (int gb = g_begin; gb < g_end; gb += BATCH) {
        unsigned sw[NSUB];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            if (i % 4 == 0) {                             // keep the word: its slot may be re-requested below
#pragma unroll
                for (int j = 0; j < NSUB; ++j) sw[j] = ring.scale_word(i, j, goff[j], gb + i);
            }
            ring.compute(i, acc, sw, gb + i < g_end);
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
            float v = 0.f, vu = 0.f;
#pragma unroll
            for (int w = 0; w < FQS16_WAVES; ++w) v += red[w][j][r][l];
            if (swiglu) {                                 // the up channel of an even (gate) channel
#pragma unroll
                for (int w = 0; w < FQS16_WAVES; ++w) vu += red[w][j][r][l | 1];
            }
            const int m = 4 * (l >> 4) + r;
            const int c = 16 * j + (l & 15);
            const int n = n_first + c;
            if (m < M && c < cols && n < N) {
                const float f = osc[i] * outer;
                if (!swiglu) {
                    fq_v2f pr = {v * f, 0.f};
                    if (R) pr[0] = fmaf(v, f, __uint_as_float((unsigned)R[(size_t)m * N + n] << 16));   // residual, one rounding
                    fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
                    Y[(size_t)m * N + n] = __builtin_bit_cast(unsigned short, pk[0]);
                } else if ((l & 1) == 0) {                // fused epilogue: H[m, n/2] = SiLU(gate) * up
                    fq_v2f pr = {fq_silu_mul(v * f, vu * f), 0.f};
                    fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
                    Y[(size_t)m * (N >> 1) + (n >> 1)] = __builtin_bit_cast(unsigned short, pk[0]);
                }
            }
        }
    }
}

namespace {

template <int NSUB, bool WORDS, int BATCH>
void fq_launch_small16b(bool rounds, unsigned grid, hipStream_t stream, const uint8_t* A, const float* a_scale,
                        const uint8_t* wp, const uint8_t* gs, float tscale, uint16_t* Y, int M, int N, int K, int cols, int swiglu, const uint16_t* R) {
    if (rounds)
        hipLaunchKernelGGL((fq_gemm_small16_kernel<NSUB, WORDS, true, BATCH>), dim3(grid), dim3(FQS16_THREADS), 0, stream,
                           A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R, static_cast<float*>(nullptr));
    else
        hipLaunchKernelGGL((fq_gemm_small16_kernel<NSUB, WORDS, false, BATCH>), dim3(grid), dim3(FQS16_THREADS), 0, stream,
                           A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R, static_cast<float*>(nullptr));
}

// The fused form (bf16 activations in, quantised by the kernel): slices of at most four groups per wave
// (K <= 4096), for which a slice of X fits into registers beside the ring.
template <int NSUB, bool WORDS>
bool fq_launch_linear16w(int per, unsigned grid, hipStream_t stream, const uint16_t* X, float* a_scale_out,
                         const uint8_t* wp, const uint8_t* gs, float tscale, uint16_t* Y, int M, int N, int K, int cols) {
    if (per > 4) return false;
    const size_t lds = (size_t)8 * (size_t)(K + 16);      // the codes of X
    static fq_device_once attr_once;                       // (one per template instance)
    fq_once_per_device(attr_once, [] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fq_gemm_small16_kernel<NSUB, WORDS, false, 4, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 8 * (4096 + 16));
    });
    hipLaunchKernelGGL((fq_gemm_small16_kernel<NSUB, WORDS, false, 4, true>), dim3(grid), dim3(FQS16_THREADS), lds, stream,
                       reinterpret_cast<const uint8_t*>(X), static_cast<const float*>(nullptr), wp, gs, tscale, Y, M, N, K, cols,
                       0, static_cast<const uint16_t*>(nullptr), a_scale_out);
    return true;
}

// Ring depth: the shortest of 4, 8, 12 that holds a wave's slice of `per` groups, at most 12 / 8 / 4
// groups for 1 / 2 / 3-4 sub-tiles (registers); longer slices go round the ring (ROUNDS).
template <int NSUB, bool WORDS>
void fq_launch_small16w(int per, unsigned grid, hipStream_t stream, const uint8_t* A, const float* a_scale,
                        const uint8_t* wp, const uint8_t* gs, float tscale, uint16_t* Y, int M, int N, int K, int cols, int swiglu, const uint16_t* R) {
    constexpr int CAP = NSUB == 1 ? 12 : (NSUB == 2 ? 8 : 4);
    if (CAP >= 12 && per > 8)
        fq_launch_small16b<NSUB, WORDS, CAP >= 12 ? 12 : CAP>(per > 12, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
    else if (CAP >= 8 && per > 4)
        fq_launch_small16b<NSUB, WORDS, CAP >= 8 ? 8 : CAP>(per > 8, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
    else
        fq_launch_small16b<NSUB, WORDS, 4>(per > 4, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
}

template <int NSUB>
void fq_launch_small16(bool words, int per, unsigned grid, hipStream_t stream, const uint8_t* A, const float* a_scale,
                       const uint8_t* wp, const uint8_t* gs, float tscale, uint16_t* Y, int M, int N, int K, int cols, int swiglu, const uint16_t* R) {
    if (words) fq_launch_small16w<NSUB, true>(per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
    else       fq_launch_small16w<NSUB, false>(per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// 16 < M <= 64, general form of the kernel above: MT <= 4 row tiles of 16 rows share every unpacked
// weight operand (the weights are still read from HBM once), and the group scales of the
// workgroup's channels (cols x K/128 bytes, contiguous in memory) are copied to LDS at the start
// instead of being fetched per group.
// ---------------------------------------------------------------------------------------------
#define FQSM_MAXCOLS 64

template <int MT, int NSUB>
struct fqsm_ring {
    static constexpr int BATCH = MT >= 3 ? 2 : (MT == 2 ? 4 : (NSUB <= 2 ? 8 : 4));
    fq_v4i bq[BATCH][NSUB];
    fq_v4i aq[BATCH][MT][2];

    // request group g into slot i; groups at or past g_end request nothing and read as zeros
    // (LOAD_A = false: the activations of the slot come from elsewhere)
    template <bool LOAD_A = true>
    __device__ __forceinline__ void issue(int i, __amdgpu_buffer_rsrc_t rsA, __amdgpu_buffer_rsrc_t rsW,
                                          const unsigned (&aoff)[MT], const unsigned (&woff)[NSUB], int g, int g_end) {
        const unsigned dead = g < g_end ? 0u : FQS16_OOB;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            aq[i][t][0] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsA, aoff[t] | dead, g * FQ_GROUP, 0));
            aq[i][t][1] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsA, (aoff[t] + 16u) | dead, g * FQ_GROUP, 0));
        }
#pragma unroll
        for (int j = 0; j < NSUB; ++j)                    // streamed once: non-temporal
            bq[i][j] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsW, woff[j] | dead, g * 2048, 2));
    }

    // slot i (group g) -> accumulators; a dead group is all zeros and adds nothing.  `sc` points at
    // this lane's first channel in the LDS scale table [group][64 channels].
    __device__ __forceinline__ void compute(int i, fq_v4f (&acc)[MT][NSUB], const uint8_t* sc, int g) const {
        const fq_v4f zero4 = {0.f, 0.f, 0.f, 0.f};
        fq_v8i zp;
#pragma unroll
        for (int r = 0; r < 8; ++r) zp[r] = (int)FQ_ZP_BYTES;
        fq_v8i a[MT];
        fq_v4f c0[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            a[t] = fqs_join(aq[i][t][0], aq[i][t][1]);
            c0[t] = FQ_MFMA16(a[t], zp, zero4);           // zero point: -2^-6 * sum_k a_k in every column
        }
        const uint8_t* scg = sc + g * FQSM_MAXCOLS;
#pragma unroll
        for (int j = 0; j < NSUB; ++j) {
            const fq_v8i b = fq_unpack_chunk(bq[i][j]);
            const float s = __builtin_amdgcn_cvt_f32_fp8((int)scg[16 * j], 0);
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const fq_v4f p = FQ_MFMA16(a[t], b, c0[t]);
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[t][j][r] = fmaf(s, p[r], acc[t][j][r]);
            }
        }
    }
};

template <int MT, int NSUB, bool ROUNDS>
__global__ __launch_bounds__(FQS16_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void fq_gemm_smallm_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* Y, int M, int N, int K, int cols,
    int swiglu, const uint16_t* R) {
    typedef fqsm_ring<MT, NSUB> ring_t;
    constexpr int BATCH = ring_t::BATCH;
    // LDS: first the scale table [G][64] bytes, later (after a barrier) the partial sums
    // [wave][row tile][sub-tile][reg][lane] floats
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    float* red = reinterpret_cast<float*>(smem);
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
    // the scale bytes of this workgroup: (channel c, group g) at gs[(n_first + c) * G + g]; up to 8 per thread now,
    // the rest (K > 8192) after the ring has been requested.  Where rows of scales are whole words (K a multiple of
    // 512) a thread fetches words, two instead of eight loads ahead of the weights in the queue: a load costs the
    // address path the same whatever its width.
    const int nsc = FQSM_MAXCOLS * G;
    const bool scw = (G & 3) == 0;
    unsigned scb[8];
    if (scw) {
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const int idx = 4 * (threadIdx.x + x * FQS16_THREADS);    // idx = c * G + g
            const int c = idx / G;
            const bool on = idx < nsc && c < cols && n_first + c < N;
            scb[x] = __builtin_amdgcn_raw_buffer_load_b32(rsG, on ? (unsigned)(n_first * G + idx) : FQS16_OOB, 0, 0);
        }
    } else {
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int idx = threadIdx.x + x * FQS16_THREADS;
            const int c = idx / G;
            const bool on = idx < nsc && c < cols && n_first + c < N;
            scb[x] = __builtin_amdgcn_raw_buffer_load_b8(rsG, on ? (unsigned)(n_first * G + idx) : FQS16_OOB, 0, 0);
        }
    }
    // per sub-tile: byte offset of this lane's chunk in group 0 of its packed block
    unsigned woff[NSUB];
#pragma unroll
    for (int j = 0; j < NSUB; ++j) {
        const int c = 16 * j + r16;
        const int n = n_first + c;
        const bool on = (c < cols) && (n < N);            // masked lanes request nothing and store nothing
        woff[j] = on ? (unsigned)(n >> 5) * (unsigned)G * 2048u + (unsigned)(kq >> 1) * 1024u +
                       (unsigned)((kq & 1) * 32 + (n & 31)) * 16u
                     : FQS16_OOB;
    }
    unsigned aoff[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = 16 * t + r16;
        aoff[t] = (unsigned)(m < M ? m : M - 1) * (unsigned)K + (unsigned)kq * 32u;
    }
    // output factors of the elements this thread writes at the end, fetched up front
    constexpr int NOUT = (MT * NSUB * 256 + FQS16_THREADS - 1) / FQS16_THREADS;
    float osc[NOUT];
#pragma unroll
    for (int i = 0; i < NOUT; ++i) {
        const int idx = threadIdx.x + i * FQS16_THREADS;
        const int m = 16 * (idx / (256 * NSUB)) + 4 * ((idx & 63) >> 4) + ((idx >> 6) & 3);
        osc[i] = a_scale[m < M ? m : M - 1];
    }

    fq_v4f acc[MT][NSUB];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int j = 0; j < NSUB; ++j) acc[t][j] = (fq_v4f){0.f, 0.f, 0.f, 0.f};

    ring_t ring;
#pragma unroll
    for (int i = 0; i < BATCH; ++i) ring.issue(i, rsA, rsW, aoff, woff, g_begin + i, g_end);
    __builtin_amdgcn_sched_barrier(0);                    // all requests go out before anything else
    // scale table: transposed to [group][channel] so that a lane's sub-tiles are 16 bytes apart
    if (scw) {
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const int idx = 4 * (threadIdx.x + x * FQS16_THREADS);
            const int c = idx / G, g = idx - c * G;       // (G % 4 == 0: the word's four groups belong to one channel)
            if (idx < nsc) {
#pragma unroll
                for (int e = 0; e < 4; ++e) smem[(g + e) * FQSM_MAXCOLS + c] = (uint8_t)(scb[x] >> (8 * e));
            }
        }
        for (int idx = 4 * (threadIdx.x + 2 * FQS16_THREADS); idx < nsc; idx += 4 * FQS16_THREADS) {
            const int c = idx / G, g = idx - c * G;
            const bool on = c < cols && n_first + c < N;
            const unsigned w = __builtin_amdgcn_raw_buffer_load_b32(rsG, on ? (unsigned)(n_first * G + idx) : FQS16_OOB, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) smem[(g + e) * FQSM_MAXCOLS + c] = (uint8_t)(w >> (8 * e));
        }
    } else {
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int idx = threadIdx.x + x * FQS16_THREADS;
            const int c = idx / G, g = idx - c * G;
            if (idx < nsc) smem[g * FQSM_MAXCOLS + c] = (uint8_t)scb[x];
        }
        for (int idx = threadIdx.x + 8 * FQS16_THREADS; idx < nsc; idx += FQS16_THREADS) {
            const int c = idx / G, g = idx - c * G;
            const bool on = c < cols && n_first + c < N;
            smem[g * FQSM_MAXCOLS + c] = (uint8_t)__builtin_amdgcn_raw_buffer_load_b8(
                rsG, on ? (unsigned)(n_first * G + idx) : FQS16_OOB, 0, 0);
        }
    }
    __syncthreads();
    const uint8_t* sc = smem + r16;
    // ROUNDS == false: no slice is longer than BATCH groups, the ring is used once and never refilled
    for (int gb = g_begin; gb < g_end; gb += BATCH) {
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const int g = gb + i < G ? gb + i : G - 1;    // (a dead slot may read any scale: its sums are zero)
            ring.compute(i, acc, sc, g);
            __builtin_amdgcn_sched_barrier(0);            // slot by slot, as the data lands
            if (ROUNDS) {
                ring.issue(i, rsA, rsW, aoff, woff, gb + BATCH + i, g_end);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (!ROUNDS) break;
    }

    // ---- sum the K-slices of the 8 waves through LDS (over the scale table), scale, write bf16 ----
    __syncthreads();                                      // every wave is done with the scale table
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int j = 0; j < NSUB; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[(((wave * MT + t) * NSUB + j) * 4 + r) * 64 + lane] = acc[t][j][r];
    __syncthreads();
    const float outer = tscale * 512.0f;                  // weights were fed in units of 2^-9
#pragma unroll
    for (int i = 0; i < NOUT; ++i) {
        const int idx = threadIdx.x + i * FQS16_THREADS;  // MT * NSUB * 256 outputs: [row tile][sub-tile][reg][lane]
        const int l = idx & 63, r = (idx >> 6) & 3, j = (idx >> 8) % NSUB, t = idx / (256 * NSUB);
        if (t < MT) {
            float v = 0.f, vu = 0.f;
#pragma unroll
            for (int w = 0; w < FQS16_WAVES; ++w) v += red[w * (MT * NSUB * 256) + idx];
            if (swiglu) {                                 // the up channel of an even (gate) channel
#pragma unroll
                for (int w = 0; w < FQS16_WAVES; ++w) vu += red[w * (MT * NSUB * 256) + (idx | 1)];
            }
            const int m = 16 * t + 4 * (l >> 4) + r;
            const int c = 16 * j + (l & 15);
            const int n = n_first + c;
            if (m < M && c < cols && n < N) {
                const float f = osc[i] * outer;
                if (!swiglu) {
                    fq_v2f pr = {v * f, 0.f};
                    if (R) pr[0] = fmaf(v, f, __uint_as_float((unsigned)R[(size_t)m * N + n] << 16));   // residual, one rounding
                    fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
                    Y[(size_t)m * N + n] = __builtin_bit_cast(unsigned short, pk[0]);
                } else if ((l & 1) == 0) {                // fused epilogue: H[m, n/2] = SiLU(gate) * up
                    fq_v2f pr = {fq_silu_mul(v * f, vu * f), 0.f};
                    fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
                    Y[(size_t)m * (N >> 1) + (n >> 1)] = __builtin_bit_cast(unsigned short, pk[0]);
                }
            }
        }
    }
}

namespace {

template <int MT, int NSUB>
bool fq_launch_smallm(int per, unsigned grid, hipStream_t stream, const uint8_t* A, const float* a_scale,
                      const uint8_t* wp, const uint8_t* gs, float tscale, uint16_t* Y, int M, int N, int K, int cols, int swiglu, const uint16_t* R) {
    const int G = K / FQ_GROUP;
    const size_t red_bytes = (size_t)FQS16_WAVES * MT * NSUB * 256 * sizeof(float);
    const size_t sc_bytes = (size_t)FQSM_MAXCOLS * G;
    const size_t lds = red_bytes > sc_bytes ? red_bytes : sc_bytes;
    if (lds > 160 * 1024) return false;
    const bool rounds = per > fqsm_ring<MT, NSUB>::BATCH;
    const void* fn = rounds ? reinterpret_cast<const void*>(fq_gemm_smallm_kernel<MT, NSUB, true>)
                            : reinterpret_cast<const void*>(fq_gemm_smallm_kernel<MT, NSUB, false>);
    if (lds > 64 * 1024) (void)hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (rounds)
        hipLaunchKernelGGL((fq_gemm_smallm_kernel<MT, NSUB, true>), dim3(grid), dim3(FQS16_THREADS), lds, stream,
                           A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
    else
        hipLaunchKernelGGL((fq_gemm_smallm_kernel<MT, NSUB, false>), dim3(grid), dim3(FQS16_THREADS), lds, stream,
                           A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
    return true;
}

template <int MT>
bool fq_launch_smallm_mt(int nsub, int per, unsigned grid, hipStream_t stream, const uint8_t* A, const float* a_scale,
                         const uint8_t* wp, const uint8_t* gs, float tscale, uint16_t* Y, int M, int N, int K, int cols, int swiglu, const uint16_t* R) {
    switch (nsub) {
        case 1: return fq_launch_smallm<MT, 1>(per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
        case 2: return fq_launch_smallm<MT, 2>(per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
        case 3: return fq_launch_smallm<MT, 3>(per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
        default: return fq_launch_smallm<MT, 4>(per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
    }
}

}  // namespace

namespace {

// How a small-M problem is cut up: channels per workgroup (an even share of N over the compute units,
// a multiple of 8, at most 64), workgroups, groups per wave, sub-tiles of 16 channels, and whether the
// scale bytes of four consecutive groups are one aligned word.
struct fqs_shape {
    int cols;
    unsigned grid;
    int per, nsub;
    bool words;
};

fqs_shape fqs_shape_of(int N, int K, const uint8_t* gs) {
    const int cus = fq_device_cus();
    fqs_shape sh;
    sh.cols = ((N + cus - 1) / cus + 7) & ~7;
    sh.cols = sh.cols < 8 ? 8 : (sh.cols > 64 ? 64 : sh.cols);
    sh.grid = (unsigned)((N + sh.cols - 1) / sh.cols);
    const int G = K / FQ_GROUP;
    sh.per = (G + FQS16_WAVES - 1) / FQS16_WAVES;
    sh.nsub = (sh.cols + 15) / 16;
    sh.words = (sh.per % 4 == 0) && (G % 4 == 0) && ((reinterpret_cast<uintptr_t>(gs) & 3) == 0);
    return sh;
}

}  // namespace

bool fq_linear_small_serves(int M, int K) {
    return M >= 1 && M <= FQS16_FUSED_MAX_M && (K / FQ_GROUP + FQS16_WAVES - 1) / FQS16_WAVES <= 4;
}

bool fq_launch_linear_small(const uint16_t* X, float* a_scale_out, const uint8_t* wp, const uint8_t* gs, float tscale,
                            uint16_t* Y, int M, int N, int K, hipStream_t stream) {
    if (!fq_linear_small_serves(M, K)) return false;
    const fqs_shape sh = fqs_shape_of(N, K, gs);
    switch (2 * sh.nsub + (sh.words ? 1 : 0)) {
        case 2: return fq_launch_linear16w<1, false>(sh.per, sh.grid, stream, X, a_scale_out, wp, gs, tscale, Y, M, N, K, sh.cols);
        case 3: return fq_launch_linear16w<1, true>(sh.per, sh.grid, stream, X, a_scale_out, wp, gs, tscale, Y, M, N, K, sh.cols);
        case 4: return fq_launch_linear16w<2, false>(sh.per, sh.grid, stream, X, a_scale_out, wp, gs, tscale, Y, M, N, K, sh.cols);
        case 5: return fq_launch_linear16w<2, true>(sh.per, sh.grid, stream, X, a_scale_out, wp, gs, tscale, Y, M, N, K, sh.cols);
        case 6: return fq_launch_linear16w<3, false>(sh.per, sh.grid, stream, X, a_scale_out, wp, gs, tscale, Y, M, N, K, sh.cols);
        case 7: return fq_launch_linear16w<3, true>(sh.per, sh.grid, stream, X, a_scale_out, wp, gs, tscale, Y, M, N, K, sh.cols);
        case 8: return fq_launch_linear16w<4, false>(sh.per, sh.grid, stream, X, a_scale_out, wp, gs, tscale, Y, M, N, K, sh.cols);
        default: return fq_launch_linear16w<4, true>(sh.per, sh.grid, stream, X, a_scale_out, wp, gs, tscale, Y, M, N, K, sh.cols);
    }
}

bool fq_launch_gemm_small(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                          float tscale, uint16_t* Y, int M, int N, int K, bool swiglu_epilogue, const uint16_t* R, hipStream_t stream) {
    const int swiglu = swiglu_epilogue ? 1 : 0;
    const fqs_shape sh = fqs_shape_of(N, K, gs);
    const int cols = sh.cols, per = sh.per, nsub = sh.nsub;
    const unsigned grid = sh.grid;
    if (M <= 16) {
        const bool words = sh.words;
        switch (nsub) {
            case 1: fq_launch_small16<1>(words, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R); break;
            case 2: fq_launch_small16<2>(words, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R); break;
            case 3: fq_launch_small16<3>(words, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R); break;
            default: fq_launch_small16<4>(words, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R); break;
        }
        return true;
    }
    if (M > 64) return false;
    switch ((M + 15) / 16) {                              // false: the scale table does not fit LDS (K > 300000)
        case 2: return fq_launch_smallm_mt<2>(nsub, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
        case 3: return fq_launch_smallm_mt<3>(nsub, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
        default: return fq_launch_smallm_mt<4>(nsub, per, grid, stream, A, a_scale, wp, gs, tscale, Y, M, N, K, cols, swiglu, R);
    }
}
