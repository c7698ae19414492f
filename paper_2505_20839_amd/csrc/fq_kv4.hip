// Attention operands with an INT4 key/value cache and FP8 queries (Sec. 3.2.1: queries FP8, keys and
// values INT4 with one scaling factor per token; Sec. 2.1: those factors are FP8; Sec. 3.1.1: the
// INT4 x FP8 product also forms S = Q K^T and O = P V).  Heads are 128 wide, so one token of one head is
// exactly one quantisation group, and both caches are kept in the packed layout of the linear layers
// (fq_common.h), one matrix per head:
//     keys    N = tokens (padded to 32), K = 128 head dimensions   (one group per token)
//     values  N = 128 head dimensions,   K = tokens (padded to 128, padding = code of q = 0)
// so that in both products the contraction index runs along the 32 consecutive codes a lane holds.
//
// Scores: the M <= 16 GEMM's arithmetic with a single group -- unpack to E4M3 (mask and shift; the
// zero point of 8 comes out again through one more MFMA against a constant operand, computed once per
// query tile), v_mfma_f32_16x16x128_f8f6f4, and the token's scale applied in FP32 to the finished sum.
// Output: the token's scale sits on the contraction index, so it cannot multiply a finished sum.  It is
// applied exactly all the same: P[r,t] * sigma[t] has at most 8 significant bits and q at most 4, both
// are exact bf16 numbers, and v_mfma_f32_16x16x32_bf16 forms exact products and adds them in FP32.
#include "fq_common.h"
#include "fq_kernels.h"

#define FQK_HEAD 128
#define FQK_OOB 0xFFFFFF00u

namespace {

typedef __bf16 fqk_v8bf __attribute__((ext_vector_type(8)));

// packed-cache bytes of one head
__host__ __device__ inline size_t fqk_key_bytes(int T) { return (size_t)((T + 31) / 32) * 32u * (FQK_HEAD / 2); }
__host__ __device__ inline size_t fqk_value_bytes(int T) { return (size_t)FQK_HEAD * (size_t)((T + 127) / 128 * 128) / 2u; }

// One thread per packed byte.  VALUES = false: weight matrix row n = token, column k = dimension;
// VALUES = true: row n = dimension, column k = token (tokens past T hold q = 0).
template <bool VALUES>
__global__ __launch_bounds__(256) void fqk_pack_kernel(const int8_t* __restrict__ codes, uint8_t* __restrict__ packed,
                                                       int T, size_t per_head) {
    const size_t idx = (size_t)blockIdx.x * 256u + threadIdx.x;
    if (idx >= per_head) return;
    const int h = blockIdx.y;
    const int8_t* src = codes + (size_t)h * T * FQK_HEAD;
    const int G = VALUES ? (T + 127) / 128 : 1;
    const size_t blk = idx >> 11;
    const int in = (int)(idx & 2047u);
    const int nt = (int)(blk / (size_t)G), g = (int)(blk % (size_t)G);
    const int hh = in >> 10, lane = (in >> 4) & 63, ij = in & 15;
    const int n = nt * 32 + (lane & 31);
    const int k_lo = g * FQ_GROUP + 64 * hh + 32 * (lane >> 5) + ij, k_hi = k_lo + 16;
    unsigned lo = VALUES ? 8 : 0, hi = lo;                // padding: q = 0 along the sum over tokens; keys as fq_pack_weights pads
    if (VALUES) {                                         // n = dimension (always < 128), k = token
        if (k_lo < T) lo = fq_code_from_q(src[(size_t)k_lo * FQK_HEAD + n]);
        if (k_hi < T) hi = fq_code_from_q(src[(size_t)k_hi * FQK_HEAD + n]);
    } else if (n < T) {                                   // n = token, k = dimension
        lo = fq_code_from_q(src[(size_t)n * FQK_HEAD + k_lo]);
        hi = fq_code_from_q(src[(size_t)n * FQK_HEAD + k_hi]);
    }
    packed[(size_t)h * per_head + idx] = (uint8_t)(lo | (hi << 4));
}

template <bool VALUES>
__global__ __launch_bounds__(256) void fqk_unpack_kernel(const uint8_t* __restrict__ packed, int8_t* __restrict__ codes,
                                                         int T, size_t per_head) {
    const size_t idx = (size_t)blockIdx.x * 256u + threadIdx.x;   // element (t, c) of the head
    if (idx >= (size_t)T * FQK_HEAD) return;
    const int h = blockIdx.y;
    const int t = (int)(idx / FQK_HEAD), c = (int)(idx % FQK_HEAD);
    int hi;
    const size_t off = VALUES ? fq_weight_byte(c, t, (T + 127) / 128, &hi) : fq_weight_byte(t, c, 1, &hi);
    const unsigned byte = packed[(size_t)h * per_head + off];
    codes[(size_t)h * T * FQK_HEAD + idx] = (int8_t)fq_q_from_code(hi ? (byte >> 4) : (byte & 0xFu));
}

#define FQ_MFMA16(a, b, c) __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4((a), (b), (c), 0, 0, 0, 0, 0, 0)

__device__ __forceinline__ fq_v8i fqk_join(fq_v4i lo, fq_v4i hi) {
    fq_v8i r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return r;
}

// ---- S = Q K^T ------------------------------------------------------------------------------------------
// grid (token chunks, heads); a workgroup of 4 waves covers 4 * NSUB * 16 tokens, wave w the sub-tiles
// w * NSUB .. of 16 tokens each.  Lane l = 16 * kq + r holds, of the A operand, dimensions 32 kq .. of query
// row r, and of the B operand the same dimensions of token r of the sub-tile: one 16-byte chunk of the
// packed cache.  MT row tiles of 16 queries share every unpacked operand.
// WIDE (T a multiple of 4, S 8-byte aligned): a lane ends up with 4 rows x 1 token; the four lanes of a quad hold the
// same rows of four neighbouring tokens, and a 4 x 4 transpose of bf16 pairs inside the quad (two DPP exchanges)
// leaves each lane with one row x four tokens = one 8-byte store instead of four 2-byte ones.
#define FQK_S_NSUB 4
template <int MT, bool WIDE>
__global__ __launch_bounds__(256) void fq_kv4_scores_kernel(
    const uint8_t* __restrict__ Q, const float* __restrict__ q_scale, const uint8_t* __restrict__ kp,
    const uint8_t* __restrict__ ks, float out_scale, uint16_t* __restrict__ S, int R, int T) {
    const int h = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r16 = lane & 15, kq = lane >> 4;
    const int t_first = (blockIdx.x * 4 + wave) * (FQK_S_NSUB * 16);
    if (t_first >= T) return;
    const size_t kbytes = fqk_key_bytes(T);
    const __amdgpu_buffer_rsrc_t rsK = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(kp) + (size_t)h * kbytes, 0, (int)kbytes, 0x00020000);
    // all of this wave's cache chunks are requested before anything else (streamed once: non-temporal)
    fq_v4i bq[FQK_S_NSUB];
    float sig[FQK_S_NSUB];
#pragma unroll
    for (int j = 0; j < FQK_S_NSUB; ++j) {
        const int t = t_first + 16 * j + r16;
        const unsigned off = t < T ? (unsigned)(t >> 5) * 2048u + (unsigned)(kq >> 1) * 1024u +
                                     (unsigned)((kq & 1) * 32 + (t & 31)) * 16u
                                   : FQK_OOB;
        bq[j] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsK, off, 0, 2));
    }
    // token scales: lane (kq, r) fetches the one of token r of sub-tile kq, and the four lanes with the same r pass
    // them round (one byte load per lane instead of four: a load costs the address path the same whatever its width)
    {
        const int t = t_first + 16 * kq + r16;
        const float own = t < T ? fq_e4m3_to_float(ks[(size_t)h * T + t]) : 0.f;
        static_assert(FQK_S_NSUB == 4, "one sub-tile per lane quarter");
#pragma unroll
        for (int j = 0; j < FQK_S_NSUB; ++j) sig[j] = __shfl(own, 16 * j + r16, 64);
    }
    fq_v8i a[MT];
    fq_v4f c0[MT];
    float rs[MT][4];
    fq_v8i zp;
#pragma unroll
    for (int r = 0; r < 8; ++r) zp[r] = (int)FQ_ZP_BYTES;
    const fq_v4f zero4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int row = 16 * m + r16;
        const fq_v4i* qrow = reinterpret_cast<const fq_v4i*>(Q + ((size_t)h * R + (row < R ? row : R - 1)) * FQK_HEAD + 32 * kq);
        a[m] = fqk_join(qrow[0], qrow[1]);
        c0[m] = FQ_MFMA16(a[m], zp, zero4);               // -2^-6 * sum_c Q[r, c] in every column
#pragma unroll
        for (int i = 0; i < 4; ++i) {                     // output rows of this lane: 16 m + 4 kq + i
            const int orow = 16 * m + 4 * kq + i;
            rs[m][i] = q_scale[(size_t)h * R + (orow < R ? orow : R - 1)] * (out_scale * 512.0f);   // codes were fed in units of 2^-9
        }
    }
#pragma unroll
    for (int j = 0; j < FQK_S_NSUB; ++j) {
        const fq_v8i b = fq_unpack_chunk(bq[j]);
        const int t = t_first + 16 * j + r16;             // this lane's output column
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const fq_v4f p = FQ_MFMA16(a[m], b, c0[m]);
            if (WIDE) {
                const fq_v2f pr0 = {(sig[j] * p[0]) * rs[m][0], (sig[j] * p[1]) * rs[m][1]};
                const fq_v2f pr1 = {(sig[j] * p[2]) * rs[m][2], (sig[j] * p[3]) * rs[m][3]};
                const unsigned pk0 = __builtin_bit_cast(unsigned, __builtin_convertvector(pr0, fq_v2bf));   // rows 0, 1
                const unsigned pk1 = __builtin_bit_cast(unsigned, __builtin_convertvector(pr1, fq_v2bf));   // rows 2, 3
                const bool oddl = lane & 1, upper = (lane & 2) != 0;
                const unsigned sel = oddl ? 0x03020706u : 0x05040100u;   // even: (own.lo, partner.lo); odd: (partner.hi, own.hi)
                const unsigned n0 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)pk0, 0xB1, 0xF, 0xF, false);
                const unsigned n1 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)pk1, 0xB1, 0xF, 0xF, false);
                const unsigned a0 = __builtin_amdgcn_perm(n0, pk0, sel);  // row 0 (even lane) / 1 (odd), the pair's two tokens
                const unsigned a1 = __builtin_amdgcn_perm(n1, pk1, sel);  // row 2 / 3
                const unsigned give = upper ? a0 : a1;
                const unsigned got = (unsigned)__builtin_amdgcn_update_dpp(0, (int)give, 0x4E, 0xF, 0xF, false);
                const fq_v2i out = upper ? (fq_v2i){(int)got, (int)a1} : (fq_v2i){(int)a0, (int)got};
                const int orow = 16 * m + 4 * kq + (lane & 3);            // the row this lane now holds, for tokens t4 .. t4 + 3
                const int t4 = t_first + 16 * j + (r16 & 12);
                if (orow < R && t4 < T)
                    *reinterpret_cast<fq_v2i*>(S + ((size_t)h * R + orow) * T + t4) = out;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int orow = 16 * m + 4 * kq + i;
                    if (orow < R && t < T) {
                        const fq_v2f pr = {(sig[j] * p[i]) * rs[m][i], 0.f};
                        const fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
                        S[((size_t)h * R + orow) * T + t] = __builtin_bit_cast(unsigned short, pk[0]);
                    }
                }
            }
        }
    }
}

// ---- O = P V --------------------------------------------------------------------------------------------
// A workgroup of 8 waves per head and slice of DT of the 8 dimension tiles (grid: heads x 8 / DT; fewer tiles per
// workgroup when there are few heads, so that the grid still covers the chip); wave w takes the 32-token blocks
// w, w + 8, ...; the partial results are added through LDS.  Per block: A' = bf16(P * sigma) for (16 query rows) x (32 tokens) -- lane
// l = 16 * kq + r holds tokens 8 kq .. 8 kq + 7 of row r -- and, for each of the 8 tiles of 16 dimensions,
// the B operand for (32 tokens) x (16 dimensions): lane l holds tokens 8 kq .. of dimension l % 16, which are
// 8 nibbles of one 16-byte chunk of the packed cache (chunk: 32 consecutive tokens of one dimension; low
// nibbles of bytes 0-7 are tokens 0-7, of bytes 8-15 tokens 8-15, the high nibbles tokens 16-31).
// A 4-bit code c = q + 8 becomes a bf16 number by bit operations alone: 0x4180 | c << 3 is 16 + c (the binade
// [16, 32) has a spacing of 1/8).  The matrix cores therefore sum A' * (q + 24); one more MFMA per block against
// an all-ones operand delivers sum A', and 24 times that is taken off at the end (all products are exact; the
// offset costs a few FP32 roundings of the larger intermediate sum, far below the tolerance).
// FAST: P rows and the scale rows are 8-byte aligned (ldp and T multiples of 8), so a lane's 8 codes are one
// 8-byte load each, converted by the hardware; otherwise byte loads.  (16-byte aligned rows take the kernel of
// 16-byte steps further down.)
#define FQK_O_WAVES 8
#ifndef FQK_O_FILL
#define FQK_O_FILL 2                                     // workgroups per compute unit the grid aims for
#endif
// the kernel of 16-byte steps: at most 4 dimension tiles per workgroup, and one workgroup per compute unit is enough
// (measured, 128-wide heads x 4 rows x 4096 tokens: 128 heads 10.0 us with 4 tiles, 11.0 with 2, 13.8 with 1; 256 heads
// 16.3 us with 4 tiles, 21.9 with 8)
#ifndef FQK_O_WIDE_FILL
#define FQK_O_WIDE_FILL 1
#endif
#ifndef FQK_O_WIDE_MAXDT
#define FQK_O_WIDE_MAXDT 4
#endif
#ifndef FQK_O_WIDE_PF
#define FQK_O_WIDE_PF(MT, DT) ((DT) <= 4)                // request a group ahead (registers allow it)
#endif
// The tail both output kernels share: the waves' partial sums (DT dimension tiles and the row sums of A') are added through
// LDS in the order of the waves, the offset of 24 per code comes off, the row's scale goes on, one rounding to bf16.
template <int MT, int DT>
__device__ __forceinline__ void fqk_output_finish(const fq_v4f (&acc)[MT][DT + 1], float* red, const float* __restrict__ p_scale,
                                                  uint16_t* __restrict__ O, int h, int d0, int R) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int d = 0; d < DT + 1; ++d)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[(((wave * MT + m) * (DT + 1) + d) * 4 + i) * 64 + lane] = acc[m][d][i];
    __syncthreads();
    for (int idx = threadIdx.x; idx < MT * DT * 4 * 64; idx += 64 * FQK_O_WAVES) {
        const int l = idx & 63, i = (idx >> 6) & 3, d = (idx >> 8) % DT, m = (idx >> 8) / DT;
        const int row = 16 * m + 4 * (l >> 4) + i, dim = 16 * (d0 + d) + (l & 15);
        if (row < R) {
            float v = 0.f, s1 = 0.f;                      // fixed order: deterministic
#pragma unroll
            for (int w = 0; w < FQK_O_WAVES; ++w) {
                v += red[(((w * MT + m) * (DT + 1) + d) * 4 + i) * 64 + l];
                s1 += red[(((w * MT + m) * (DT + 1) + DT) * 4 + i) * 64 + l];
            }
            const fq_v2f pr = {fmaf(-24.0f, s1, v) * p_scale[(size_t)h * R + row], 0.f};
            const fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
            O[((size_t)h * R + row) * FQK_HEAD + dim] = __builtin_bit_cast(unsigned short, pk[0]);
        }
    }
}

template <int MT, bool FAST, int DT, bool PF>
__global__ __launch_bounds__(64 * FQK_O_WAVES) void fq_kv4_output_kernel(
    const uint8_t* __restrict__ P, const float* __restrict__ p_scale, const uint8_t* __restrict__ vp,
    const uint8_t* __restrict__ vs, uint16_t* __restrict__ O, int R, int T, int ldp) {
    extern __shared__ float red[];                        // [waves][MT][DT + 1][4][64]: DT dimension tiles + the row sums
    const int d0 = blockIdx.y * DT;                       // first dimension tile of this workgroup
    const int h = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r16 = lane & 15, kq = lane >> 4;
    const int G = (T + 127) / 128;                        // 128-token groups of the packed value cache
    const size_t vbytes = fqk_value_bytes(T);
    const __amdgpu_buffer_rsrc_t rsV = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(vp) + (size_t)h * vbytes, 0, (int)vbytes, 0x00020000);
    fq_v4f acc[MT][DT + 1];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int d = 0; d < DT + 1; ++d) acc[m][d] = (fq_v4f){0.f, 0.f, 0.f, 0.f};
    fqk_v8bf ones;
#pragma unroll
    for (int j = 0; j < 8; ++j) ones[j] = __builtin_bit_cast(__bf16, (unsigned short)0x3F80);
    const int nblocks = (T + 31) / 32;
    // what a lane needs of one block, as it comes from memory: the DT dimension tiles' codes (8 bytes of chunk
    // (group blk / 4, half, kh, dimension)), and in FAST mode the 8 scale bytes and the 8 P codes of each row tile;
    // with PF (grids that leave compute units with a single workgroup or none: nothing else hides the latency) the
    // next block's are requested before the current one is worked on
    struct fqk_raw { fq_v2i vq[DT]; fq_v2i ws; fq_v2i wp[MT]; };
    auto fetch = [&](int blk, fqk_raw& raw) __attribute__((always_inline)) {
        const int t0 = 32 * blk + 8 * kq;
        const bool on = blk < nblocks;
#pragma unroll
        for (int d = 0; d < DT; ++d) {
            const int dim = 16 * (d0 + d) + r16;
            const int g = blk >> 2, hh = (blk >> 1) & 1, kh = blk & 1;
            const unsigned off = ((unsigned)(dim >> 5) * (unsigned)G + (unsigned)g) * 2048u + (unsigned)hh * 1024u +
                                 (unsigned)(kh * 32 + (dim & 31)) * 16u + (unsigned)(kq & 1) * 8u;
            raw.vq[d] = __builtin_bit_cast(fq_v2i, __builtin_amdgcn_raw_buffer_load_b64(rsV, on ? off : 0xFFFFFF00u, 0, 2));
        }
        if (FAST) {
            raw.ws = (fq_v2i){0, 0};
            if (on && t0 < T) raw.ws = *reinterpret_cast<const fq_v2i*>(vs + (size_t)h * T + t0);   // T % 8 == 0: all 8 or none
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const int row = 16 * m + r16;
                raw.wp[m] = (fq_v2i){0, 0};
                if (on && t0 < T)
                    raw.wp[m] = *reinterpret_cast<const fq_v2i*>(P + ((size_t)h * R + (row < R ? row : R - 1)) * ldp + t0);
            }
        }
    };
    fqk_raw cur, nxt;
    if (PF) fetch(wave, cur);
    for (int blk = wave; blk < nblocks; blk += FQK_O_WAVES) {
        const int t0 = 32 * blk + 8 * kq;                 // this lane's first token of the block
        if (PF) fetch(blk + FQK_O_WAVES, nxt);
        else    fetch(blk, cur);
        const fq_v2i* vq = cur.vq;
        // sigma of the lane's 8 tokens (zero past T), as FP32
        float sg[8];
        if (FAST) {
            const fq_v2i w = cur.ws;
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const fq_v2f lo = __builtin_amdgcn_cvt_pk_f32_fp8(w[x], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(w[x], true);
                sg[4 * x] = lo[0]; sg[4 * x + 1] = lo[1]; sg[4 * x + 2] = hi[0]; sg[4 * x + 3] = hi[1];
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) sg[j] = (t0 + j < T) ? fq_e4m3_to_float(vs[(size_t)h * T + t0 + j]) : 0.f;
        }
        fqk_v8bf a[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const int row = 16 * m + r16;
            const uint8_t* prow = P + ((size_t)h * R + (row < R ? row : R - 1)) * ldp + t0;
            float pv[8];
            if (FAST) {
                const fq_v2i w = cur.wp[m];
#pragma unroll
                for (int x = 0; x < 2; ++x) {
                    const fq_v2f lo = __builtin_amdgcn_cvt_pk_f32_fp8(w[x], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(w[x], true);
                    pv[4 * x] = lo[0]; pv[4 * x + 1] = lo[1]; pv[4 * x + 2] = hi[0]; pv[4 * x + 3] = hi[1];
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) pv[j] = (t0 + j < T) ? fq_e4m3_to_float(prow[j]) : 0.f;
            }
            // P * sigma: at most 8 significant bits, exact in FP32 and in bf16 (tokens past T: both factors are 0)
            // (so the conversion's rounding never acts: one v_cvt_pk_bf16_f32 per pair)
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                const fq_v2f pr = {pv[j] * sg[j], pv[j + 1] * sg[j + 1]};
                const fq_v2bf pb = __builtin_convertvector(pr, fq_v2bf);
                a[m][j] = pb[0];
                a[m][j + 1] = pb[1];
            }
            acc[m][DT] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], ones, acc[m][DT], 0, 0, 0);   // sum_t A'[r, t], every column
        }
#pragma unroll
        for (int d = 0; d < DT; ++d) {
            // codes of this lane's 8 tokens: the low (kq < 2) or high nibbles of the 8 bytes
            const unsigned x0 = ((kq & 2) ? ((unsigned)vq[d][0] >> 4) : (unsigned)vq[d][0]) & 0x0F0F0F0Fu;
            const unsigned x1 = ((kq & 2) ? ((unsigned)vq[d][1] >> 4) : (unsigned)vq[d][1]) & 0x0F0F0F0Fu;
            fq_v4i bw;                                    // two bf16 per word: 0x4180 | c << 3 = 16 + c
            bw[0] = (int)((__builtin_amdgcn_perm(0u, x0, 0x0C010C00u) << 3) | 0x41804180u);
            bw[1] = (int)((__builtin_amdgcn_perm(0u, x0, 0x0C030C02u) << 3) | 0x41804180u);
            bw[2] = (int)((__builtin_amdgcn_perm(0u, x1, 0x0C010C00u) << 3) | 0x41804180u);
            bw[3] = (int)((__builtin_amdgcn_perm(0u, x1, 0x0C030C02u) << 3) | 0x41804180u);
            const fqk_v8bf b = __builtin_bit_cast(fqk_v8bf, bw);
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[m][d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], b, acc[m][d], 0, 0, 0);
        }
        if (PF) cur = nxt;
    }
    fqk_output_finish<MT, DT>(acc, red, p_scale, O, h, d0, R);
}


// The same product for caches and probability rows in 16-byte steps (T and ldp multiples of 16, P and the scales 16-byte
// aligned): a step of a wave is a whole 128-token group.  Lane l = 16 * kq + r fetches, per dimension tile, the
// whole 16-byte chunk of tokens 32 kq .. 32 kq + 31 of dimension r, and the 32 probability codes and 32 scales of the
// same tokens (two 16-byte loads each): 4 + DT wave-level loads per 128 tokens where the kernel above issues
// 4 * (2 + DT) -- a load costs the address path the same whatever its width.  Four matrix instructions use them up:
// number j4 takes, in every lane, tokens 32 kq + 8 j4 .. + 7 (the order of the summation index is free as long
// as both operands agree), i.e. bytes 8 j4 .. of the codes and scales and, of the chunk, the low (j4 < 2) or high
// nibbles of bytes 8 (j4 % 2) ...  A nibble becomes the bf16 number 16 + c in a byte shuffle: low byte 0x80 | c << 3,
// high byte 0x41.  The next group's loads are requested before the current one is worked on.
template <int MT, int DT, bool PF>
__global__ __launch_bounds__(64 * FQK_O_WAVES) void fq_kv4_output_wide_kernel(
    const uint8_t* __restrict__ P, const float* __restrict__ p_scale, const uint8_t* __restrict__ vp,
    const uint8_t* __restrict__ vs, uint16_t* __restrict__ O, int R, int T, int ldp) {
    extern __shared__ float red[];                        // [waves][MT][DT + 1][4][64]
    const int d0 = blockIdx.y * DT;
    const int h = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r16 = lane & 15, kq = lane >> 4;
    const int G = (T + 127) / 128;
    const size_t vbytes = fqk_value_bytes(T);
    const __amdgpu_buffer_rsrc_t rsV = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(vp) + (size_t)h * vbytes, 0, (int)vbytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsS = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(vs) + (size_t)h * T, 0, T, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsP = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(P) + (size_t)h * R * ldp, 0, R * ldp, 0x00020000);
    fq_v4f acc[MT][DT + 1];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int d = 0; d < DT + 1; ++d) acc[m][d] = (fq_v4f){0.f, 0.f, 0.f, 0.f};
    fqk_v8bf ones;
#pragma unroll
    for (int j = 0; j < 8; ++j) ones[j] = __builtin_bit_cast(__bf16, (unsigned short)0x3F80);
    unsigned prow[MT];                                    // byte offset of this lane's probability row(s) in the head
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int row = 16 * m + r16;
        prow[m] = (unsigned)(row < R ? row : R - 1) * (unsigned)ldp;
    }
    unsigned vlane[DT];                                   // this lane's chunk inside a 2048-byte block, per dimension tile
#pragma unroll
    for (int d = 0; d < DT; ++d) {
        const int dim = 16 * (d0 + d) + r16;
        vlane[d] = (unsigned)(dim >> 5) * (unsigned)G * 2048u + (unsigned)(kq >> 1) * 1024u +
                   (unsigned)((kq & 1) * 32 + (dim & 31)) * 16u;
    }
    struct fqk_raw { fq_v4i vq[DT]; fq_v4i ws[2]; fq_v4i wp[MT][2]; };
    auto fetch = [&](int g, fqk_raw& raw) __attribute__((always_inline)) {
        const bool on = g < G;
        const int t0 = 128 * g + 32 * kq;
#pragma unroll
        for (int d = 0; d < DT; ++d)                      // (streamed once: non-temporal)
            raw.vq[d] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(
                rsV, on ? vlane[d] + (unsigned)g * 2048u : FQK_OOB, 0, 2));
#pragma unroll
        for (int x = 0; x < 2; ++x) {                     // T % 16 == 0: a 16-byte step lies before T or past it
            const int tt = t0 + 16 * x;
            const bool in = on && tt < T;
            raw.ws[x] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsS, in ? (unsigned)tt : FQK_OOB, 0, 0));
#pragma unroll
            for (int m = 0; m < MT; ++m)
                raw.wp[m][x] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(
                    rsP, in ? prow[m] + (unsigned)tt : FQK_OOB, 0, 0));
        }
    };
    fqk_raw cur, nxt;
    if (PF) fetch(wave, cur);
    for (int g = wave; g < G; g += FQK_O_WAVES) {
        if (PF) fetch(g + FQK_O_WAVES, nxt);
        else    fetch(g, cur);
#pragma unroll
        for (int j4 = 0; j4 < 4; ++j4) {
            const int x = j4 >> 1, w0 = 2 * (j4 & 1);     // which 16-byte step of codes and scales, which 8 bytes of it
            float sg[8];                                  // sigma of the lane's 8 tokens (zero past T)
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                const int w = cur.ws[x][w0 + y];
                const fq_v2f lo = __builtin_amdgcn_cvt_pk_f32_fp8(w, false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(w, true);
                sg[4 * y] = lo[0]; sg[4 * y + 1] = lo[1]; sg[4 * y + 2] = hi[0]; sg[4 * y + 3] = hi[1];
            }
            fqk_v8bf a[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float pv[8];
#pragma unroll
                for (int y = 0; y < 2; ++y) {
                    const int w = cur.wp[m][x][w0 + y];
                    const fq_v2f lo = __builtin_amdgcn_cvt_pk_f32_fp8(w, false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(w, true);
                    pv[4 * y] = lo[0]; pv[4 * y + 1] = lo[1]; pv[4 * y + 2] = hi[0]; pv[4 * y + 3] = hi[1];
                }
                // P * sigma: at most 8 significant bits, exact in FP32 and in bf16 (the conversion's rounding never acts)
#pragma unroll
                for (int j = 0; j < 8; j += 2) {
                    const fq_v2f pr = {pv[j] * sg[j], pv[j + 1] * sg[j + 1]};
                    const fq_v2bf pb = __builtin_convertvector(pr, fq_v2bf);
                    a[m][j] = pb[0];
                    a[m][j + 1] = pb[1];
                }
                acc[m][DT] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], ones, acc[m][DT], 0, 0, 0);   // sum_t A'[r, t], every column
            }
#pragma unroll
            for (int d = 0; d < DT; ++d) {
                fq_v4i bw;
#pragma unroll
                for (int y = 0; y < 2; ++y) {
                    const unsigned w = (unsigned)cur.vq[d][w0 + y];
                    const unsigned c3 = (((j4 >> 1) ? (w >> 1) : (w << 3)) & 0x78787878u) | 0x80808080u;   // 0x80 | c << 3, 4 tokens
                    bw[2 * y] = (int)__builtin_amdgcn_perm(0x41414141u, c3, 0x04010400u);
                    bw[2 * y + 1] = (int)__builtin_amdgcn_perm(0x41414141u, c3, 0x04030402u);
                }
                const fqk_v8bf b = __builtin_bit_cast(fqk_v8bf, bw);
#pragma unroll
                for (int m = 0; m < MT; ++m) acc[m][d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], b, acc[m][d], 0, 0, 0);
            }
        }
        if (PF) cur = nxt;
    }
    fqk_output_finish<MT, DT>(acc, red, p_scale, O, h, d0, R);
}

}  // namespace

size_t fq_kv4_key_bytes(int T) { return fqk_key_bytes(T); }
size_t fq_kv4_value_bytes(int T) { return fqk_value_bytes(T); }

void fq_launch_kv4_pack(const int8_t* codes, uint8_t* packed, int H, int T, bool values, hipStream_t stream) {
    const size_t per_head = values ? fqk_value_bytes(T) : fqk_key_bytes(T);
    const dim3 grid((unsigned)((per_head + 255u) / 256u), (unsigned)H);
    if (values) hipLaunchKernelGGL(fqk_pack_kernel<true>, grid, dim3(256), 0, stream, codes, packed, T, per_head);
    else        hipLaunchKernelGGL(fqk_pack_kernel<false>, grid, dim3(256), 0, stream, codes, packed, T, per_head);
}

void fq_launch_kv4_unpack(const uint8_t* packed, int8_t* codes, int H, int T, bool values, hipStream_t stream) {
    const size_t per_head = values ? fqk_value_bytes(T) : fqk_key_bytes(T);
    const dim3 grid((unsigned)(((size_t)T * FQK_HEAD + 255u) / 256u), (unsigned)H);
    if (values) hipLaunchKernelGGL(fqk_unpack_kernel<true>, grid, dim3(256), 0, stream, packed, codes, T, per_head);
    else        hipLaunchKernelGGL(fqk_unpack_kernel<false>, grid, dim3(256), 0, stream, packed, codes, T, per_head);
}

void fq_launch_kv4_scores(const uint8_t* Q, const float* q_scale, const uint8_t* kp, const uint8_t* ks, float out_scale,
                          uint16_t* S, int H, int R, int T, hipStream_t stream) {
    const dim3 grid((unsigned)((T + 4 * FQK_S_NSUB * 16 - 1) / (4 * FQK_S_NSUB * 16)), (unsigned)H);
    const bool wide = (T % 4) == 0 && (reinterpret_cast<uintptr_t>(S) % 8) == 0;   // rows of S are then 8-byte aligned
#define FQK_SCORES(MT_) \
    do { \
        if (wide) hipLaunchKernelGGL((fq_kv4_scores_kernel<MT_, true>), grid, dim3(256), 0, stream, Q, q_scale, kp, ks, out_scale, S, R, T); \
        else      hipLaunchKernelGGL((fq_kv4_scores_kernel<MT_, false>), grid, dim3(256), 0, stream, Q, q_scale, kp, ks, out_scale, S, R, T); \
    } while (0)
    switch ((R + 15) / 16) {
        case 1: FQK_SCORES(1); break;
        case 2: FQK_SCORES(2); break;
        case 3: FQK_SCORES(3); break;
        default: FQK_SCORES(4); break;
    }
#undef FQK_SCORES
}

namespace {

template <int MT, bool FAST, int DT, bool PF>
void fqk_launch_output_pf(const uint8_t* P, const float* p_scale, const uint8_t* vp, const uint8_t* vs, uint16_t* O,
                          int H, int R, int T, int ldp, hipStream_t stream) {
    constexpr size_t lds = (size_t)FQK_O_WAVES * MT * (DT + 1) * 4 * 64 * sizeof(float);
    static fq_device_once attr_once;                      // (one per template instance)
    fq_once_per_device(attr_once, [] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fq_kv4_output_kernel<MT, FAST, DT, PF>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    hipLaunchKernelGGL((fq_kv4_output_kernel<MT, FAST, DT, PF>), dim3((unsigned)H, 8 / DT), dim3(64 * FQK_O_WAVES), lds,
                       stream, P, p_scale, vp, vs, O, R, T, ldp);
}

template <int MT, int DT>
void fqk_launch_output_wide(const uint8_t* P, const float* p_scale, const uint8_t* vp, const uint8_t* vs, uint16_t* O,
                            int H, int R, int T, int ldp, hipStream_t stream) {
    constexpr size_t lds = (size_t)FQK_O_WAVES * MT * (DT + 1) * 4 * 64 * sizeof(float);
    constexpr bool PF = FQK_O_WIDE_PF(MT, DT);
    static fq_device_once attr_once;                      // (one per template instance)
    fq_once_per_device(attr_once, [] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fq_kv4_output_wide_kernel<MT, DT, PF>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    hipLaunchKernelGGL((fq_kv4_output_wide_kernel<MT, DT, PF>), dim3((unsigned)H, 8 / DT), dim3(64 * FQK_O_WAVES), lds,
                       stream, P, p_scale, vp, vs, O, R, T, ldp);
}

// MODE 0: byte loads; 1: 8-byte steps; 2: 16-byte steps (the wide kernel)
template <int MT, int MODE, int DT>
void fqk_launch_output(const uint8_t* P, const float* p_scale, const uint8_t* vp, const uint8_t* vs, uint16_t* O,
                       int H, int R, int T, int ldp, hipStream_t stream) {
    if (MODE == 2)
        fqk_launch_output_wide<MT, DT>(P, p_scale, vp, vs, O, H, R, T, ldp, stream);
    // fewer workgroups than twice the compute units (only possible at one dimension tile per workgroup): prefetch
    else if (DT == 1 && (long)H * 8 < (long)FQK_O_FILL * fq_device_cus())
        fqk_launch_output_pf<MT, MODE == 1, DT, true>(P, p_scale, vp, vs, O, H, R, T, ldp, stream);
    else
        fqk_launch_output_pf<MT, MODE == 1, DT, false>(P, p_scale, vp, vs, O, H, R, T, ldp, stream);
}

template <int MT, int MODE>
void fqk_launch_output_dt(int dt, const uint8_t* P, const float* p_scale, const uint8_t* vp, const uint8_t* vs, uint16_t* O,
                          int H, int R, int T, int ldp, hipStream_t stream) {
    if (dt == 8)      fqk_launch_output<MT, MODE, 8>(P, p_scale, vp, vs, O, H, R, T, ldp, stream);
    else if (dt == 4) fqk_launch_output<MT, MODE, 4>(P, p_scale, vp, vs, O, H, R, T, ldp, stream);
    else if (dt == 2) fqk_launch_output<MT, MODE, 2>(P, p_scale, vp, vs, O, H, R, T, ldp, stream);
    else              fqk_launch_output<MT, MODE, 1>(P, p_scale, vp, vs, O, H, R, T, ldp, stream);
}

}  // namespace

void fq_launch_kv4_output(const uint8_t* P, const float* p_scale, const uint8_t* vp, const uint8_t* vs, uint16_t* O,
                          int H, int R, int T, int ldp, hipStream_t stream) {
    const uintptr_t both = reinterpret_cast<uintptr_t>(P) | reinterpret_cast<uintptr_t>(vs) | (uintptr_t)T | (uintptr_t)ldp;
    // (the kernel of 16-byte steps addresses a head's probability rows through 32-bit buffer offsets)
    const bool rows32 = (unsigned long long)R * (unsigned long long)ldp < 0xFFFFFF00ull;
    const int mode = ((both % 16) == 0 && rows32) ? 2 : (both % 8) == 0 ? 1 : 0;
    // dimension tiles per workgroup: the most that still give `fill` workgroups per compute unit
    const int cus = fq_device_cus();
    int dt = mode == 2 ? FQK_O_WIDE_MAXDT : 8;
    const int fill = mode == 2 ? FQK_O_WIDE_FILL : FQK_O_FILL;
    while (dt > 1 && (long)H * (8 / dt) < (long)fill * cus) dt >>= 1;
#define FQK_OUTPUT(MT_) \
    do { \
        if (mode == 2)      fqk_launch_output_dt<MT_, 2>(dt, P, p_scale, vp, vs, O, H, R, T, ldp, stream); \
        else if (mode == 1) fqk_launch_output_dt<MT_, 1>(dt, P, p_scale, vp, vs, O, H, R, T, ldp, stream); \
        else                fqk_launch_output_dt<MT_, 0>(dt, P, p_scale, vp, vs, O, H, R, T, ldp, stream); \
    } while (0)
    if (R <= 16) FQK_OUTPUT(1);
    else         FQK_OUTPUT(2);
#undef FQK_OUTPUT
}
