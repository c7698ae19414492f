// Device helpers shared by the large-M GEMM kernels (fq_gemm_large.hip, fq_gemm_ksplit.hip): the FP8 and
// fp16 MFMA wrappers, the zero-point plane layout, the global -> LDS transfers of A tiles, packed weights and
// zero-point units, and the table mode's look-up.
#pragma once
#include "fq_common.h"

#define FQL_XCDS 8

#define FQ_MFMA(a, b, c) __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4((a), (b), (c), 0, 0, 0, 0, 0, 0)

namespace {

typedef __attribute__((address_space(3))) void* fql_lds_ptr;
typedef _Float16 fql_v8h __attribute__((ext_vector_type(8)));

#define FQ_MFMA_F16(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_f16((a), (b), (c), 0, 0, 0)
#define FQL_ZPLANES 2

// Zero-point planes: Z[m, g] = -2^-6 * sum_{k in group g} A[m, k] as two fp16 terms, hi = fp16(Z) and
// lo = fp16(Z - hi), 22 significant bits together (what is left, at most 2^-22 |Z|, is far below the
// FP32 accumulation noise of the main sum).  Stored as units of [M rows][8 groups] fp16 (16 bytes
// per row), unit index u = plane * C2 + g / 8 with C2 = 2 * ceil(G / 16) (groups past G are zero),
// so that one 16-byte chunk is what one lane of the 32x32x16 fp16 MFMA holds of the A operand.
__host__ __device__ inline int fql_c2(int G) { return 2 * ((G + 15) / 16); }

// LDS layout of one A stage (one 128-wide group of up to 256 rows): row-major, 8 slots of 16 bytes per
// row; slot c of row r holds bytes 16*x .. 16*x+15 of the row's group with x = c ^ ((r >> 1) & 7).
// The XOR makes the operand reads (lane = row, fixed x) hit 16 different bank groups per 16 lanes,
// while the global->LDS transfer (buffer_load_dwordx4 ... lds, LDS address linear in the lane) still
// fetches whole 128-byte rows: 8 rows per instruction.
// Addressing: the buffer descriptor covers all of A, so rows past M read as zero.  The bounds
// check of a buffer load looks at the per-lane offset only, so the row is part of that offset
// (a per-lane constant plus a scalar term per transfer); the group travels in the scalar offset.
// A tile of 32 * NMT rows is fetched by the 4 waves: NT = NMT transfers of 8 rows per wave and group.
// Per-lane byte offset of transfer 0 without the tile's first row (that part is scalar):
__device__ __forceinline__ unsigned fql_a_lane_base(int wave, int lane, int K, int nt) {
    const int row = wave * (8 * nt) + (lane >> 3);        // tile row of transfer 0
    const int c0 = (lane & 7) ^ ((row >> 1) & 7);         // == (lane & 7) ^ (lane >> 4): the wave's term drops out
    return (unsigned)row * (unsigned)K + (unsigned)c0 * 16u;
}

// `oob` = FQL_OOB requests the tile out of range instead: zeros arrive, and nothing is fetched.
#define FQL_OOB 0xFFFFFF00u
template <int NT>
__device__ __forceinline__ void fql_issue_a(__amdgpu_buffer_rsrc_t rsrc, unsigned abase, int m0, int K,
                                            fq_v4i* lds_stage, int wave, int g, unsigned oob = 0u) {
    fq_v4i* dst = lds_stage + wave * (64 * NT);           // this wave's 8 * NT rows
    const int sg = g * FQ_GROUP;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        // odd transfers start 8 rows further, where the swizzle flips bit 2 of the column
        const unsigned v = ((abase ^ ((j & 1) ? 64u : 0u)) + (unsigned)(m0 + 8 * j) * (unsigned)K) | oob;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (fql_lds_ptr)(dst + 64 * j), 16, v, sg, 0, 0);
    }
}

// One group of this wave's packed weights (2 KiB: two halves of 64 lanes x 16 bytes) -> LDS.
__device__ __forceinline__ void fql_issue_b(__amdgpu_buffer_rsrc_t rsrc, fq_v4i* dst, unsigned lane16, unsigned blk_off) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (fql_lds_ptr)dst, 16, lane16, blk_off, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (fql_lds_ptr)(dst + 64), 16, lane16, blk_off + 1024u, 0, 0);
}

// One round of zero-point units (up to 8, numbers u0 ..) -> an A stage: NMT transfers of 64 rows per
// wave (4 waves), the same number as an A tile takes, so that the pipeline's wait counts do not change; slots
// past the last unit are requested out of range (zeros).  Unit slot s occupies chunks [s * RT, (s+1) * RT).
template <int NMT, int WAVES = 4>
__device__ __forceinline__ void fql_issue_z(__amdgpu_buffer_rsrc_t rsZ, fq_v4i* lds_stage, int wave, int lane,
                                            int m0, int M, int u0, int nu) {
    constexpr int RT = 32 * NMT, SUBS = RT / 64;
    static_assert(RT % 64 == 0 && (4 * NMT) % WAVES == 0, "whole transfers of 64 rows, an equal number per wave");
#pragma unroll
    for (int t = 0; t < 4 * NMT / WAVES; ++t) {
        const int q = wave + WAVES * t;
        const int slot = q / SUBS, sub = q - slot * SUBS;
        // rows past M are masked like slots past the last unit: the range check sees the per-lane
        // offset only, and the last unit's scalar offset would carry such a row past the workspace
        const int row = m0 + 64 * sub + lane;
        const unsigned v = (slot < nu && row < M) ? (unsigned)row * 16u : 0xFFFFFF00u;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsZ, (fql_lds_ptr)(lds_stage + slot * RT + 64 * sub), 16, v,
                                                 (int)((unsigned)(u0 + slot) * (unsigned)M * 16u), 0, 0);
    }
}

// ---- table mode (Sec. 3.1.1 step 1): the group scale folded into a 16-entry FP8 table ----
// T[c] = E4M3(q * sigma), q = c - 8, rounded to nearest even and saturating at +-448: the paper's
// in-register table {-8 sigma .. 7 sigma} of one group of one channel, 16 bytes in four registers.
__device__ __forceinline__ fq_v4i fql_lut_table(float sigma) {
    fq_v4i t;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = fminf(fmaxf((float)(4 * i + e - 8) * sigma, -448.f), 448.f);   // q * sigma is exact in FP32
        int r = 0;
        r = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], r, false);
        r = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], r, true);
        t[i] = r;
    }
    return t;
}

// Four codes (one per byte, 0..15) -> their four table entries: two 8-entry byte permutes and a select
// on bit 3 of each code.
__device__ __forceinline__ int fql_lut4(unsigned x, fq_v4i t) {
    const unsigned lo = x & 0x07070707u;
    const unsigned r0 = __builtin_amdgcn_perm((unsigned)t[1], (unsigned)t[0], lo);
    const unsigned r1 = __builtin_amdgcn_perm((unsigned)t[3], (unsigned)t[2], lo);
    const unsigned b3 = x & 0x08080808u;
    const unsigned mask = (b3 << 5) - (b3 >> 3);          // 0xFF in every byte whose code is 8 or more
    return (int)((r0 & ~mask) | (r1 & mask));
}

__device__ __forceinline__ fq_v8i fql_unpack_chunk_lut(fq_v4i w, fq_v4i t) {
    fq_v8i r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const unsigned u = (unsigned)w[i];
        r[i]     = fql_lut4(u & 0x0F0F0F0Fu, t);
        r[4 + i] = fql_lut4((u >> 4) & 0x0F0F0F0Fu, t);
    }
    return r;
}

// s_waitcnt immediate (gfx9 encoding) that waits until at most n vector-memory transfers are pending
// and leaves the other counters alone.
#define FQL_WAIT_VM(n) ((((n) & 0xF) | (((n) >> 4) << 14)) | 0x0F70)

// The gscale operands of one round of zero-point units (numbers u0 .. u0 + nu - 1; unit pairs 2 ci, 2 ci + 1 are
// the two lane halves of MFMA chunk ci): for each of the round's up to 4 chunks, 8 consecutive groups of this
// lane's channel as fp16 (E4M3 -> fp16 is exact, whatever the rounding mode).  The 8 scale bytes of groups
// g0 .. g0 + 7 start at byte n * G + g0 of the array, which is a multiple of 4 only when G is: the aligned words
// around them are fetched and shifted into place.  `rsS` covers the scale array rounded up to whole words (the
// array's last word may hold fewer than four scales, and a word that crosses the end of the range would read as
// zero; the array is 16-byte aligned, so that word lies in the same cache line as its valid bytes).  Everything
// that is not wanted -- a chunk past the round's units, groups past G, a channel past N -- is requested out of
// range and reads as zero, so all the loads are issued back to back without a branch.
// Two halves, so that the loads can be issued long before their use (under load they take several microseconds):
// fql_scales_issue requests the raw words, fql_scales_finish turns them into operands.
struct fql_raw_scales { unsigned d[4][3]; };

__device__ __forceinline__ void fql_scales_issue(__amdgpu_buffer_rsrc_t rsS, unsigned srow, bool n_ok, int G, int C2,
                                                 int u0, int nu, int hl, fql_raw_scales& raw) {
    const bool unaligned_rows = (G & 3) != 0;             // (the array itself is 16-byte aligned)
#pragma unroll
    for (int ci = 0; ci < 4; ++ci) {
        const int c = ((u0 + 2 * ci) % C2) >> 1;          // chunk index inside its plane
        const int g0 = 16 * c + 8 * hl;
        const unsigned o = srow + (unsigned)g0;
        const unsigned ob = (2 * ci < nu && n_ok && g0 < G) ? (o & ~3u) : FQL_OOB;
        // one load instruction per chunk: the address path takes as long for a lane's 4 bytes as for its 12
        if (unaligned_rows) {
            typedef unsigned v3u __attribute__((ext_vector_type(3)));
            const v3u t = __builtin_bit_cast(v3u, __builtin_amdgcn_raw_buffer_load_b96(rsS, ob, 0, 0));
            raw.d[ci][0] = t[0]; raw.d[ci][1] = t[1]; raw.d[ci][2] = t[2];
        } else {
            typedef unsigned v2u __attribute__((ext_vector_type(2)));
            const v2u t = __builtin_bit_cast(v2u, __builtin_amdgcn_raw_buffer_load_b64(rsS, ob, 0, 0));
            raw.d[ci][0] = t[0]; raw.d[ci][1] = t[1]; raw.d[ci][2] = 0u;
        }
    }
}

__device__ __forceinline__ void fql_scales_finish(const fql_raw_scales& raw, unsigned srow, int G, int C2, int u0, int hl,
                                                  fql_v8h sig[4]) {
#pragma unroll
    for (int ci = 0; ci < 4; ++ci) {
        const int c = ((u0 + 2 * ci) % C2) >> 1;
        const int g0 = 16 * c + 8 * hl;
        const unsigned o = srow + (unsigned)g0;
        unsigned w[2];
        w[0] = __builtin_amdgcn_alignbyte(raw.d[ci][1], raw.d[ci][0], o & 3u);
        w[1] = __builtin_amdgcn_alignbyte(raw.d[ci][2], raw.d[ci][1], o & 3u);
        // bytes of groups >= G belong to the next channel: cleared
        const int nv = G - g0;                            // valid groups from g0 on
        if (nv < 4) w[0] &= nv <= 0 ? 0u : (1u << (8 * nv)) - 1u;
        if (nv < 8) w[1] &= nv <= 4 ? 0u : (1u << (8 * (nv - 4))) - 1u;
        fq_v4i pk;
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            pk[2 * x]     = __builtin_bit_cast(int, __builtin_amdgcn_cvt_pkrtz(
                __builtin_amdgcn_cvt_f32_fp8((int)w[x], 0), __builtin_amdgcn_cvt_f32_fp8((int)w[x], 1)));
            pk[2 * x + 1] = __builtin_bit_cast(int, __builtin_amdgcn_cvt_pkrtz(
                __builtin_amdgcn_cvt_f32_fp8((int)w[x], 2), __builtin_amdgcn_cvt_f32_fp8((int)w[x], 3)));
        }
        sig[ci] = __builtin_bit_cast(fql_v8h, pk);
    }
}


__device__ __forceinline__ fq_v8i fql_join(fq_v4i lo, fq_v4i hi) {
    fq_v8i r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return r;
}

}  // namespace
