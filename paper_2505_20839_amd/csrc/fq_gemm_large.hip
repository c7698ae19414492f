// W4A8-FP GEMM for large M (compute bound): INT4 weights x E4M3 activations on the gfx950 FP8
// matrix cores (Sec. 3.1.1: unpack INT4 to FP8 in registers, FP8 MMA with FP32 accumulation,
// scale and write bf16).  Differences from the paper's H100 kernel: the group scale is not folded
// into a rounded FP8 table but applied exactly, in FP32, to each group's partial sum; all output
// scaling is FP32 with a single rounding to bf16.
//
// Work split.  A workgroup of 4 waves owns one output tile of 256 (or 128) rows x 128 channels;
// wave w owns 32 channels and all rows of the tile (NMT = 8 or 4 MFMA tiles of 32x32), so every
// weight is unpacked exactly once per workgroup and each unpacked operand is reused by all row tiles.
// Two workgroups share a compute unit (80 KiB of LDS and one wave per SIMD each): the two waves of
// a SIMD belong to different workgroups, so no barrier couples them, and each fills the other's
// stalls inside the loop (the workgroups of a launch run in step, so their prologues and epilogues
// mostly coincide).
// Per 128-wide group g:
//     P   = A[:, g, first 64] * Wq[g, first 64]            v_mfma_f32_32x32x64_f8f6f4, C = 0
//     P  += A[:, g, last 64]  * Wq[g, last 64]             same, C = P
//     acc += e4m3(gscale[n, g]) * P                        16 v_fma_f32 per 32x32 tile
// The packed codes carry a zero point of 8 (byte c reads as the E4M3 number c * 2^-9), so unpacking
// is a mask and a shift, and the sum above comes out too large by 2^-6 * gscale[n, g] * sum_k A[m, k]
// per group.  That excess is a product of a per-(row, group) and a per-(channel, group) factor: the
// activation quantiser (or else a small kernel launched first) writes Z[m, g] = -2^-6 * sum_k A[m, k]
// (FP32, split into two fp16 terms: 22 significant bits), and each tile ends with  acc += Z * gscale^T
// as fp16 MFMAs of depth K / 128; the first round of Z is fetched into the idle A stage during the
// tile's last group.
// A tiles go global -> LDS directly (buffer_load_dwordx4 ... lds, two stages of 32 KiB, one group
// per barrier); packed weights go global -> LDS the same way (2 x 2 KiB private to each wave) and
// are unpacked one group ahead, a slice under each MFMA.
//
// Tile order.  Workgroup b runs on XCD b % 8 (round-robin dispatch); each XCD gets a contiguous
// range of tiles in an order that walks panels of 4 row tiles, row tile fastest, so the workgroups
// an XCD runs at one time cover a few row tiles x a few channel tiles and share them in its L2.
// The tiles an XCD cannot fill a whole round of its slots with are cut into two 128-row halves (the
// NMT = 4 variant, later workgroups of the same launch), so that the last round keeps all units busy
// for half the time.
#include <type_traits>
#include "fq_common.h"
#include "fq_kernels.h"
#include "fq_gemm_large_common.h"

#define FQL_WAVES 4
#define FQL_THREADS (64 * FQL_WAVES)
#define FQL_BM 256
#define FQL_BN (32 * FQL_WAVES)
#define FQL_STAGE_BYTES (FQL_BM * FQ_GROUP)          // 32 KiB: 256 rows x 128 E4M3 bytes
#define FQL_STAGE_CHUNKS (FQL_STAGE_BYTES / 16)
#define FQL_STAGES 2                                 // one group in use, one in flight
#define FQL_LDS_BYTES (FQL_STAGES * FQL_STAGE_BYTES + FQL_WAVES * 4096)   // 80 KiB: two workgroups per CU
#define FQL_OUT_STRIDE (FQL_BN * 2 + 16)             // bytes per row of the output tile staged in LDS

namespace {

// Tiles of XCD x: [lo, lo + count) of the row-tile-fastest order; the first `nfull` are run whole
// by the first launch, the rest as halves by the second.
struct fql_split {
    int lo, nfull, nhalf;                                 // nhalf = number of 128-row items (2 per tile)
};

__host__ __device__ inline fql_split fql_xcd_split(int x, int ntiles, int slots) {
    const int base = ntiles / FQL_XCDS, rem = ntiles % FQL_XCDS;
    const int count = base + (x < rem ? 1 : 0);
    fql_split sp;
    sp.lo = x * base + (x < rem ? x : rem);
    const int r = count % slots;                          // tiles of the last, partial round
    if (r > 0 && 2 * r <= slots) { sp.nfull = count - r; sp.nhalf = 2 * r; }
    else                         { sp.nfull = count;     sp.nhalf = 0; }
    return sp;
}

// Which item workgroup `bid` of its kind (NMT = 8: whole tiles, NMT = 4: 128-row halves) runs: XCD
// x = bid % 8 (both kinds start at a multiple of 8 workgroups), j-th item of that XCD's list.  Tile
// order: panels of `pm` row tiles; inside a panel row tile fastest, then channel tile.  False: no item
// (past the end of the XCD's list, or a second half without rows).
template <int NMT>
__host__ __device__ inline bool fql_locate(unsigned bid, int M, int tiles_m, int tiles_n, int slots, int pm,
                                           int* m0, int* n0) {
    const int x = bid % FQL_XCDS, j = bid / FQL_XCDS;
    const fql_split sp = fql_xcd_split(x, tiles_m * tiles_n, slots);
    int t, half = 0;
    if (NMT == 8) {
        if (j >= sp.nfull) return false;
        t = sp.lo + j;
    } else {
        if (j >= sp.nhalf) return false;
        t = sp.lo + sp.nfull + (j >> 1);
        half = j & 1;
    }
    const int per_panel = pm * tiles_n;
    const int panel = t / per_panel, rem = t - panel * per_panel;
    const int ph = tiles_m - panel * pm < pm ? tiles_m - panel * pm : pm;   // row tiles of this panel
    const int tn = rem / ph, tm = panel * pm + (rem - tn * ph);
    *m0 = tm * FQL_BM + half * 128;
    *n0 = tn * FQL_BN;
    return *m0 < M;
}

}  // namespace

// One workgroup per row m; eight lanes per group: each sums 16 of the group's 128 activations, the
// eight partial sums are added across lanes, the two fp16 terms of -2^-6 * sum are collected in LDS
// (zeros for the padding groups g >= G) and leave as one 16-byte store per (plane, 8 groups).
#define FQL_ZP_MAXG 1024                                  // groups per row the LDS row buffer holds
__global__ __launch_bounds__(256) void fq_zero_point_kernel(const uint8_t* __restrict__ A, uint16_t* __restrict__ planes,
                                                            int M, int K) {
    __shared__ __attribute__((aligned(16))) uint16_t zrow[2][FQL_ZP_MAXG];
    const int G = K / FQ_GROUP, C2 = fql_c2(G), G8 = 8 * C2;
    const int m = blockIdx.x;
    const int sub = threadIdx.x & 7;
    const uint8_t* row = A + (size_t)m * K + 16 * sub;
    if (M <= FQ_KSPLIT_MAX_M) {                           // the arrival counters behind the planes start at zero
        unsigned* counters = reinterpret_cast<unsigned*>(planes + (size_t)FQL_ZPLANES * C2 * M * 8);
        for (int i = blockIdx.x * 256 + threadIdx.x; i < FQ_KSPLIT_COUNTERS; i += gridDim.x * 256) counters[i] = 0u;
    }
    for (int g0 = 0; g0 < G8; g0 += FQL_ZP_MAXG) {        // (one pass unless K > 131072)
        const int gn = G8 - g0 < FQL_ZP_MAXG ? G8 - g0 : FQL_ZP_MAXG;
        for (int gl = threadIdx.x >> 3; gl < gn; gl += 32) {
            const int g = g0 + gl;
            float z = 0.f;
            if (g < G) {
                const fq_v4i v = *reinterpret_cast<const fq_v4i*>(row + (size_t)g * FQ_GROUP);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const fq_v2f lo = __builtin_amdgcn_cvt_pk_f32_fp8(v[j], false);
                    const fq_v2f hi = __builtin_amdgcn_cvt_pk_f32_fp8(v[j], true);
                    z += (lo[0] + lo[1]) + (hi[0] + hi[1]);
                }
            }
            z += __shfl_xor(z, 1, 64);
            z += __shfl_xor(z, 2, 64);
            z += __shfl_xor(z, 4, 64);
            if (sub == 0) {
                z *= -0.015625f;
                const _Float16 hi = (_Float16)z;                  // round to nearest even
                const _Float16 lo = (_Float16)(z - (float)hi);    // the difference is exact in FP32
                zrow[0][gl] = __builtin_bit_cast(uint16_t, hi);
                zrow[1][gl] = __builtin_bit_cast(uint16_t, lo);
            }
        }
        __syncthreads();
        for (int t = threadIdx.x; t < 2 * (gn >> 3); t += 256) {
            const int plane = t / (gn >> 3), ul = t - plane * (gn >> 3);
            const fq_v4i v = *reinterpret_cast<const fq_v4i*>(&zrow[plane][8 * ul]);
            *reinterpret_cast<fq_v4i*>(planes + (((size_t)plane * C2 + (g0 >> 3) + ul) * M + m) * 8) = v;
        }
        __syncthreads();
    }
}

// One item: NMT row tiles of 32 rows (8, or 4 for the half tiles) x 128 channels.  `bid` counts the
// workgroups of the item's kind.
// LUT: the paper's table mode instead of the exact one.  The weights enter the matrix cores as
// E4M3(q * sigma) (looked up in a per-group table that is built one group ahead), the products
// accumulate straight into the tile (no per-group scaling, no zero point, `planes` unused), and
// the output factor is a_scale * w_tscale alone.  Everything else (tile order, transfers, epilogues)
// is shared with the exact mode.
template <int NMT, bool LUT = false>
__device__ __forceinline__ void fql_item(
    fq_v4i* lds, const unsigned bid,
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* Y, int M, int N, int K,
    int tiles_m, int tiles_n, int slots, int pm, const uint16_t* __restrict__ planes, const int swiglu,
    const uint16_t* R, unsigned* rowmax = nullptr) {
    constexpr int NT = NMT;                               // A transfers per wave and stage
    const int G = K / FQ_GROUP;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    int m0, n0;
    if (!fql_locate<NMT>(bid, M, tiles_m, tiles_n, slots, pm, &m0, &n0)) return;
    const int nw0 = n0 + wave * 32;                       // first output channel of this wave
    const bool wave_on = nw0 < N;                         // waves past N compute a duplicate tile and store nothing
    const int n = nw0 + (lane & 31);                      // this lane's output channel
    const bool n_ok = n < N;
    const int nt = wave_on ? (nw0 >> 5) : ((N - 1) >> 5);
    const unsigned wblk = (unsigned)nt * (unsigned)G * 2048u;     // byte offset of this wave's block (nt, 0)
    const unsigned lane16 = (unsigned)lane * 16u;
    // buffer descriptors (raw, no stride): out-of-range bytes read as zero
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(A), 0, (int)((unsigned)M * (unsigned)K), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(wp), 0, (int)((unsigned)((N + 31) >> 5) * (unsigned)G * 2048u), 0x00020000);
    const int C2 = fql_c2(G), ZU = FQL_ZPLANES * C2;      // zero-point units of this item's rows
    const __amdgpu_buffer_rsrc_t rsZ = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(planes), 0, (int)((unsigned)ZU * (unsigned)M * 16u), 0x00020000);
    const unsigned abase = fql_a_lane_base(wave, lane, K, NT);
    const uint8_t* gsrow = gs + (size_t)(n_ok ? n : N - 1) * G;

    // operand read offsets (in chunks) of this lane inside a 32-row tile: (half h, part) -> slot
    const int r32 = lane & 31, sw = (r32 >> 1) & 7;
    const int o00 = r32 * 8 + ((2 * (lane >> 5)) ^ sw);   // h = 0, bytes 0..15 of the lane's 32
    const int o01 = o00 ^ 1, o10 = o00 ^ 4, o11 = o00 ^ 5;

    fq_v16f acc[NMT];
#pragma unroll
    for (int t = 0; t < NMT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    fq_v16f zero;
#pragma unroll
    for (int r = 0; r < 16; ++r) zero[r] = 0.f;

    // ---- prologue ----
    // The scale words of the first zero-point round are requested before anything else and wait in registers until
    // the main loop is over: asked for at that point, with every compute unit streaming, they take about 5 us.
    const __amdgpu_buffer_rsrc_t rsS = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(gs), 0, (int)(((unsigned)N * (unsigned)G + 3u) & ~3u), 0x00020000);
    const unsigned srow = n_ok ? (unsigned)n * (unsigned)G : FQL_OOB;    // channels past N read zeros
    fql_raw_scales zraw;
    if (!LUT) fql_scales_issue(rsS, srow, n_ok, G, C2, 0, ZU < 8 ? ZU : 8, lane >> 5, zraw);
    fql_issue_a<NT>(rsA, abase, m0, K, lds, wave, 0);
    // Packed weights also travel global -> LDS directly, into two 2 KiB buffers private to the wave
    // ([half h][lane][16 bytes], the order they have in memory); buffer g & 1 holds group g.
    fq_v4i* wbuf = lds + FQL_STAGES * FQL_STAGE_CHUNKS + wave * 256;
    fql_issue_b(rsW, wbuf, lane16, wblk);
    fql_issue_b(rsW, wbuf + 128, lane16, wblk + (G > 1 ? 2048u : 0u));
    unsigned psb[2];                                      // scale bytes in flight (group g+1, g+2)
    psb[0] = gsrow[0];
    psb[1] = gsrow[G > 1 ? 1 : 0];
    fq_v8i b0[2], b1[2];                                  // unpacked operands: [u] current, [u^1] next
    float sc[2];
    __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(0));
    sc[0] = __builtin_amdgcn_cvt_f32_fp8((int)psb[0], 0);
    if (LUT) {
        const fq_v4i t0 = fql_lut_table(sc[0]);
        b0[0] = fql_unpack_chunk_lut(wbuf[lane], t0);
        b1[0] = fql_unpack_chunk_lut(wbuf[64 + lane], t0);
    } else {
        b0[0] = fq_unpack_chunk(wbuf[lane]);
        b1[0] = fq_unpack_chunk(wbuf[64 + lane]);
    }
    b0[1] = b0[0]; b1[1] = b1[0]; sc[1] = 0.f;
    __syncthreads();

    fq_v16f pprev = zero;                                 // partial sums of the previous row tile
    float sprev = 0.f;                                    // and their group scale
    // One group per barrier, unrolled by two so that the register pairs [u] / [u^1] are static.
    // Every load is unconditional (group indices are clamped at G-1 instead of skipped; a clamped
    // "ghost" group is multiplied by a zero scale).
    //
    // The body is software-pipelined by hand, one step per MFMA: the step fetches the A operand of
    // the next step from LDS, issues its MFMA, and fills the MFMA's shadow with half of the previous
    // row tile's scale-accumulate (8 v_fma) and a share of the next group's unpack.  Scheduling
    // barriers keep the compiler from undoing that order.
    const int npairs = (G + 1) >> 1;
    fq_v8i an = fql_join(lds[o00], lds[o01]);             // operand of the very first step
    // One pair of groups; LAST is the tile's last pair, whose second group fetches the first round
    // of zero-point units instead of a further A tile.
    auto pair_of_groups = [&](const int p, auto last_tag) __attribute__((always_inline)) {
        constexpr bool LAST = decltype(last_tag)::value;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int g = 2 * p + u;
            const fq_v4i* cur = lds + u * FQL_STAGE_CHUNKS;
            {   // A tile of the next group -> the stage the previous group used (all waves are past
                // the barrier that ended it)
                const int g1 = g + 1 < G ? g + 1 : G - 1;
                if (LAST && u == 1 && !LUT)
                    fql_issue_z<NMT>(rsZ, lds + (u ^ 1) * FQL_STAGE_CHUNKS, wave, lane, m0, M, 0, ZU < 8 ? ZU : 8);
                else
                    fql_issue_a<NT>(rsA, abase, m0, K, lds + (u ^ 1) * FQL_STAGE_CHUNKS, wave, g1);
            }
            // Group g+1 sits in buffer u^1 (requested one group ago) and is unpacked slice by slice
            // under the MFMAs below; buffer u (group g, already unpacked) is refilled with group g+2.
            const unsigned qs = psb[u ^ 1];
            {
                const int g2 = g + 2 < G ? g + 2 : G - 1;
                fql_issue_b(rsW, wbuf + u * 128, lane16, wblk + (unsigned)g2 * 2048u);
                psb[u] = gsrow[g2];
            }
            // Transfers requested after group g+1's weights and scale byte: the NT A transfers and the
            // 3 just above -> once at most that many are pending, g+1 has landed.
            __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(NT + 3));
            const fq_v4i* nxt = wbuf + (u ^ 1) * 128 + lane;
            const float s = sc[u];
            fq_v4i tabn = {0, 0, 0, 0};                   // table of group g+1 (all zero for a ghost group)
            if (LUT) tabn = fql_lut_table((g + 1 < G) ? __builtin_amdgcn_cvt_f32_fp8((int)qs, 0) : 0.f);
            fq_v4i q = nxt[0];                            // packed words 0..3; 4..7 are fetched half-way
            fq_v16f pt;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mt = 0; mt < NMT; ++mt) {
                const int tp = (mt + NMT - 1) % NMT;
                const float sp = (mt == 0) ? sprev : s;   // the last row tile of the previous group used the old scale
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const fq_v8i ac = an;
                    // A operand of the next step (none after the last step of a group: the next
                    // stage is only complete after the barrier)
                    if (h == 0) {
                        an = fql_join(cur[mt * 256 + o10], cur[mt * 256 + o11]);
                    } else if (mt + 1 < NMT) {
                        an = fql_join(cur[(mt + 1) * 256 + o00], cur[(mt + 1) * 256 + o01]);
                    }
                    if (LUT) {
                        acc[mt] = FQ_MFMA(ac, h == 0 ? b0[u] : b1[u], acc[mt]);
                    } else {
                        if (h == 0) pt = FQ_MFMA(ac, b0[u], zero);
                        else        pt = FQ_MFMA(ac, b1[u], pt);
#pragma unroll
                        for (int r = 8 * h; r < 8 * h + 8; ++r) acc[tp][r] = fmaf(sp, pprev[r], acc[tp][r]);
                    }
                    // a share of the next group's unpack: half a packed word per step with 8 row
                    // tiles, a whole word's half twice with 4
#pragma unroll
                    for (int e = 0; e < 8 / NMT; ++e) {
                        const int slot = (8 / NMT) * mt + e;                    // packed word 0..7
                        const unsigned w = (unsigned)q[slot & 3];
                        const unsigned x = (h == 0 ? w : (w >> 4)) & 0x0F0F0F0Fu;
                        const int ev = LUT ? fql_lut4(x, tabn) : (int)x;   // exact mode: byte c = c * 2^-9 in E4M3
                        if (slot < 4) b0[u ^ 1][4 * h + (slot & 3)] = ev;
                        else          b1[u ^ 1][4 * h + (slot & 3)] = ev;
                    }
                    if (mt == NMT / 2 - 1 && h == 1) q = nxt[64];
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // the two LDS reads
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // the MFMA
                    __builtin_amdgcn_sched_group_barrier(0x002, 24, 0);  // its shadow: VALU work
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (!LUT) pprev = pt;
            }
            sprev = s;
            {
                const float t = __builtin_amdgcn_cvt_f32_fp8((int)qs, 0);
                sc[u ^ 1] = (g + 1 < G) ? t : 0.f;
            }
            // the next group's A tile: this wave's part has landed once only the 3 transfers issued
            // after it are pending; the barrier then vouches for the other waves' parts
            __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(3));
            __syncthreads();
            {
                const fq_v4i* nxs = lds + (u ^ 1) * FQL_STAGE_CHUNKS;
                an = fql_join(nxs[o00], nxs[o01]);
            }
        }
    };
    for (int p = 0; p < npairs - 1; ++p) pair_of_groups(p, std::false_type());
    pair_of_groups(npairs - 1, std::true_type());
    // last pending row tile of the last group
    if (!LUT) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[NMT - 1][r] = fmaf(sprev, pprev[r], acc[NMT - 1][r]);
    }

    // ---- residual tile (activation addition, Sec. 3.1.1 step 3): requested now, used in the epilogue ----
    // Step `it` of the epilogue handles rows 8 * it + 4 * (lane / 32) + 0..3 of this lane's channel.
    // Lanes l, l ^ 1 hold neighbouring channels: the even lane fetches the pair's two bf16 of rows
    // 0, 1 as one dword each, the odd lane those of rows 2, 3, and they swap in the epilogue.
    // Channels past N wrap into the next row (never stored), rows past M read zero.  All of these
    // loads have landed before this workgroup's first store (the zero-point rounds wait for every
    // transfer), and no other workgroup touches this tile: R may be the output array itself.
    const bool full_tile = (m0 + 32 * NMT <= M) && (n0 + FQL_BN <= N) && ((N & 7) == 0);
    const bool add_full = R != nullptr && full_tile;
    unsigned rres[4 * NMT][2];
    if (add_full) {
        const __amdgpu_buffer_rsrc_t rsR = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(R) + (size_t)m0 * N + n0, 0, (int)((unsigned)(32 * NMT) * (unsigned)N * 2u), 0x00020000);
        const unsigned rlane = ((unsigned)(4 * (lane >> 5) + 2 * (lane & 1)) * (unsigned)N +
                                (unsigned)(wave * 32 + ((lane & 31) & ~1))) * 2u;
#pragma unroll
        for (int it = 0; it < 4 * NMT; ++it)
#pragma unroll
            for (int x = 0; x < 2; ++x)
                rres[it][x] = __builtin_amdgcn_raw_buffer_load_b32(rsR, rlane, (8 * it + x) * N * 2, 0);
    }

    // ---- zero point: acc += Z * gscale^T over the groups, on the fp16 matrix cores ----
    // Rounds of up to 8 units of Z (32 * NMT rows x 8 groups, 16 bytes per row); round r sits in A
    // stage r & 1 (round 0 arrived during the last group) while the next round is on its way to
    // the other stage.  Units 2c and 2c + 1 of a plane are the two lane halves of MFMA chunk c.
    if (LUT) {                                            // no zero point; the stages are reused below
        __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(0));
        __syncthreads();
    } else {
        constexpr int RT = 32 * NMT;                      // rows of the item
        const int hl = lane >> 5;                         // which half of a chunk's 16 groups this lane holds
        const int rounds = (ZU + 7) >> 3;
        for (int r = 0; r < rounds; ++r) {
            const int u0 = 8 * r;
            const int nu = ZU - u0 < 8 ? ZU - u0 : 8;
            // gscale operands of this round's chunks (8 consecutive groups of this lane's channel as fp16), from the
            // words requested a round ago (the first time: before the main loop)
            fql_v8h sig[4];
            fql_scales_finish(zraw, srow, G, C2, u0, hl, sig);
            if (r + 1 < rounds) {                         // that stage was last read before the previous barrier
                const int nn = ZU - u0 - 8 < 8 ? ZU - u0 - 8 : 8;
                fql_issue_z<NMT>(rsZ, lds + ((r + 1) & 1) * FQL_STAGE_CHUNKS, wave, lane, m0, M, u0 + 8, nn);
                fql_scales_issue(rsS, srow, n_ok, G, C2, u0 + 8, nn, hl, zraw);
            }
            const fq_v4i* stage = lds + (r & 1) * FQL_STAGE_CHUNKS;
#pragma unroll
            for (int ci = 0; ci < 4; ++ci) {
                if (2 * ci < nu) {
                    const fq_v4i* unit = stage + (2 * ci + hl) * RT + (lane & 31);
#pragma unroll
                    for (int mt = 0; mt < NMT; ++mt)
                        acc[mt] = FQ_MFMA_F16(__builtin_bit_cast(fql_v8h, unit[32 * mt]), sig[ci], acc[mt]);
                }
            }
            __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(0));   // the next round (and, the first time, the last ghost weights)
            __syncthreads();
        }
    }

    // ---- epilogue: per-token and per-tensor factors, one rounding to bf16, store ----
    // The stages are reused once more (the barrier below orders that after the last read of the
    // zero-point units): the first 32 * NMT * FQL_OUT_STRIDE bytes become the output tile, which also
    // covers part of the weight buffers (their ghost transfers have landed: the zero-point rounds
    // waited for all transfers), 1 KiB behind the largest tile holds the row factors.
    float* osc = reinterpret_cast<float*>(reinterpret_cast<char*>(lds) + FQL_BM * FQL_OUT_STRIDE);
    for (int i = threadIdx.x; i < 32 * NMT; i += FQL_THREADS) {   // x 2^9: the weights were fed in units of 2^-9
        int m = m0 + i;
        osc[i] = a_scale[m < M ? m : M - 1] * (LUT ? tscale : tscale * 512.0f);
    }
    __syncthreads();
    if (swiglu) {
        // Fused gate/up epilogue (Sec. 3.1.1 step 3): even channels are gate, odd channels up rows;
        // H[m, n/2] = bf16(SiLU(gate) * up), H being [M, N/2].  Lanes l and l^1 hold the two channels
        // of a pair for the same rows: the even lane finishes rows rl, rl+1 of a step, the odd lane
        // rows rl+2, rl+3, each after getting the other's two values by a lane swap.
        const int NH = N >> 1;
        const bool full_h = (m0 + 32 * NMT <= M) && (n0 + FQL_BN <= N) && ((NH & 7) == 0);
        if (full_h) {
            constexpr int HS = FQL_BN + 16;               // LDS row stride in bytes: 64 bf16 + pad
            char* tile = reinterpret_cast<char*>(lds);
            const int odd = lane & 1;
            char* wcol = tile + (4 * (lane >> 5) + 2 * odd) * HS + (wave * 16 + ((lane & 31) >> 1)) * 2;
            constexpr int AHEAD = 3;
            const float* oscl = osc + 4 * (lane >> 5);
            fq_v4f scq[AHEAD + 1];
#pragma unroll
            for (int it = 0; it < AHEAD; ++it) scq[it] = *reinterpret_cast<const fq_v4f*>(&oscl[8 * it]);
#pragma unroll
            for (int it = 0; it < 4 * NMT; ++it) {        // step it: rows 8 * it + 4 * (lane / 32) + 0..3 of the item
                const int mt = it >> 2, j = it & 3;
                if (it + AHEAD < 4 * NMT)
                    scq[(it + AHEAD) % (AHEAD + 1)] = *reinterpret_cast<const fq_v4f*>(&oscl[8 * (it + AHEAD)]);
                const fq_v4f sc4 = scq[it % (AHEAD + 1)];
                const float f0 = acc[mt][4 * j] * sc4[0], f1 = acc[mt][4 * j + 1] * sc4[1];
                const float f2 = acc[mt][4 * j + 2] * sc4[2], f3 = acc[mt][4 * j + 3] * sc4[3];
                const float s0 = odd ? f0 : f2, s1 = odd ? f1 : f3;       // what the partner lane needs
                const float r0 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s0), 0xB1, 0xF, 0xF, false));
                const float r1 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s1), 0xB1, 0xF, 0xF, false));
                const fq_v2f pr = odd ? (fq_v2f){fq_silu_mul(r0, f2), fq_silu_mul(r1, f3)}
                                      : (fq_v2f){fq_silu_mul(f0, r0), fq_silu_mul(f1, r1)};
                const unsigned pk = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, fq_v2bf));
                char* dst = wcol + (8 * it) * HS;
                *reinterpret_cast<unsigned short*>(dst) = (unsigned short)pk;
                *reinterpret_cast<unsigned short*>(dst + HS) = (unsigned short)(pk >> 16);
            }
            __syncthreads();
            // wave w stores rows 8*NMT*w ..., eight rows of 128 bytes per instruction
            const __amdgpu_buffer_rsrc_t rsH = __builtin_amdgcn_make_buffer_rsrc(
                Y + (size_t)(m0 + wave * (8 * NMT)) * NH + (n0 >> 1), 0, (int)((unsigned)(8 * NMT) * (unsigned)NH * 2u), 0x00020000);
            const unsigned hlane = (unsigned)(lane >> 3) * (unsigned)NH * 2u + (unsigned)(lane & 7) * 16u;
            const char* rd = tile + (wave * (8 * NMT) + (lane >> 3)) * HS + (lane & 7) * 16;
#pragma unroll
            for (int j = 0; j < NMT; ++j) {
                const fq_v4i v = *reinterpret_cast<const fq_v4i*>(rd + 8 * j * HS);
                __builtin_amdgcn_raw_buffer_store_b128(v, rsH, hlane, 8 * j * NH * 2, 0);
                if (rowmax) {
                    // largest |H| of this row's 64 columns of the tile: bf16 magnitudes order like 16-bit integers;
                    // the 8 lanes of a row fold theirs and one of them raises the row's maximum (the bits of the
                    // number as FP32), which the quantiser of the next layer takes its scale from
                    typedef unsigned short v2us __attribute__((ext_vector_type(2)));
                    v2us mx = __builtin_bit_cast(v2us, (unsigned)v[0] & 0x7FFF7FFFu);
#pragma unroll
                    for (int e = 1; e < 4; ++e)
                        mx = __builtin_elementwise_max(mx, __builtin_bit_cast(v2us, (unsigned)v[e] & 0x7FFF7FFFu));
                    unsigned m16 = mx[0] > mx[1] ? mx[0] : mx[1];
#pragma unroll
                    for (int o = 1; o < 8; o <<= 1) {
                        const unsigned other = (unsigned)__shfl_xor((int)m16, o, 64);
                        m16 = other > m16 ? other : m16;
                    }
                    if ((lane & 7) == 0) atomicMax(&rowmax[m0 + wave * (8 * NMT) + (lane >> 3) + 8 * j], m16 << 16);
                }
            }
            return;
        }
        // ragged tile: element-wise (both lanes of a pair are inside or both outside, N being even)
        if (!wave_on || !n_ok) return;
#pragma unroll
        for (int mt = 0; mt < NMT; ++mt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ml = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const float f = acc[mt][r] * osc[ml];
                const float up = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(f), 0xB1, 0xF, 0xF, false));
                if (m0 + ml < M && (lane & 1) == 0) {
                    fq_v2f pr = {fq_silu_mul(f, up), 0.f};
                    fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
                    const unsigned short hb = __builtin_bit_cast(unsigned short, pk[0]);
                    Y[(size_t)(m0 + ml) * NH + (n >> 1)] = hb;
                    if (rowmax) atomicMax(&rowmax[m0 + ml], ((unsigned)hb & 0x7FFFu) << 16);
                }
            }
        }
        return;
    }
    if (full_tile) {
        // Transpose through LDS so that every store instruction writes whole 256-byte rows.
        // A step covers four rows of the lane's channel (registers 4 j .. 4 j + 3).  The four lanes of a quad hold
        // the same four rows of four neighbouring channels: a 4 x 4 transpose inside the quad (bf16 pairs, two
        // exchanges by DPP) leaves lane q of the quad with row q of the step for all four channels, 8 bytes that
        // go to LDS in one write -- a quarter of the LDS instructions that one 16-bit write per value takes.
        // LDS tile: 256 bytes per row, no padding; the 64-byte segment of wave w in row r sits at segment
        // w ^ (r & 3), so that the four rows a quad writes fall on different segments (two per bank half: the
        // least a 512-byte instruction can do).
        char* tile = reinterpret_cast<char*>(lds);
        const int q4 = lane & 3;                          // row of the step this lane ends up with
        char* wrow = tile + (4 * (lane >> 5) + q4) * 256 + ((wave ^ q4) * 64) + (lane & 28) * 2;
        const bool oddl = lane & 1, upper = (lane & 2) != 0;
        // byte selectors of v_perm_b32 (operand order {partner, own}: bytes 0-3 own, 4-7 partner)
        const unsigned sel_a = oddl ? 0x03020706u : 0x05040100u;   // even: (own.lo, partner.lo); odd: (partner.hi, own.hi)
        // The row factors are fetched from LDS three steps (of four rows) ahead of their use: the
        // compiler may not move these reads across the tile writes, so the distance is spelled out.
        constexpr int AHEAD = 3;
        const float* oscl = osc + 4 * (lane >> 5);
        fq_v4f scq[AHEAD + 1];
#pragma unroll
        for (int it = 0; it < AHEAD; ++it) scq[it] = *reinterpret_cast<const fq_v4f*>(&oscl[8 * it]);
#pragma unroll
        for (int it = 0; it < 4 * NMT; ++it) {            // step it: rows 8 * it + 4 * (lane / 32) + 0..3 of the item
            const int mt = it >> 2, j = it & 3;
            if (it + AHEAD < 4 * NMT)
                scq[(it + AHEAD) % (AHEAD + 1)] = *reinterpret_cast<const fq_v4f*>(&oscl[8 * (it + AHEAD)]);
            const fq_v4f sc4 = scq[it % (AHEAD + 1)];
            fq_v4f res = {0.f, 0.f, 0.f, 0.f};
            if (add_full) {                               // this lane's four residual values (see the loads above)
                const unsigned d0 = rres[it][0], d1 = rres[it][1];
                const unsigned p0 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)d0, 0xB1, 0xF, 0xF, false);
                const unsigned p1 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)d1, 0xB1, 0xF, 0xF, false);
                const unsigned a[4] = {oddl ? p0 : d0, oddl ? p1 : d1, oddl ? d0 : p0, oddl ? d1 : p1};
                const unsigned sh = oddl ? 0u : 16u;
#pragma unroll
                for (int e = 0; e < 4; ++e) res[e] = __uint_as_float((a[e] << sh) & 0xFFFF0000u);
            }
            unsigned pk[2];                               // (row 0, row 1) and (row 2, row 3) of this lane's channel
#pragma unroll
            for (int e = 0; e < 4; e += 2) {
                const fq_v2f pr = add_full ? (fq_v2f){fmaf(acc[mt][4 * j + e], sc4[e], res[e]),
                                                      fmaf(acc[mt][4 * j + e + 1], sc4[e + 1], res[e + 1])}
                                           : (fq_v2f){acc[mt][4 * j + e] * sc4[e], acc[mt][4 * j + e + 1] * sc4[e + 1]};
                pk[e >> 1] = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, fq_v2bf));
            }
            // lanes (0,1) and (2,3) of the quad swap halves: even lanes then hold rows 0 and 2, odd lanes rows 1 and 3,
            // each for the pair's two channels
            const unsigned n0p = (unsigned)__builtin_amdgcn_update_dpp(0, (int)pk[0], 0xB1, 0xF, 0xF, false);
            const unsigned n1p = (unsigned)__builtin_amdgcn_update_dpp(0, (int)pk[1], 0xB1, 0xF, 0xF, false);
            const unsigned a0 = __builtin_amdgcn_perm(n0p, pk[0], sel_a);   // row 0 (even) / row 1 (odd), channels of the pair
            const unsigned a1 = __builtin_amdgcn_perm(n1p, pk[1], sel_a);   // row 2 (even) / row 3 (odd)
            // the two pairs of the quad swap: lanes 0, 1 keep rows 0, 1 and receive the other pair's channels of
            // them, lanes 2, 3 keep rows 2, 3
            const unsigned give = upper ? a0 : a1;
            const unsigned got = (unsigned)__builtin_amdgcn_update_dpp(0, (int)give, 0x4E, 0xF, 0xF, false);
            const fq_v2i out = upper ? (fq_v2i){(int)got, (int)a1} : (fq_v2i){(int)a0, (int)got};
            *reinterpret_cast<fq_v2i*>(wrow + it * (8 * 256)) = out;
        }
        __syncthreads();
        // wave w stores rows 8*NMT*w ..., four rows of 256 bytes per instruction; the row steps
        // travel in the scalar offset of the buffer store
        const __amdgpu_buffer_rsrc_t rsY = __builtin_amdgcn_make_buffer_rsrc(
            Y + (size_t)(m0 + wave * (8 * NMT)) * N + n0, 0, (int)((unsigned)(8 * NMT) * (unsigned)N * 2u), 0x00020000);
        const unsigned ylane = (unsigned)(lane >> 4) * (unsigned)N * 2u + (unsigned)(lane & 15) * 16u;
        // (row R of the tile keeps its segment s at s ^ (R & 3); R & 3 = (lane / 16) & 3 for every row this lane reads)
        const int rq = (lane >> 4) & 3, ch = lane & 15;
        const char* rd = tile + (wave * (8 * NMT) + (lane >> 4)) * 256 + (((ch >> 2) ^ rq) * 64) + (ch & 3) * 16;
#pragma unroll
        for (int j = 0; j < 2 * NMT; ++j) {
            const fq_v4i v = *reinterpret_cast<const fq_v4i*>(rd + 4 * j * 256);
            __builtin_amdgcn_raw_buffer_store_b128(v, rsY, ylane, 4 * j * N * 2, 0);
        }
        return;
    }
    // ragged tile: element-wise stores with bounds checks
    if (!wave_on || !n_ok) return;
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int ml = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (m0 + ml < M) {
                float v = acc[mt][r] * osc[ml];
                if (R) v = fmaf(acc[mt][r], osc[ml], __uint_as_float((unsigned)R[(size_t)(m0 + ml) * N + n] << 16));
                fq_v2f pr = {v, 0.f};
                fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
                Y[(size_t)(m0 + ml) * N + n] = __builtin_bit_cast(unsigned short, pk[0]);
            }
        }
    }
}

// Workgroups [0, full_wgs) run whole tiles, the rest the half tiles of the tail round: one launch, so
// the halves start as soon as the first compute units run out of whole tiles.
__global__ __launch_bounds__(FQL_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void fq_gemm_large_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* Y, int M, int N, int K,
    int tiles_m, int tiles_n, int slots, int pm, const uint16_t* __restrict__ planes, unsigned full_wgs,
    int swiglu, const uint16_t* R, unsigned* rowmax) {
    extern __shared__ fq_v4i lds[];                       // 2 A stages (64 KiB) + 4 x 4 KiB of packed weights
    if (blockIdx.x < full_wgs)
        fql_item<8>(lds, blockIdx.x, A, a_scale, wp, gs, tscale, Y, M, N, K, tiles_m, tiles_n, slots, pm, planes, swiglu, R,
                    rowmax);
    else
        fql_item<4>(lds, blockIdx.x - full_wgs, A, a_scale, wp, gs, tscale, Y, M, N, K, tiles_m, tiles_n, slots, pm, planes,
                    swiglu, R, rowmax);
}

// The table mode of the same items (no zero-point planes).
__global__ __launch_bounds__(FQL_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void fq_gemm_large_lut_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* Y, int M, int N, int K,
    int tiles_m, int tiles_n, int slots, int pm, unsigned full_wgs, int swiglu, const uint16_t* R) {
    extern __shared__ fq_v4i lds[];
    if (blockIdx.x < full_wgs)
        fql_item<8, true>(lds, blockIdx.x, A, a_scale, wp, gs, tscale, Y, M, N, K, tiles_m, tiles_n, slots, pm, nullptr, swiglu, R);
    else
        fql_item<4, true>(lds, blockIdx.x - full_wgs, A, a_scale, wp, gs, tscale, Y, M, N, K, tiles_m, tiles_n, slots, pm, nullptr,
                          swiglu, R);
}

size_t fq_gemm_plane_bytes(int M, int K) {
    return (size_t)FQL_ZPLANES * fql_c2(K / FQ_GROUP) * (size_t)M * 16;
}

size_t fq_gemm_large_workspace_bytes(int M, int K) {
    return fq_gemm_plane_bytes(M, K) + (M <= FQ_KSPLIT_MAX_M ? FQ_KSPLIT_COUNTERS * sizeof(unsigned) : 0);
}

void fq_gemm_large_plan(int M, int N, int cus, int out[4]) {
    const int tiles_m = (M + FQL_BM - 1) / FQL_BM, tiles_n = (N + FQL_BN - 1) / FQL_BN;
    int slots = 2 * cus / FQL_XCDS;
    if (slots < 1) slots = 1;
    const int pm = tiles_m < 4 ? tiles_m : 4;
    out[0] = out[1] = out[2] = out[3] = 0;
    for (int x = 0; x < FQL_XCDS; ++x) {
        const fql_split sp = fql_xcd_split(x, tiles_m * tiles_n, slots);
        int m0, n0;
        for (int j = 0; j < sp.nfull; ++j)
            if (fql_locate<8>((unsigned)(j * FQL_XCDS + x), M, tiles_m, tiles_n, slots, pm, &m0, &n0))
                ++out[(m0 + 256 <= M && n0 + FQL_BN <= N && (N & 7) == 0) ? 0 : 1];
        for (int j = 0; j < sp.nhalf; ++j)
            if (fql_locate<4>((unsigned)(j * FQL_XCDS + x), M, tiles_m, tiles_n, slots, pm, &m0, &n0))
                ++out[(m0 + 128 <= M && n0 + FQL_BN <= N && (N & 7) == 0) ? 2 : 3];
    }
}

void fq_launch_zero_point(const uint8_t* A, void* workspace, int M, int K, hipStream_t stream) {
    hipLaunchKernelGGL(fq_zero_point_kernel, dim3((unsigned)M), dim3(256), 0, stream, A,
                       static_cast<uint16_t*>(workspace), M, K);
}

void fq_launch_gemm_large(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                          float tscale, uint16_t* Y, int M, int N, int K, void* workspace, bool prepared,
                          bool swiglu, const uint16_t* R, hipStream_t stream, bool lut, unsigned* rowmax) {
    static fq_device_once attr_once;
    fq_once_per_device(attr_once, [] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fq_gemm_large_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, FQL_LDS_BYTES);
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fq_gemm_large_lut_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, FQL_LDS_BYTES);
    });
    const int cus = fq_device_cus();
    uint16_t* planes = static_cast<uint16_t*>(workspace); // zero-point planes
    if (!prepared && !lut) fq_launch_zero_point(A, workspace, M, K, stream);
    const int tiles_m = (M + FQL_BM - 1) / FQL_BM, tiles_n = (N + FQL_BN - 1) / FQL_BN;
    int slots = 2 * cus / FQL_XCDS;                       // resident workgroups per XCD: two per compute unit
    if (slots < 1) slots = 1;
    int pm = 4;                                           // row tiles per panel: an XCD's 64 resident tiles then span
    if (pm > tiles_m) pm = tiles_m;                       // 4 row tiles x 16 channel tiles, 4 MiB of A and of W at K = 4096
    int max_full = 0, max_half = 0;
    for (int x = 0; x < FQL_XCDS; ++x) {
        const fql_split sp = fql_xcd_split(x, tiles_m * tiles_n, slots);
        max_full = sp.nfull > max_full ? sp.nfull : max_full;
        max_half = sp.nhalf > max_half ? sp.nhalf : max_half;
    }
    const unsigned full_wgs = (unsigned)(max_full * FQL_XCDS), half_wgs = (unsigned)(max_half * FQL_XCDS);
    if (lut) {
        hipLaunchKernelGGL(fq_gemm_large_lut_kernel, dim3(full_wgs + half_wgs), dim3(FQL_THREADS), FQL_LDS_BYTES, stream,
                           A, a_scale, wp, gs, tscale, Y, M, N, K, tiles_m, tiles_n, slots, pm, full_wgs, swiglu ? 1 : 0, R);
        return;
    }
    hipLaunchKernelGGL(fq_gemm_large_kernel, dim3(full_wgs + half_wgs), dim3(FQL_THREADS), FQL_LDS_BYTES, stream,
                       A, a_scale, wp, gs, tscale, Y, M, N, K, tiles_m, tiles_n, slots, pm, planes, full_wgs,
                       swiglu ? 1 : 0, R, swiglu ? rowmax : nullptr);
}
