// W4A8-FP GEMM for problems with too few output tiles to fill the chip (Sec. 3.1.1; same arithmetic and
// operand formats as fq_gemm_large.hip): a workgroup of 8 waves owns one tile of 32 * NMT rows x 32 * NW
// channels and splits K over KS = 8 / NW groups of NW waves.  Each K split streams its own A tiles through
// its own two LDS stages and its own packed weights (128 x 64 tiles: straight into registers, two groups
// ahead -- a lane consumes exactly the 32 bytes it loads), with the main loop of the large-M kernel (two chained
// v_mfma_f32_32x32x64_f8f6f4 per row tile and group, the group scale applied in FP32 to each group's
// partial sum); the splits' partial tiles are then added through LDS, each wave taking over NMT / KS row
// tiles, and the zero-point update and the epilogue finish those.  Two shapes are built:
//     NMT = 8, NW = 4, KS = 2   256 x 128 tiles, K halved: for M > 128 when whole tiles of that size would
//                               leave half the compute units idle (e.g. a down projection, N = 4096)
//     NMT = 4, NW = 2, KS = 4   128 x 64 tiles, K quartered: for 64 < M <= 512 (batched decode, chunked
//                               prefill), where 128-channel tiles are too few and the small-M kernels
//                               re-read the activations once per compute unit from L2
//     NMT = 2, NW = 2, KS = 4   64 x 64 tiles, the zero point through the matrix cores (no workspace): M just
//                               below 64 with many channels, where the M <= 64 kernel is slowest
// One workgroup per compute unit (64 to 160 KiB of LDS, two waves per SIMD).
//
// K slices: when even these tiles are fewer than the compute units, S workgroups share a tile, each taking a
// contiguous 1/S of the groups (and splitting that among its waves as above).  A workgroup's loop is bound by
// what one compute unit can pull from L2 (about 110 GB/s measured, and every step of a 128 x 64 tile moves
// 80 KiB for 8 matrix instructions per wave), so a tile finishes S times sooner.  Each slice writes its folded
// partial tile (FP32, in the accumulators' own layout) to the workspace and counts itself in; the workgroup that
// arrives last adds the S partial tiles in the order of the slices -- a fixed order, so the result does not
// depend on which one that is -- and goes on to the zero-point update and the epilogue; it leaves the counter at
// zero for the next call.  The S workgroups of a tile run on the same XCD, so the partial tiles stay in its L2.
#include <type_traits>
#include "fq_common.h"
#include "fq_kernels.h"
#include "fq_gemm_large_common.h"

#define FQK_WAVES 8
#define FQK_THREADS (64 * FQK_WAVES)

namespace {

// LDS: KS * 2 stages of 32 * NMT rows x 128 bytes, then (256 x 128 shape) 8 x 4 KiB of packed weights; reused for the fold
// (8 waves x NMT tiles of 4 KiB, all at once where they fit, else half of them at a time), the zero-point units and the output tile.
template <int NMT, int NW, int KS>
struct fqk_cfg {
    static constexpr int BM = 32 * NMT, BN = 32 * NW;
    static constexpr int STG = 8 * BM;                    // 16-byte chunks per A stage
    static constexpr int OUT_STRIDE = BN * 2 + 16;        // bytes per row of the output tile staged in LDS
    static constexpr bool WREG = NMT <= 4;                // packed weights through registers instead of LDS
    static constexpr int LOOP_LDS = KS * 2 * STG * 16 + (WREG ? 0 : FQK_WAVES * 4096);
    // row tiles that go through LDS at a time when the K splits' partial tiles are added: all of them where the
    // stages have room for 8 waves x NMT tiles of 4 KiB, else half
    static constexpr int HALF = FQK_WAVES * NMT * 4096 <= LOOP_LDS ? NMT : (NMT / 2 > 0 ? NMT / 2 : 1);
    static constexpr int FOLD_LDS = FQK_WAVES * HALF * 4096;
    static constexpr int EPI_LDS = BM * OUT_STRIDE + 1024;
    static constexpr int LDS = LOOP_LDS > FOLD_LDS ? (LOOP_LDS > EPI_LDS ? LOOP_LDS : EPI_LDS)
                                                   : (FOLD_LDS > EPI_LDS ? FOLD_LDS : EPI_LDS);
    static_assert(NW * KS == FQK_WAVES && (NMT % KS == 0 || KS % NMT == 0) && (4 * NMT) % NW == 0 && 8 % NMT == 0, "shape");
    static_assert(LDS <= 160 * 1024, "LDS");
};

// ZPM: the zero point comes out through one more matrix instruction per operand half against a constant operand
// (every byte -2^-6), as in the small-M kernels, instead of the Z planes of a workspace: for problems that have none.
template <int NMT, int NW, int KS, bool ZPM = false>
__global__ __launch_bounds__(FQK_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void fq_gemm_ksplit_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* Y, int M, int N, int K,
    int tiles_m, int tiles_n, int pm, const uint16_t* __restrict__ planes, const uint16_t* R,
    int S, unsigned* counters, float* partials) {
    typedef fqk_cfg<NMT, NW, KS> cfg;
    constexpr int NT = 4 * NMT / NW;                      // A transfers (8 rows each) per wave and stage
    constexpr int OWN = NMT >= KS ? NMT / KS : 1;         // row tiles a wave finishes (fewer row tiles than splits:
                                                          // the first NMT splits finish one each, the others none)
    extern __shared__ fq_v4i lds[];
    const int G = K / FQ_GROUP;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nw = wave % NW, kw = wave / NW;             // position along the channels / which K split
    // which tile: XCD x = blockIdx % 8 runs a contiguous range of the tiles, panels of `pm` row tiles, row
    // tile fastest inside a panel, so that the tiles an XCD runs at one time share rows of A and channels of W
    // (with K slices: workgroup j of an XCD is slice j % S of the XCD's tile j / S)
    int m0, n0, tile, slice;
    {
        const int x = blockIdx.x % FQL_XCDS, js = blockIdx.x / FQL_XCDS;
        const int j = js / S;
        slice = js - j * S;
        const int ntiles = tiles_m * tiles_n, base = ntiles / FQL_XCDS, rem = ntiles % FQL_XCDS;
        if (j >= base + (x < rem ? 1 : 0)) return;
        const int t = x * base + (x < rem ? x : rem) + j;
        tile = t;
        const int per_panel = pm * tiles_n;
        const int panel = t / per_panel, rest = t - panel * per_panel;
        const int ph = tiles_m - panel * pm < pm ? tiles_m - panel * pm : pm;
        const int tn = rest / ph, tm = panel * pm + (rest - tn * ph);
        m0 = tm * cfg::BM;
        n0 = tn * cfg::BN;
    }
    // the output factor of row m0 + threadIdx.x, fetched now so that the epilogue does not wait for it
    // (x 2^9: the weights are fed in units of 2^-9)
    static_assert(cfg::BM <= FQK_THREADS, "one row factor per thread");
    float row_factor = 0.f;
    if ((int)threadIdx.x < cfg::BM) {
        const int m = m0 + (int)threadIdx.x;
        row_factor = a_scale[m < M ? m : M - 1] * (tscale * 512.0f);
    }
    const int nw0 = n0 + nw * 32;                         // first output channel of this wave
    const bool wave_on = nw0 < N;                         // waves past N compute a duplicate tile and store nothing
    const int n = nw0 + (lane & 31);
    const bool n_ok = n < N;
    const int nt = wave_on ? (nw0 >> 5) : ((N - 1) >> 5);
    const unsigned wblk = (unsigned)nt * (unsigned)G * 2048u;
    const unsigned lane16 = (unsigned)lane * 16u;
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(A), 0, (int)((unsigned)M * (unsigned)K), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(wp), 0, (int)((unsigned)((N + 31) >> 5) * (unsigned)G * 2048u), 0x00020000);
    const int C2 = fql_c2(G), ZU = FQL_ZPLANES * C2;
    const __amdgpu_buffer_rsrc_t rsZ = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(planes), 0, (int)((unsigned)ZU * (unsigned)M * 16u), 0x00020000);
    const unsigned abase = fql_a_lane_base(nw, lane, K, NT);
    const uint8_t* gsrow = gs + (size_t)(n_ok ? n : N - 1) * G;
    // this workgroup's slice of the groups: [sb, se); this split's groups: [gb, ge); every split runs `gper`
    // steps, the surplus ones as ghosts with scale 0
    const int sper = (G + S - 1) / S;
    const int sb = slice * sper < G ? slice * sper : G;
    const int se = sb + sper < G ? sb + sper : G;
    const int gper = (se - sb + KS - 1) / KS;
    const int gb = sb + kw * gper < se ? sb + kw * gper : se;
    const int ge = gb + gper < se ? gb + gper : se;
    const int glast = G - 1;
    auto gclamp = [&](int j) { const int g = gb + j; return g < ge ? g : (ge > gb ? ge - 1 : glast); };
    // ghost steps request their operands out of range: zeros arrive at once and nothing is fetched
    auto ghost = [&](int j) { return gb + j < ge ? 0u : FQL_OOB; };

    const int r32 = lane & 31, sw = (r32 >> 1) & 7;
    const int o00 = r32 * 8 + ((2 * (lane >> 5)) ^ sw);
    const int o01 = o00 ^ 1, o10 = o00 ^ 4, o11 = o00 ^ 5;

    fq_v16f acc[NMT];
#pragma unroll
    for (int t = 0; t < NMT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    fq_v16f zero;
#pragma unroll
    for (int r = 0; r < 16; ++r) zero[r] = 0.f;
    fq_v8i zpb;
#pragma unroll
    for (int r = 0; r < 8; ++r) zpb[r] = (int)FQ_ZP_BYTES;

    // ---- prologue ----
    fq_v4i* stages = lds + kw * (2 * cfg::STG);           // this split's two A stages
    fq_v4i* wbuf = lds + KS * 2 * cfg::STG + wave * 256;  // this wave's two weight buffers
    // (both A stages are free at the start: the second group's tile travels with the first instead of one step later)
    fq_v4i wraw[2][2];                                    // (WREG) the packed weights of the next two groups
    auto load_w = [&](int slot, int j) __attribute__((always_inline)) {
        const unsigned off = wblk + (unsigned)gclamp(j) * 2048u;
        wraw[slot][0] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsW, lane16 | ghost(j), off, 0));
        wraw[slot][1] = __builtin_bit_cast(fq_v4i, __builtin_amdgcn_raw_buffer_load_b128(rsW, lane16 | ghost(j), off + 1024u, 0));
    };
    fql_issue_a<NT>(rsA, abase, m0, K, stages, nw, gclamp(0), ghost(0));
    if (cfg::WREG) {
        load_w(0, 0);
        load_w(1, 1);
    } else {
        fql_issue_b(rsW, wbuf, lane16 | ghost(0), wblk + (unsigned)gclamp(0) * 2048u);
        fql_issue_b(rsW, wbuf + 128, lane16 | ghost(1), wblk + (unsigned)gclamp(1) * 2048u);
    }
    fql_issue_a<NT>(rsA, abase, m0, K, stages + cfg::STG, nw, gclamp(1), ghost(1));
    unsigned psb[2];
    psb[0] = gsrow[gclamp(0)];
    psb[1] = gsrow[gclamp(1)];
    fq_v8i b0[2], b1[2];
    float sc[2];
    __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(0));
    b0[0] = fq_unpack_chunk(cfg::WREG ? wraw[0][0] : wbuf[lane]);
    b1[0] = fq_unpack_chunk(cfg::WREG ? wraw[0][1] : wbuf[64 + lane]);
    sc[0] = gb < ge ? __builtin_amdgcn_cvt_f32_fp8((int)psb[0], 0) : 0.f;
    b0[1] = b0[0]; b1[1] = b1[0]; sc[1] = 0.f;
    __syncthreads();

    fq_v16f pprev = zero;
    float sprev = 0.f;
    const int npairs = (gper + 1) >> 1;
    fq_v8i an = fql_join(stages[o00], stages[o01]);
    for (int p = 0; p < npairs; ++p) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int j = 2 * p + u;                      // step of this split; group gb + j
            const fq_v4i* cur = stages + u * cfg::STG;
            if (j > 0) fql_issue_a<NT>(rsA, abase, m0, K, stages + (u ^ 1) * cfg::STG, nw, gclamp(j + 1), ghost(j + 1));
            const unsigned qs = psb[u ^ 1];
            // (WREG: slot u held group j, unpacked during the last step; the compiler times the wait for slot u ^ 1)
            if (cfg::WREG) load_w(u, j + 2);
            else           fql_issue_b(rsW, wbuf + u * 128, lane16 | ghost(j + 2), wblk + (unsigned)gclamp(j + 2) * 2048u);
            psb[u] = gsrow[gclamp(j + 2)];
            if (!cfg::WREG) __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(NT + 3));
            const fq_v4i* nxt = wbuf + (u ^ 1) * 128 + lane;
            const float s = sc[u];
            fq_v4i q = cfg::WREG ? wraw[u ^ 1][0] : nxt[0];
            fq_v16f pt;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mt = 0; mt < NMT; ++mt) {
                const int tp = (mt + NMT - 1) % NMT;
                const float sp = (mt == 0) ? sprev : s;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const fq_v8i ac = an;
                    if (h == 0) {
                        an = fql_join(cur[mt * 256 + o10], cur[mt * 256 + o11]);
                    } else if (mt + 1 < NMT) {
                        an = fql_join(cur[(mt + 1) * 256 + o00], cur[(mt + 1) * 256 + o01]);
                    }
                    if (ZPM) pt = FQ_MFMA(ac, zpb, h == 0 ? zero : pt);   // -2^-6 * sum_k a_k in every column
                    if (h == 0) pt = FQ_MFMA(ac, b0[u], ZPM ? pt : zero);
                    else        pt = FQ_MFMA(ac, b1[u], pt);
#pragma unroll
                    for (int r = 8 * h; r < 8 * h + 8; ++r) acc[tp][r] = fmaf(sp, pprev[r], acc[tp][r]);
#pragma unroll
                    for (int e = 0; e < 8 / NMT; ++e) {
                        const int slot = (8 / NMT) * mt + e;
                        const unsigned w = (unsigned)q[slot & 3];
                        const int ev = (int)((h == 0 ? w : (w >> 4)) & 0x0F0F0F0Fu);
                        if (slot < 4) b0[u ^ 1][4 * h + (slot & 3)] = ev;
                        else          b1[u ^ 1][4 * h + (slot & 3)] = ev;
                    }
                    if (mt == NMT / 2 - 1 && h == 1) q = cfg::WREG ? wraw[u ^ 1][1] : nxt[64];
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, ZPM ? 2 : 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 24, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                pprev = pt;
            }
            sprev = s;
            {
                const float t = __builtin_amdgcn_cvt_f32_fp8((int)qs, 0);
                sc[u ^ 1] = (gb + j + 1 < ge) ? t : 0.f;
            }
            __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(3));
            __syncthreads();
            {
                const fq_v4i* nxs = stages + (u ^ 1) * cfg::STG;
                an = fql_join(nxs[o00], nxs[o01]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[NMT - 1][r] = fmaf(sprev, pprev[r], acc[NMT - 1][r]);

    // ---- fold: add the K splits' partial tiles through LDS ----
    // Row tiles are handed out in blocks: split kw finishes row tiles kw * OWN .. kw * OWN + OWN - 1 (for its
    // NW waves' channels).  All row tiles go through LDS at once where they fit, else half of them at a time: every
    // wave writes its partial tiles of the pass ([wave][tile of the pass][4 x 4 registers][64 lanes], 16 bytes per lane and access), and
    // the waves that own one of them add up the KS partials in the order of the splits (a fixed order: the result
    // is deterministic).
    __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(0));           // ghost transfers have landed: the stages can be reused
    __syncthreads();
    fq_v16f fin[OWN];
    const bool owner = kw * OWN < NMT;                    // this wave finishes row tiles kw * OWN ..
#pragma unroll
    for (int i = 0; i < OWN; ++i) fin[i] = zero;
    {
        fq_v4f* fold = reinterpret_cast<fq_v4f*>(lds);
        constexpr int HALF = cfg::HALF;                   // row tiles per pass
        constexpr int PASSES = NMT / HALF;
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
            for (int t = 0; t < HALF; ++t)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const fq_v16f& a = acc[pass * HALF + t];
                    fold[((wave * HALF + t) * 4 + r4) * 64 + lane] = (fq_v4f){a[4 * r4], a[4 * r4 + 1], a[4 * r4 + 2], a[4 * r4 + 3]};
                }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < OWN; ++i) {
                const int mt = kw * OWN + i;              // (runtime: only used for addresses)
                if (mt / HALF == pass) {
                    const int t = mt - pass * HALF;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        fq_v4f v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int k2 = 0; k2 < KS; ++k2) v += fold[(((k2 * NW + nw) * HALF + t) * 4 + r4) * 64 + lane];
#pragma unroll
                        for (int e = 0; e < 4; ++e) fin[i][4 * r4 + e] = v[e];
                    }
                }
            }
            __syncthreads();
        }
    }
    const int mown = m0 + kw * (32 * OWN);                // first row of this wave's own row tiles

    // the first round of zero-point units is requested now: it travels while the slices hand over
    const int rounds = ZPM ? 0 : (ZU + 7) >> 3;
    if (!ZPM) fql_issue_z<NMT, FQK_WAVES>(rsZ, lds, wave, lane, m0, M, 0, ZU < 8 ? ZU : 8);
    const __amdgpu_buffer_rsrc_t rsS = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(gs), 0, (int)(((unsigned)N * (unsigned)G + 3u) & ~3u), 0x00020000);
    const unsigned srow = n_ok ? (unsigned)n * (unsigned)G : FQL_OOB;    // channels past N read zeros
    fql_raw_scales zraw;                                  // the round's scale words, requested a round ahead
    if (!ZPM) fql_scales_issue(rsS, srow, n_ok, G, C2, 0, ZU < 8 ? ZU : 8, lane >> 5, zraw);

    // ---- K slices: hand the partial tile over; the workgroup that arrives last adds them up and goes on ----
    // The partial tiles and the counter are written and read with device-scope accesses (the sc1 bit: they go to
    // the level at which all XCDs agree and bypass the caches on the way back), and a wave's stores have been
    // acknowledged there (vmcnt = 0) before its workgroup counts itself in: a device-scope fence would do the same
    // by writing back the whole L2, once per workgroup, which cost more than the GEMM.  A tile's partial sums are
    // laid out [slice][wave][own row tile][4 x 4 registers][64 lanes], 16 bytes per lane and access.
    if (!ZPM && S > 1) {
        constexpr int SC1 = 16;                           // cache policy of the buffer builtins: device scope
        constexpr unsigned WAVE_BYTES = (unsigned)OWN * 4096u;
        const __amdgpu_buffer_rsrc_t rsP = __builtin_amdgcn_make_buffer_rsrc(
            partials + (size_t)tile * S * FQK_WAVES * (WAVE_BYTES / 4), 0, (int)((unsigned)S * FQK_WAVES * WAVE_BYTES), 0x00020000);
#pragma unroll
        for (int i = 0; i < OWN; ++i)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const fq_v4f v = {fin[i][4 * r4], fin[i][4 * r4 + 1], fin[i][4 * r4 + 2], fin[i][4 * r4 + 3]};
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(fq_v4i, v), rsP, lane16,
                                                       (unsigned)(slice * FQK_WAVES + wave) * WAVE_BYTES + (unsigned)(i * 4 + r4) * 1024u, SC1);
            }
        __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(0));       // this wave's partial sums have arrived ...
        __syncthreads();
        unsigned* flag = reinterpret_cast<unsigned*>(lds + cfg::LDS / 16 - 1);   // (past the zero-point units on their way)
        if (threadIdx.x == 0)                             // ... before the workgroup counts itself in
            flag[0] = __hip_atomic_fetch_add(&counters[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const unsigned arrived = *reinterpret_cast<volatile unsigned*>(flag);
        if (arrived != (unsigned)(S - 1)) return;
        if (threadIdx.x == 0)                             // every slice has counted: ready for the next call
            __hip_atomic_store(&counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // four slices' worth of loads are in flight at a time; the sum runs in the order of the slices
#pragma unroll
        for (int i = 0; i < OWN; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) fin[i][r] = 0.f;
            for (int sl0 = 0; sl0 < S; sl0 += 4) {
                fq_v4f part[4][4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int sl = sl0 + q < S ? sl0 + q : S - 1;       // (a repeat of the last slice, dropped below)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
                        part[q][r4] = __builtin_bit_cast(fq_v4f, __builtin_amdgcn_raw_buffer_load_b128(
                            rsP, lane16, (unsigned)(sl * FQK_WAVES + wave) * WAVE_BYTES + (unsigned)(i * 4 + r4) * 1024u, SC1));
                }
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (sl0 + q < S) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) fin[i][r] += part[q][r >> 2][r & 3];
                    }
            }
        }
    }

    // ---- zero point: fin += Z * gscale^T over all groups (fp16 matrix cores), 8 units of Z per round ----
    if (!ZPM) {
        constexpr int RT = 32 * NMT;
        const int hl = lane >> 5;
        for (int r = 0; r < rounds; ++r) {
            const int u0 = 8 * r;
            const int nu = ZU - u0 < 8 ? ZU - u0 : 8;
            __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(0));
            __syncthreads();                              // round r has landed (stage r & 1)
            fql_v8h sig[4];
            fql_scales_finish(zraw, srow, G, C2, u0, hl, sig);
            if (r + 1 < rounds) {
                const int nn = ZU - u0 - 8 < 8 ? ZU - u0 - 8 : 8;
                fql_issue_z<NMT, FQK_WAVES>(rsZ, lds + ((r + 1) & 1) * cfg::STG, wave, lane, m0, M, u0 + 8, nn);
                fql_scales_issue(rsS, srow, n_ok, G, C2, u0 + 8, nn, hl, zraw);
            }
            const fq_v4i* stage = lds + (r & 1) * cfg::STG;
#pragma unroll
            for (int ci = 0; ci < 4; ++ci) {
                if (2 * ci < nu) {
                    const fq_v4i* unit = stage + (2 * ci + hl) * RT + kw * (32 * OWN) + (lane & 31);
#pragma unroll
                    for (int i = 0; i < OWN; ++i)
                        fin[i] = FQ_MFMA_F16(__builtin_bit_cast(fql_v8h, unit[32 * i]), sig[ci], fin[i]);
                }
            }
        }
        __syncthreads();                                  // the last round has been read: LDS is free again
    }

    // ---- epilogue: per-token and per-tensor factors, the residual if any, one rounding to bf16, store ----
    float* osc = reinterpret_cast<float*>(reinterpret_cast<char*>(lds) + cfg::BM * cfg::OUT_STRIDE);
    if ((int)threadIdx.x < cfg::BM) osc[threadIdx.x] = row_factor;
    __syncthreads();
    const bool full_tile = (m0 + cfg::BM <= M) && (n0 + cfg::BN <= N) && ((N & 7) == 0);
    if (full_tile) {
        // transpose through LDS so that every store instruction writes whole rows of the tile
        char* tile = reinterpret_cast<char*>(lds);
        char* wcol = tile + (kw * (32 * OWN) + 4 * (lane >> 5)) * cfg::OUT_STRIDE + (nw * 32 + (lane & 31)) * 2;
        const float* oscl = osc + kw * (32 * OWN) + 4 * (lane >> 5);
#pragma unroll
        for (int it = 0; it < (owner ? 4 * OWN : 0); ++it) {   // step it: rows 8 * it + 4 * (lane / 32) + 0..3 of the wave's own rows
            const int i = it >> 2, jj = it & 3;
            const fq_v4f sc4 = *reinterpret_cast<const fq_v4f*>(&oscl[8 * it]);
#pragma unroll
            for (int e = 0; e < 4; e += 2) {
                fq_v2f pr = {fin[i][4 * jj + e] * sc4[e], fin[i][4 * jj + e + 1] * sc4[e + 1]};
                if (R) {                                  // this lane's residual values, in their own positions
                    const size_t ro = (size_t)(mown + 8 * it + 4 * (lane >> 5) + e) * N + n;
                    pr[0] = fmaf(fin[i][4 * jj + e], sc4[e], __uint_as_float((unsigned)R[ro] << 16));
                    pr[1] = fmaf(fin[i][4 * jj + e + 1], sc4[e + 1], __uint_as_float((unsigned)R[ro + N] << 16));
                }
                const unsigned pk = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, fq_v2bf));
                char* dst = wcol + (8 * it + e) * cfg::OUT_STRIDE;
                *reinterpret_cast<unsigned short*>(dst) = (unsigned short)pk;
                *reinterpret_cast<unsigned short*>(dst + cfg::OUT_STRIDE) = (unsigned short)(pk >> 16);
            }
        }
        __syncthreads();                                  // (all residual reads of the tile precede all of its stores)
        constexpr int RPW = cfg::BM / FQK_WAVES, LPR = cfg::BN / 8, RPI = 64 / LPR;
        const __amdgpu_buffer_rsrc_t rsY = __builtin_amdgcn_make_buffer_rsrc(
            Y + (size_t)(m0 + wave * RPW) * N + n0, 0, (int)((unsigned)RPW * (unsigned)N * 2u), 0x00020000);
        const unsigned ylane = (unsigned)(lane / LPR) * (unsigned)N * 2u + (unsigned)(lane % LPR) * 16u;
        const char* rd = tile + (wave * RPW + (lane / LPR)) * cfg::OUT_STRIDE + (lane % LPR) * 16;
#pragma unroll
        for (int j = 0; j < RPW / RPI; ++j) {
            const fq_v4i v = *reinterpret_cast<const fq_v4i*>(rd + RPI * j * cfg::OUT_STRIDE);
            __builtin_amdgcn_raw_buffer_store_b128(v, rsY, ylane, RPI * j * N * 2, 0);
        }
        return;
    }
    // ragged tile: element-wise, with bounds checks.  (In-place residual: an element is read and written by the
    // same lane, and nobody else touches it.)
    if (!wave_on || !n_ok || !owner) return;
#pragma unroll
    for (int i = 0; i < OWN; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int ml = kw * (32 * OWN) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (m0 + ml < M) {
                float v = fin[i][r] * osc[ml];
                if (R) v = fmaf(fin[i][r], osc[ml], __uint_as_float((unsigned)R[(size_t)(m0 + ml) * N + n] << 16));
                const fq_v2f pr = {v, 0.f};
                const fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
                Y[(size_t)(m0 + ml) * N + n] = __builtin_bit_cast(unsigned short, pk[0]);
            }
        }
    }
}

template <int NMT, int NW, int KS, bool ZPM = false>
void fqk_launch(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs, float tscale, uint16_t* Y,
                int M, int N, int K, const uint16_t* planes, const uint16_t* R, int S, unsigned* counters, float* partials,
                hipStream_t stream) {
    typedef fqk_cfg<NMT, NW, KS> cfg;
    static fq_device_once attr_once;                      // (one per template instance)
    fq_once_per_device(attr_once, [] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fq_gemm_ksplit_kernel<NMT, NW, KS, ZPM>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, cfg::LDS);
    });
    const int tiles_m = (M + cfg::BM - 1) / cfg::BM, tiles_n = (N + cfg::BN - 1) / cfg::BN;
    const int ntiles = tiles_m * tiles_n;
    const int pm = tiles_m < 4 ? tiles_m : 4;
    const unsigned grid = (unsigned)((ntiles + FQL_XCDS - 1) / FQL_XCDS * FQL_XCDS * S);
    hipLaunchKernelGGL((fq_gemm_ksplit_kernel<NMT, NW, KS, ZPM>), dim3(grid), dim3(FQK_THREADS), cfg::LDS, stream,
                       A, a_scale, wp, gs, tscale, Y, M, N, K, tiles_m, tiles_n, pm, planes, R, S, counters, partials);
}

}  // namespace

// Which shape of this kernel, if any, serves the problem better than the large-M kernel's own tiles:
// 0 = none, 1 = 256 x 128 tiles with K halved, 2 = 128 x 64 tiles with K quartered.
// Measured on MI355X (large-M kernel -> this kernel, prepared workspace): the 128 x 64 shape wins wherever its
// tiles fit one round of the compute units -- M = 128, K = 4096: N = 4096 20.7 -> 14.0 us, N = 11008 21.5 -> 16.5,
// N = 14336 23.6 -> 17.4; M = 128, N = 4096, K = 11008: 55.4 -> 21.7 (4 K slices); M = 512, N = 4096: K = 4096
// 21.1 -> 16.4, K = 11008 55.5 -> 38.9; 8192 x 8192 at M = 256: 49.3 -> 29.9 -- and loses beyond one round
// (M = 256, N = 11008: 23.4 -> 29.9; M = 512, N = 14336: 33.0 -> 59.4), except for a single row tile with a long K,
// where two rounds still win (M = 128: 20480 x 5120 46.7 -> 43.7, 28672 x 8192 74.5 -> 63.3; at K = 4096 the two
// are equal).  A step of a workgroup moves 80 KiB for 8 matrix instructions per wave and takes as long as that
// transfer (1.2 us measured), so one compute unit cannot run more than one round of such tiles well.
// The 256 x 128 shape brought nothing on the shapes tried (down projection 2048 x 4096 x 11008: 105 us
// either way; 1024 x 4096 x 4096: 29.3 -> 37.1) and is not chosen automatically.
int fq_gemm_ksplit_choice(int M, int N, int K, int cus) {
    const int G = K / FQ_GROUP;
    if (M <= 64 || M > FQ_KSPLIT_MAX_M || G < 8) return 0;
    const long long rounds = (M <= 128 && G >= 40) ? 2 : 1;
    return (long long)((M + 127) / 128) * ((N + 63) / 64) <= rounds * cus ? 2 : 0;
}

// K slices of the 128 x 64 shape: as many as fill the compute units, each with at least two groups per K split
// of its workgroup, none of them empty, at most 8; 1 where the shape is not the 128 x 64 one or the tiles exceed
// the counters.
int fq_gemm_ksplit_slices(int choice, int M, int N, int K, int cus) {
    if (choice != 2 || M > FQ_KSPLIT_MAX_M) return 1;
    const int G = K / FQ_GROUP;
    const long long tiles = (long long)((M + 127) / 128) * ((N + 63) / 64);
    if (tiles > FQ_KSPLIT_COUNTERS) return 1;
    int S = (int)(cus / tiles);
    if (S > G / 8) S = G / 8;
    if (S > 8) S = 8;
    if (S < 1) S = 1;
    while (S > 1 && (long long)((G + S - 1) / S) * (S - 1) >= G) --S;
    return S;
}

size_t fq_gemm_ksplit_partial_bytes(int choice, int M, int N, int K, int cus) {
    const int S = fq_gemm_ksplit_slices(choice, M, N, K, cus);
    if (S <= 1) return 0;
    return (size_t)S * (size_t)((M + 127) / 128) * (size_t)((N + 63) / 64) * (128u * 64u * sizeof(float));
}

void fq_launch_gemm_ksplit(int choice, const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                           float tscale, uint16_t* Y, int M, int N, int K, void* workspace, bool prepared,
                           const uint16_t* R, hipStream_t stream) {
    if (!prepared) fq_launch_zero_point(A, workspace, M, K, stream);
    const uint16_t* planes = static_cast<const uint16_t*>(workspace);
    // behind the planes: the tiles' arrival counters (zeroed by whatever prepared the workspace), then the partial tiles
    const size_t plane_bytes = fq_gemm_plane_bytes(M, K);
    unsigned* counters = reinterpret_cast<unsigned*>(static_cast<char*>(workspace) + plane_bytes);
    float* partials = reinterpret_cast<float*>(counters + FQ_KSPLIT_COUNTERS);
    const int S = fq_gemm_ksplit_slices(choice, M, N, K, fq_device_cus());
    if (choice == 1) fqk_launch<8, 4, 2>(A, a_scale, wp, gs, tscale, Y, M, N, K, planes, R, 1, counters, partials, stream);
    else             fqk_launch<4, 2, 4>(A, a_scale, wp, gs, tscale, Y, M, N, K, planes, R, S, counters, partials, stream);
}

// 16 < M <= 64 without a workspace: 64 x 64 tiles, K quartered, the zero point through the matrix cores.  Measured
// against the M <= 64 kernel (N = 14336, K = 4096): M = 64 16.2 -> 13.7 us, M = 48 13.3 -> 14.0, M = 33 12.1 -> 13.9 (its
// time hardly depends on M: 2 us until the first operands arrive, 7.4 us of loop at the rate the weights stream, 1.7 us
// of fold and epilogue); N = 11008: M = 64 14.9 -> 12.8; N = 4096 (64 tiles for 256 compute units): 11.7 -> 10.9;
// N = 4096, K = 11008: 25.7 -> 26.5.  So: the top of the range, at least half a round of tiles, K up to 8192.
bool fq_gemm_ksplit64_serves(int M, int N, int K, int cus) {
    const int tiles = (N + 63) / 64;
    return M > FQ_KSPLIT64_MIN_M && M <= 64 && K / FQ_GROUP >= 8 && K <= 8192 && tiles <= cus && 2 * tiles >= cus;
}

void fq_launch_gemm_ksplit64(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs, float tscale,
                             uint16_t* Y, int M, int N, int K, const uint16_t* R, hipStream_t stream) {
    fqk_launch<2, 2, 4, true>(A, a_scale, wp, gs, tscale, Y, M, N, K, nullptr, R, 1, nullptr, nullptr, stream);
}
