// W4A8-FP GEMM for problems with too few output tiles to fill the chip (Sec. 3.1.1; same arithmetic and
// operand formats as fq_gemm_large.hip): a workgroup of 8 waves owns one tile of 32 * NMT rows x 32 * NW
// channels and splits K over KS = 8 / NW groups of NW waves.  Each K split streams its own A tiles through
// its own two LDS stages and its own packed weights, with the main loop of the large-M kernel (two chained
// v_mfma_f32_32x32x64_f8f6f4 per row tile and group, the group scale applied in FP32 to each group's
// partial sum); the splits' partial tiles are then added through LDS, each wave taking over NMT / KS row
// tiles, and the zero-point update and the epilogue finish those.  Two shapes are built:
//     NMT = 8, NW = 4, KS = 2   256 x 128 tiles, K halved: for M > 128 when whole tiles of that size would
//                               leave half the compute units idle (e.g. a down projection, N = 4096)
//     NMT = 4, NW = 2, KS = 4   128 x 64 tiles, K quartered: for 64 < M <= 512 (batched decode, chunked
//                               prefill), where 128-channel tiles are too few and the small-M kernels
//                               re-read the activations once per compute unit from L2
// One workgroup per compute unit (160 KiB of LDS, two waves per SIMD).
#include <type_traits>
#include "fq_common.h"
#include "fq_kernels.h"
#include "fq_gemm_large_common.h"

#define FQK_WAVES 8
#define FQK_THREADS (64 * FQK_WAVES)

namespace {

// LDS: KS * 2 stages of 32 * NMT rows x 128 bytes, then 8 x 4 KiB of packed weights; reused for the fold
// (8 waves x NMT tiles of 4 KiB, half of them at a time), the zero-point units and the output tile.
template <int NMT, int NW, int KS>
struct fqk_cfg {
    static constexpr int BM = 32 * NMT, BN = 32 * NW;
    static constexpr int STG = 8 * BM;                    // 16-byte chunks per A stage
    static constexpr int OUT_STRIDE = BN * 2 + 16;        // bytes per row of the output tile staged in LDS
    static constexpr int LOOP_LDS = KS * 2 * STG * 16 + FQK_WAVES * 4096;
    static constexpr int FOLD_LDS = FQK_WAVES * (NMT / 2 > 0 ? NMT / 2 : 1) * 4096;
    static constexpr int EPI_LDS = BM * OUT_STRIDE + 1024;
    static constexpr int LDS = LOOP_LDS > FOLD_LDS ? (LOOP_LDS > EPI_LDS ? LOOP_LDS : EPI_LDS)
                                                   : (FOLD_LDS > EPI_LDS ? FOLD_LDS : EPI_LDS);
    static_assert(NW * KS == FQK_WAVES && NMT % KS == 0 && (4 * NMT) % NW == 0 && 8 % NMT == 0, "shape");
    static_assert(LDS <= 160 * 1024, "LDS");
};

template <int NMT, int NW, int KS>
__global__ __launch_bounds__(FQK_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void fq_gemm_ksplit_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* Y, int M, int N, int K,
    int tiles_m, int tiles_n, int pm, const uint16_t* __restrict__ planes, const uint16_t* R) {
    typedef fqk_cfg<NMT, NW, KS> cfg;
    constexpr int NT = 4 * NMT / NW;                      // A transfers (8 rows each) per wave and stage
    constexpr int OWN = NMT / KS;                         // row tiles a wave finishes
    extern __shared__ fq_v4i lds[];
    const int G = K / FQ_GROUP;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nw = wave % NW, kw = wave / NW;             // position along the channels / which K split
    // which tile: XCD x = blockIdx % 8 runs a contiguous range of the tiles, panels of `pm` row tiles, row
    // tile fastest inside a panel, so that the tiles an XCD runs at one time share rows of A and channels of W
    int m0, n0;
    {
        const int x = blockIdx.x % FQL_XCDS, j = blockIdx.x / FQL_XCDS;
        const int ntiles = tiles_m * tiles_n, base = ntiles / FQL_XCDS, rem = ntiles % FQL_XCDS;
        if (j >= base + (x < rem ? 1 : 0)) return;
        const int t = x * base + (x < rem ? x : rem) + j;
        const int per_panel = pm * tiles_n;
        const int panel = t / per_panel, rest = t - panel * per_panel;
        const int ph = tiles_m - panel * pm < pm ? tiles_m - panel * pm : pm;
        const int tn = rest / ph, tm = panel * pm + (rest - tn * ph);
        m0 = tm * cfg::BM;
        n0 = tn * cfg::BN;
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
    // this split's groups: [gb, ge); every split runs `gper` steps, the surplus ones as ghosts with scale 0
    const int gper = (G + KS - 1) / KS;
    const int gb = kw * gper < G ? kw * gper : G;
    const int ge = gb + gper < G ? gb + gper : G;
    const int glast = G - 1;
    auto gclamp = [&](int j) { const int g = gb + j; return g < ge ? g : (ge > gb ? ge - 1 : glast); };

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

    // ---- prologue ----
    fq_v4i* stages = lds + kw * (2 * cfg::STG);           // this split's two A stages
    fq_v4i* wbuf = lds + KS * 2 * cfg::STG + wave * 256;  // this wave's two weight buffers
    fql_issue_a<NT>(rsA, abase, m0, K, stages, nw, gclamp(0));
    fql_issue_b(rsW, wbuf, lane16, wblk + (unsigned)gclamp(0) * 2048u);
    fql_issue_b(rsW, wbuf + 128, lane16, wblk + (unsigned)gclamp(1) * 2048u);
    unsigned psb[2];
    psb[0] = gsrow[gclamp(0)];
    psb[1] = gsrow[gclamp(1)];
    fq_v8i b0[2], b1[2];
    float sc[2];
    __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(0));
    b0[0] = fq_unpack_chunk(wbuf[lane]);
    b1[0] = fq_unpack_chunk(wbuf[64 + lane]);
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
            fql_issue_a<NT>(rsA, abase, m0, K, stages + (u ^ 1) * cfg::STG, nw, gclamp(j + 1));
            const unsigned qs = psb[u ^ 1];
            {
                const int g2 = gclamp(j + 2);
                fql_issue_b(rsW, wbuf + u * 128, lane16, wblk + (unsigned)g2 * 2048u);
                psb[u] = gsrow[g2];
            }
            __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(NT + 3));
            const fq_v4i* nxt = wbuf + (u ^ 1) * 128 + lane;
            const float s = sc[u];
            fq_v4i q = nxt[0];
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
                    if (h == 0) pt = FQ_MFMA(ac, b0[u], zero);
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
                    if (mt == NMT / 2 - 1 && h == 1) q = nxt[64];
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
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
    // NW waves' channels).  Half of the row tiles go through LDS at a time: every wave writes its partial
    // tiles of that half ([wave][tile of the half][16 registers][64 lanes]), and the waves that own one of them
    // add up the KS partials in the order of the splits (a fixed order: the result is deterministic).
    __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(0));           // ghost transfers have landed: the stages can be reused
    __syncthreads();
    fq_v16f fin[OWN];
    {
        float* fold = reinterpret_cast<float*>(lds);
        constexpr int HALF = NMT / 2 > 0 ? NMT / 2 : 1;   // row tiles per pass
        constexpr int PASSES = NMT / HALF;
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
            for (int t = 0; t < HALF; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) fold[((wave * HALF + t) * 16 + r) * 64 + lane] = acc[pass * HALF + t][r];
            __syncthreads();
#pragma unroll
            for (int i = 0; i < OWN; ++i) {
                const int mt = kw * OWN + i;              // (runtime: only used for addresses)
                if (mt / HALF == pass) {
                    const int t = mt - pass * HALF;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float v = 0.f;
#pragma unroll
                        for (int k2 = 0; k2 < KS; ++k2) v += fold[(((k2 * NW + nw) * HALF + t) * 16 + r) * 64 + lane];
                        fin[i][r] = v;
                    }
                }
            }
            __syncthreads();
        }
    }
    const int mown = m0 + kw * (32 * OWN);                // first row of this wave's own row tiles

    // ---- zero point: fin += Z * gscale^T over all groups (fp16 matrix cores), 8 units of Z per round ----
    {
        constexpr int RT = 32 * NMT;
        const __amdgpu_buffer_rsrc_t rsS = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t*>(gs), 0, (int)(((unsigned)N * (unsigned)G + 3u) & ~3u), 0x00020000);
        const unsigned srow = n_ok ? (unsigned)n * (unsigned)G : 0xFFFFFF00u;
        const bool unaligned_rows = (G & 3) != 0;
        const int hl = lane >> 5;
        const int rounds = (ZU + 7) >> 3;
        fql_issue_z<NMT, FQK_WAVES>(rsZ, lds, wave, lane, m0, M, 0, ZU < 8 ? ZU : 8);
        for (int r = 0; r < rounds; ++r) {
            const int u0 = 8 * r;
            const int nu = ZU - u0 < 8 ? ZU - u0 : 8;
            __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(0));
            __syncthreads();                              // round r has landed (stage r & 1)
            if (r + 1 < rounds)
                fql_issue_z<NMT, FQK_WAVES>(rsZ, lds + ((r + 1) & 1) * cfg::STG, wave, lane, m0, M, u0 + 8,
                                            ZU - u0 - 8 < 8 ? ZU - u0 - 8 : 8);
            fql_v8h sig[4];
#pragma unroll
            for (int ci = 0; ci < 4; ++ci) {
                const int c = ((u0 + 2 * ci) % C2) >> 1;
                const int g0 = 16 * c + 8 * hl;
                unsigned w[2] = {0u, 0u};
                if (2 * ci < nu) {
                    const unsigned o = srow + (unsigned)g0;
                    const unsigned ob = (n_ok && g0 < G) ? (o & ~3u) : 0xFFFFFF00u;
                    const unsigned d0 = __builtin_amdgcn_raw_buffer_load_b32(rsS, ob, 0, 0);
                    const unsigned d1 = __builtin_amdgcn_raw_buffer_load_b32(rsS, ob, 4, 0);
                    const unsigned d2 = unaligned_rows ? __builtin_amdgcn_raw_buffer_load_b32(rsS, ob, 8, 0) : 0u;
                    w[0] = __builtin_amdgcn_alignbyte(d1, d0, o & 3u);
                    w[1] = __builtin_amdgcn_alignbyte(d2, d1, o & 3u);
                    const int nv = G - g0;
                    if (nv < 4) w[0] &= nv <= 0 ? 0u : (1u << (8 * nv)) - 1u;
                    if (nv < 8) w[1] &= nv <= 4 ? 0u : (1u << (8 * (nv - 4))) - 1u;
                }
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
    for (int i = threadIdx.x; i < cfg::BM; i += FQK_THREADS) {
        const int m = m0 + i;
        osc[i] = a_scale[m < M ? m : M - 1] * (tscale * 512.0f);   // x 2^9: the weights were fed in units of 2^-9
    }
    __syncthreads();
    const bool full_tile = (m0 + cfg::BM <= M) && (n0 + cfg::BN <= N) && ((N & 7) == 0);
    if (full_tile) {
        // transpose through LDS so that every store instruction writes whole rows of the tile
        char* tile = reinterpret_cast<char*>(lds);
        char* wcol = tile + (kw * (32 * OWN) + 4 * (lane >> 5)) * cfg::OUT_STRIDE + (nw * 32 + (lane & 31)) * 2;
        const float* oscl = osc + kw * (32 * OWN) + 4 * (lane >> 5);
#pragma unroll
        for (int it = 0; it < 4 * OWN; ++it) {            // step it: rows 8 * it + 4 * (lane / 32) + 0..3 of the wave's own rows
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
    if (!wave_on || !n_ok) return;
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

template <int NMT, int NW, int KS>
void fqk_launch(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs, float tscale, uint16_t* Y,
                int M, int N, int K, const uint16_t* planes, const uint16_t* R, hipStream_t stream) {
    typedef fqk_cfg<NMT, NW, KS> cfg;
    static fq_device_once attr_once;                      // (one per template instance)
    fq_once_per_device(attr_once, [] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fq_gemm_ksplit_kernel<NMT, NW, KS>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, cfg::LDS);
    });
    const int tiles_m = (M + cfg::BM - 1) / cfg::BM, tiles_n = (N + cfg::BN - 1) / cfg::BN;
    const int ntiles = tiles_m * tiles_n;
    const int pm = tiles_m < 4 ? tiles_m : 4;
    const unsigned grid = (unsigned)((ntiles + FQL_XCDS - 1) / FQL_XCDS * FQL_XCDS);
    hipLaunchKernelGGL((fq_gemm_ksplit_kernel<NMT, NW, KS>), dim3(grid), dim3(FQK_THREADS), cfg::LDS, stream,
                       A, a_scale, wp, gs, tscale, Y, M, N, K, tiles_m, tiles_n, pm, planes, R);
}

}  // namespace

// Which shape of this kernel, if any, serves the problem better than the large-M kernel's own tiles:
// 0 = none, 1 = 256 x 128 tiles with K halved, 2 = 128 x 64 tiles with K quartered.
// Measured on MI355X (K = 4096 unless noted; large-M kernel -> this kernel): the 128 x 64 shape wins wherever its
// tiles fit one round of the compute units -- M = 128: N = 14336 28.3 -> 21.1 us, N = 11008 26.3 -> 19.4,
// N = 4096 21.0 -> 15.9 (K = 11008: 67.9 -> 40.7); M = 256 and 512 at N = 4096: 21.1 -> 16.4 and 21.9 -> 18.3 --
// and loses beyond that (M = 256, N = 14336: 29.4 -> 38.3; M = 512: 40.0 -> 72.9): a workgroup has one group of
// each K split in flight, so a tile is bound by the latency of its transfers, and several rounds of such tiles
// add up.  The 256 x 128 shape brought nothing on the shapes tried (down projection 2048 x 4096 x 11008: 105 us
// either way; 1024 x 4096 x 4096: 29.3 -> 37.1) and is not chosen automatically.
int fq_gemm_ksplit_choice(int M, int N, int K, int cus) {
    const int G = K / FQ_GROUP;
    if (M <= 64 || M > 512 || G < 8) return 0;
    return (long long)((M + 127) / 128) * ((N + 63) / 64) <= cus ? 2 : 0;
}

void fq_launch_gemm_ksplit(int choice, const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                           float tscale, uint16_t* Y, int M, int N, int K, void* workspace, bool prepared,
                           const uint16_t* R, hipStream_t stream) {
    if (!prepared) fq_launch_zero_point(A, workspace, M, K, stream);
    const uint16_t* planes = static_cast<const uint16_t*>(workspace);
    if (choice == 1) fqk_launch<8, 4, 2>(A, a_scale, wp, gs, tscale, Y, M, N, K, planes, R, stream);
    else             fqk_launch<4, 2, 4>(A, a_scale, wp, gs, tscale, Y, M, N, K, planes, R, stream);
}
