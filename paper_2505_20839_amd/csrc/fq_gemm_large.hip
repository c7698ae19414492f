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
// A tiles go global -> LDS directly (global_load_lds_dwordx4, four stages of 32 KiB, two groups per
// barrier); packed weights go global -> registers (each wave reads only its own 32 channels) and
// are unpacked one group ahead, a slice under each pair of MFMAs.
#include "fq_common.h"
#include "fq_kernels.h"

#define FQL_THREADS 512
#define FQL_BM 256
#define FQL_STAGE_BYTES (FQL_BM * FQ_GROUP)          // 32 KiB: 256 rows x 128 E4M3 bytes
#define FQL_STAGE_CHUNKS (FQL_STAGE_BYTES / 16)
#define FQL_STAGES 4                                 // two pairs of groups: one in use, one in flight

#define FQ_MFMA(a, b, c) __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4((a), (b), (c), 0, 0, 0, 0, 0, 0)

namespace {

typedef __attribute__((address_space(3))) void* fql_lds_ptr;

// LDS layout of one A stage (one 128-wide group of 256 rows): row-major, 8 slots of 16 bytes per
// row; slot c of row r holds bytes 16*x .. 16*x+15 of the row's group with x = c ^ ((r >> 1) & 7).
// The XOR makes the operand reads (lane = row, fixed x) hit 16 different bank groups per 16 lanes,
// while the global->LDS transfer (buffer_load_dwordx4 ... lds, LDS address linear in the lane) still
// fetches whole 128-byte rows: 8 rows per instruction, 4 instructions per wave and stage.
// Addressing: the buffer descriptor covers all of A, so rows past M read as zero; the per-lane
// byte offset is fixed for the whole kernel (one register per transfer), the group travels in
// the scalar offset.
struct fql_a_addr {
    unsigned v[4];                                        // byte offset of each of the 4 transfers
};

__device__ __forceinline__ fql_a_addr fql_a_setup(int wave, int lane, int m0, int K) {
    const int row = wave * 32 + (lane >> 3);              // tile row of transfer 0
    const int c0 = (lane & 7) ^ ((row >> 1) & 7);         // == (lane & 7) ^ (lane >> 4): wave*32 drops out
    fql_a_addr a;
    // (the bounds check of a buffer load looks at this per-lane offset only, not at the scalar
    // offset, so the row must be part of it)
#pragma unroll
    for (int j = 0; j < 4; ++j)
        a.v[j] = (unsigned)(m0 + row + 8 * j) * (unsigned)K + (unsigned)(c0 ^ (4 * (j & 1))) * 16u;
    return a;
}

__device__ __forceinline__ void fql_issue_a(__amdgpu_buffer_rsrc_t rsrc, const fql_a_addr& a, fq_v4i* lds_stage,
                                            int wave, int g) {
    fq_v4i* dst = lds_stage + wave * 256;                 // this wave's 32 rows
    const int sg = g * FQ_GROUP;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (fql_lds_ptr)(dst + 64 * j), 16, a.v[j], sg, 0, 0);
}

// One group of this wave's packed weights (2 KiB: two halves of 64 lanes x 16 bytes) -> LDS.
__device__ __forceinline__ void fql_issue_b(__amdgpu_buffer_rsrc_t rsrc, fq_v4i* dst, unsigned lane16, unsigned blk_off) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (fql_lds_ptr)dst, 16, lane16, blk_off, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (fql_lds_ptr)(dst + 64), 16, lane16, blk_off + 1024u, 0, 0);
}

// s_waitcnt immediate (gfx9 encoding) that waits until at most n vector-memory transfers are pending
// and leaves the other counters alone.
#define FQL_WAIT_VM(n) ((((n) & 0xF) | (((n) >> 4) << 14)) | 0x0F70)

__device__ __forceinline__ fq_v8i fql_join(fq_v4i lo, fq_v4i hi) {
    fq_v8i r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return r;
}

}  // namespace

__global__ __launch_bounds__(FQL_THREADS) void fq_gemm_large_kernel(
    const uint8_t* __restrict__ A, const float* __restrict__ a_scale, const uint8_t* __restrict__ wp,
    const uint8_t* __restrict__ gs, float tscale, uint16_t* __restrict__ Y, int M, int N, int K) {
    extern __shared__ fq_v4i lds[];                       // 4 A stages (128 KiB) + 8 x 4 KiB of packed weights
    const int G = K / FQ_GROUP;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int m0 = blockIdx.y * FQL_BM;
    const int nw0 = blockIdx.x * 256 + wave * 32;         // first output channel of this wave
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
    const fql_a_addr aaddr = fql_a_setup(wave, lane, m0, K);
    const uint8_t* gsrow = gs + (size_t)(n_ok ? n : N - 1) * G;

    // operand read offsets (in chunks) of this lane inside a 32-row tile: (half h, part) -> slot
    const int r32 = lane & 31, sw = (r32 >> 1) & 7;
    const int o00 = r32 * 8 + ((2 * (lane >> 5)) ^ sw);   // h = 0, bytes 0..15 of the lane's 32
    const int o01 = o00 ^ 1, o10 = o00 ^ 4, o11 = o00 ^ 5;

    fq_v16f acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    fq_v16f zero;
#pragma unroll
    for (int r = 0; r < 16; ++r) zero[r] = 0.f;

    // ---- prologue ----
    fql_issue_a(rsA, aaddr, lds, wave, 0);
    fql_issue_a(rsA, aaddr, lds + FQL_STAGE_CHUNKS, wave, G > 1 ? 1 : 0);
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
    b0[0] = fq_unpack_chunk(wbuf[lane]);
    b1[0] = fq_unpack_chunk(wbuf[64 + lane]);
    sc[0] = __builtin_amdgcn_cvt_f32_fp8((int)psb[0], 0);
    b0[1] = b0[0]; b1[1] = b1[0]; sc[1] = 0.f;
    __syncthreads();

    fq_v16f pprev = zero;                                 // partial sums of the previous row tile
    float sprev = 0.f;                                    // and their group scale
    // Two groups per barrier.  Every load is unconditional (group indices are clamped at G-1
    // instead of skipped; a clamped "ghost" group is multiplied by a zero scale).
    //
    // The body is software-pipelined by hand, one step per 32x32 row tile: the two chained MFMAs of
    // the tile are issued back to back, then the step fetches the A operands of the next tile from
    // LDS and fills the MFMAs' shadow with the previous tile's scale-accumulate (16 v_fma) and an
    // eighth of the next group's unpack.  Keeping the non-MFMA part of a step longer than one MFMA
    // makes the two waves of a SIMD take turns on the matrix pipe instead of the older one hogging
    // it.  Scheduling barriers keep the compiler from undoing that order.
    const int npairs = (G + 1) >> 1;
    fq_v8i an0 = fql_join(lds[o00], lds[o01]);            // operands of the very first tile
    fq_v8i an1 = fql_join(lds[o10], lds[o11]);
    for (int p = 0; p < npairs; ++p) {
        {   // A tiles of the next pair -> the two stages the previous pair used (8 transfers)
            const int ga = 2 * p + 2 < G ? 2 * p + 2 : G - 1;
            const int gb = 2 * p + 3 < G ? 2 * p + 3 : G - 1;
            fq_v4i* nx = lds + ((p + 1) & 1) * 2 * FQL_STAGE_CHUNKS;
            fql_issue_a(rsA, aaddr, nx, wave, ga);
            fql_issue_a(rsA, aaddr, nx + FQL_STAGE_CHUNKS, wave, gb);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int g = 2 * p + u;
            const fq_v4i* cur = lds + ((p & 1) * 2 + u) * FQL_STAGE_CHUNKS;
            // Group g+1 sits in buffer u^1 (requested one group ago) and is unpacked slice by slice
            // under the MFMAs below; buffer u (group g, already unpacked) is refilled with group g+2.
            const unsigned qs = psb[u ^ 1];
            {
                const int g2 = g + 2 < G ? g + 2 : G - 1;
                fql_issue_b(rsW, wbuf + u * 128, lane16, wblk + (unsigned)g2 * 2048u);
                psb[u] = gsrow[g2];
            }
            // Transfers requested after group g+1's: its scale byte, (first group of a pair) the 8 A
            // transfers, and the 3 just above -> once at most that many are pending, g+1 has landed.
            if (u == 0) __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(11));
            else        __builtin_amdgcn_s_waitcnt(FQL_WAIT_VM(3));
            const fq_v4i* nxt = wbuf + (u ^ 1) * 128 + lane;
            const float s = sc[u];
            fq_v4i q = nxt[0];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) {
                const int tp = (mt + 7) & 7;
                const float sp = (mt == 0) ? sprev : s;   // row tile 7 of the previous group used the old scale
                const fq_v8i ac0 = an0, ac1 = an1;
                fq_v16f pt = FQ_MFMA(ac0, b0[u], zero);
                __builtin_amdgcn_s_setprio(1);            // mid-chain: win the pipe over a wave that is starting a tile
                pt = FQ_MFMA(ac1, b1[u], pt);
                __builtin_amdgcn_s_setprio(0);
                // A operands of the next tile (none after the last tile of a pair: the next pair's
                // stages are only complete after the barrier)
                if (mt < 7) {
                    an0 = fql_join(cur[(mt + 1) * 256 + o00], cur[(mt + 1) * 256 + o01]);
                    an1 = fql_join(cur[(mt + 1) * 256 + o10], cur[(mt + 1) * 256 + o11]);
                } else if (u == 0) {
                    an0 = fql_join(cur[FQL_STAGE_CHUNKS + o00], cur[FQL_STAGE_CHUNKS + o01]);
                    an1 = fql_join(cur[FQL_STAGE_CHUNKS + o10], cur[FQL_STAGE_CHUNKS + o11]);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[tp][r] = fmaf(sp, pprev[r], acc[tp][r]);
                {   // one eighth of the next group's unpack: one packed word
                    const unsigned w = (unsigned)q[mt & 3];
                    const int lo = (int)fq_codes_to_e4m3x4(w & 0x0F0F0F0Fu);
                    const int hi = (int)fq_codes_to_e4m3x4((w >> 4) & 0x0F0F0F0Fu);
                    if (mt < 4) { b0[u ^ 1][mt & 3] = lo; b0[u ^ 1][4 + (mt & 3)] = hi; }
                    else        { b1[u ^ 1][mt & 3] = lo; b1[u ^ 1][4 + (mt & 3)] = hi; }
                }
                if (mt == 3) q = nxt[64];
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA, raise priority,
                __builtin_amdgcn_sched_group_barrier(0x004, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA, lower priority
                __builtin_amdgcn_sched_group_barrier(0x004, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 5, 0);   // LDS reads for the next tile
                __builtin_amdgcn_sched_group_barrier(0x002, 32, 0);  // the MFMAs' shadow: VALU work
                __builtin_amdgcn_sched_barrier(0);
                pprev = pt;
            }
            sprev = s;
            {
                const float t = __builtin_amdgcn_cvt_f32_fp8((int)qs, 0);
                sc[u ^ 1] = (g + 1 < G) ? t : 0.f;
            }
        }
        __syncthreads();
        {
            const fq_v4i* nxs = lds + ((p + 1) & 1) * 2 * FQL_STAGE_CHUNKS;
            an0 = fql_join(nxs[o00], nxs[o01]);
            an1 = fql_join(nxs[o10], nxs[o11]);
        }
    }
    // last pending tile (row tile 7 of the last group)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[7][r] = fmaf(sprev, pprev[r], acc[7][r]);

    // ---- epilogue: per-token and per-tensor factors, one rounding to bf16, store ----
    // The stages are free now: bytes [0, 67584) become the output tile, [67584, 68608) the row factors.
    float* osc = reinterpret_cast<float*>(reinterpret_cast<char*>(lds) + 128 * 528);
    if (threadIdx.x < FQL_BM) {                           // x 2^9: the weights were fed as q * 2^-9
        int m = m0 + threadIdx.x;
        osc[threadIdx.x] = a_scale[m < M ? m : M - 1] * (tscale * 512.0f);
    }
    __syncthreads();
    const int nblk = blockIdx.x * 256;
    const bool full_tile = (m0 + FQL_BM <= M) && (nblk + 256 <= N) && ((N & 7) == 0);
    if (full_tile) {
        // Transpose through LDS so that every store instruction writes whole 512-byte rows.
        // Tile of 128 rows x 256 bf16, row stride 528 bytes; two passes (row tiles 0-3, 4-7).
        char* tile = reinterpret_cast<char*>(lds);
        const int colb = (wave * 32 + (lane & 31)) * 2;   // byte offset of this lane's column
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if (half) __syncthreads();                    // readers of the first pass are done
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int mt = half * 4 + t;
#pragma unroll
                for (int j = 0; j < 4; ++j) {             // rows 8j + 4*(lane/32) + 0..3 of the 32x32 tile
                    const int rl = 8 * j + 4 * (lane >> 5);
                    fq_v4f sc = *reinterpret_cast<const fq_v4f*>(&osc[mt * 32 + rl]);
#pragma unroll
                    for (int e = 0; e < 4; e += 2) {
                        float f0 = acc[mt][4 * j + e] * sc[e];          // row rl + e
                        float f1 = acc[mt][4 * j + e + 1] * sc[e + 1];  // row rl + e + 1
                        // lanes pair up: the even lane keeps row rl+e (its column and the next),
                        // the odd lane keeps row rl+e+1 (the previous column and its own)
                        float send = (lane & 1) ? f0 : f1;
                        float got = __int_as_float(__builtin_amdgcn_update_dpp(
                            0, __float_as_int(send), 0xB1, 0xF, 0xF, false));
                        fq_v2f pr = (lane & 1) ? (fq_v2f){got, f1} : (fq_v2f){f0, got};
                        fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
                        const int row = t * 32 + rl + e + (lane & 1);
                        *reinterpret_cast<fq_v2bf*>(tile + row * 528 + (colb & ~3)) = pk;
                    }
                }
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 8; ++j) {                 // wave w stores rows 16w .. 16w+15, two per instruction
                const int row = wave * 16 + 2 * j + (lane >> 5);
                fq_v4i v = *reinterpret_cast<const fq_v4i*>(tile + row * 528 + (lane & 31) * 16);
                const size_t m = (size_t)(m0 + half * 128 + row);
                *reinterpret_cast<fq_v4i*>(Y + m * N + nblk + (lane & 31) * 8) = v;
            }
        }
        return;
    }
    // ragged tile: element-wise stores with bounds checks
    if (!wave_on || !n_ok) return;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int ml = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (m0 + ml < M) {
                fq_v2f pr = {acc[mt][r] * osc[ml], 0.f};
                fq_v2bf pk = __builtin_convertvector(pr, fq_v2bf);
                Y[(size_t)(m0 + ml) * N + n] = __builtin_bit_cast(unsigned short, pk[0]);
            }
        }
    }
}

void fq_launch_gemm_large(const uint8_t* A, const float* a_scale, const uint8_t* wp, const uint8_t* gs,
                          float tscale, uint16_t* Y, int M, int N, int K, hipStream_t stream) {
    static bool attr_set = false;
    const int lds_bytes = FQL_STAGES * FQL_STAGE_BYTES + 8 * 4096;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fq_gemm_large_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        attr_set = true;
    }
    dim3 grid((unsigned)((N + 255) / 256), (unsigned)((M + FQL_BM - 1) / FQL_BM));
    hipLaunchKernelGGL(fq_gemm_large_kernel, grid, dim3(FQL_THREADS), lds_bytes, stream,
                       A, a_scale, wp, gs, tscale, Y, M, N, K);
}
