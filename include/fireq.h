/*
 * fireq.h -- C ABI of the W4A8-FP linear-layer library for AMD MI355X (gfx950).
 *
 * The library implements the INT4-weight x FP8-activation GEMM that runs every linear layer
 * of FireQ (arXiv 2505.20839, Sec. 3.1.1), the activation quantiser that feeds it
 * (Sec. 2.1 eq. 2), the offline weight quantiser (Sec. 2.1 eq. 1, Defs. 3.1 and 3.2) and the
 * weight packing the GEMM reads.
 *
 * Conventions for every entry point
 *   - All pointers are DEVICE pointers into memory owned by the caller.  The library
 *     allocates nothing, keeps no state between calls and never synchronises (one exception:
 *     fq_w4a8_gemm, which owns a workspace; see there): work is enqueued on `stream` (a
 *     hipStream_t passed as void*; NULL is the default stream) and the call returns at once.
 *   - Inputs are never written.  After a non-zero status the outputs are undefined.
 *   - No exception crosses this boundary; every function that can fail returns a status.
 *   - M = 0 (or N = 0 where it is an output width) is a successful no-op.
 *   - Base pointers must be 16-byte aligned (FQ_ERR_ALIGN otherwise), except a_scale and
 *     the int8 code array, which need only their natural alignment.
 *   - K must be a positive multiple of 128, the quantisation group (Sec. 3.1).
 */
#ifndef FIREQ_H
#define FIREQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    FQ_OK         = 0,
    FQ_ERR_NULL   = -1,  /* a required pointer is NULL                                        */
    FQ_ERR_SHAPE  = -2,  /* negative size, K == 0, K % 128 != 0, N == 0 with M > 0, or an     */
                         /* operand of the GEMM of 4 GiB or more (M*K, N*K/2, N*K/128, 512*N) */
    FQ_ERR_ALIGN  = -3,  /* a base pointer is not 16-byte aligned                             */
    FQ_ERR_LAUNCH = -4,  /* the HIP runtime reported an error when the kernel was launched    */
    FQ_ERR_MEMORY = -5   /* workspace missing or too small / own workspace could not be allocated */
};

#define FQ_GROUP 128     /* weights along K share one E4M3 scale per 128 (Sec. 3.1)           */

/*
 * Y = X W^T (Sec. 2.2 eq. 3) on quantised operands (Sec. 2.1, Sec. 3.1), with the per-tensor
 * factor of Def. 3.2 and the per-token factor of eq. 2 applied to the output:
 *
 *   Y[m,n] = bf16( a_scale[m] * w_tscale *
 *                  sum_g e4m3(w_gscale[n,g]) * sum_{k in group g} e4m3(A_fp8[m,k]) * q[n,k] )
 *
 * The group sums are accumulated in FP32 from exact FP8 x FP8 products, each group sum is
 * multiplied by its scale in FP32, and the result is rounded to bf16 once, to nearest even.
 *
 *   A_fp8      [M,K]  row-major OCP E4M3 codes (bias 7, max 448; NaN codes must not occur)
 *   a_scale    [M]    FP32 per-token scale (the paper's beta)
 *   Wq_packed         fq_packed_weight_bytes(N,K) bytes written by fq_pack_weights(N,K)
 *   w_gscale   [N,K/128] row-major OCP E4M3 codes, any finite value (zero, subnormal, negative)
 *   w_tscale          FP32 per-tensor factor (delta^-1 of Def. 3.2), by value
 *   Y_bf16     [M,N]  row-major bfloat16 bit patterns (output)
 *
 * For M > 64 the kernels need device scratch (the packed codes carry a zero point, and the
 * term that takes it out again, one number per row of A_fp8 and group, is computed first; for
 * 64 < M <= 512 with few output tiles, several workgroups share a tile along K and exchange
 * their FP32 partial tiles and arrival counters through it as well).
 * fq_w4a8_gemm_ws takes that scratch from the caller: `workspace` is device memory, 16-byte
 * aligned, at least fq_w4a8_gemm_workspace_bytes(M,N,K) bytes (0 = none needed, NULL is fine
 * then); it may be reused or freed once the work enqueued by the call has finished.  With
 * workspace_prepared == 0 the call fills the workspace itself (one more small kernel); with
 * workspace_prepared != 0 it takes the contents as they are, which must then have been written
 * by fq_quantize_act_ws for this very A_fp8 (same M and K); a prepared workspace serves any number of
 * GEMMs on that A_fp8, one after the other (calls that overlap in time on one workspace race on it).
 * That variant allocates nothing, keeps no state and never synchronises.  fq_w4a8_gemm is the same call on a workspace the library owns: one device
 * buffer for the whole process that grows (hipFree + hipMalloc, which synchronise the device)
 * when a call needs more than any call before it, so calls that overlap on different streams
 * race on it, and a first call must not be made under stream capture.
 */
size_t fq_w4a8_gemm_workspace_bytes(int M, int N, int K);
int fq_w4a8_gemm_ws(const uint8_t *A_fp8, const float *a_scale, const uint8_t *Wq_packed,
                    const uint8_t *w_gscale, float w_tscale, uint16_t *Y_bf16,
                    int M, int N, int K, void *workspace, size_t workspace_bytes,
                    int workspace_prepared, void *stream);
int fq_w4a8_gemm(const uint8_t *A_fp8, const float *a_scale, const uint8_t *Wq_packed,
                 const uint8_t *w_gscale, float w_tscale, uint16_t *Y_bf16,
                 int M, int N, int K, void *stream);

/*
 * fq_w4a8_gemm for callers that cannot allocate device memory and have none to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operands, result
 * and status codes as fq_w4a8_gemm_ws with workspace_prepared = 0, bit for bit; the scratch is a
 * fixed array inside the library's code object (fq_w4a8_gemm_static_max_workspace() bytes, 16 MiB,
 * one copy on every GPU the library is loaded on, held until the process ends).  The call
 * allocates nothing (no hipMalloc, hipFree or allocating library routine) and never synchronises.
 * A problem whose fq_w4a8_gemm_workspace_bytes(M,N,K) exceeds that size is refused with
 * FQ_ERR_MEMORY before anything is enqueued (M = 32768 with K = 16384 still fits).  All calls on
 * one GPU share that GPU's array: calls that overlap in time on one GPU (different streams) race
 * on it and give wrong results; calls on one stream, or ordered by events, are fine.  Nothing in
 * the array has to survive or be cleared between calls: each call writes every byte it reads.
 * The first call on a device looks the array's address up (hipGetSymbolAddress); make that call
 * outside stream capture.
 */
size_t fq_w4a8_gemm_static_max_workspace(void);
int fq_w4a8_gemm_static(const uint8_t *A_fp8, const float *a_scale, const uint8_t *Wq_packed,
                        const uint8_t *w_gscale, float w_tscale, uint16_t *Y_bf16,
                        int M, int N, int K, void *stream);

/*
 * The same GEMM in the paper's own table mode (Sec. 3.1.1 steps 1-2; App. B.1 compares it with exact
 * scales): per group and channel a 16-entry FP8 table T[q] = E4M3(q * sigma), q = -8..7 (nearest
 * even, saturating at +-448), the INT4 codes looked up in registers, and
 *
 *   Y[m,n] = bf16( a_scale[m] * w_tscale * sum_k e4m3(A_fp8[m,k]) * T_{n, k/128}[ q[n,k] ] )
 *
 * accumulated in FP32 over all of K with no separate group scale.  It is an approximation of
 * fq_w4a8_gemm (q * sigma keeps at most four significant bits: about 2 % relative error on
 * workload-like operands) and exists to measure that trade-off; the library's linear layers use
 * the exact form.  Operands, checks and status codes as for fq_w4a8_gemm; needs no workspace,
 * allocates nothing, keeps no state; every M is served by the large-M kernel.
 */
int fq_w4a8_gemm_lut(const uint8_t *A_fp8, const float *a_scale, const uint8_t *Wq_packed,
                     const uint8_t *w_gscale, float w_tscale, uint16_t *Y_bf16,
                     int M, int N, int K, void *stream);

/*
 * The gate and up projections of a feed-forward block in one call, with the epilogue fused
 * (Sec. 3.1.1 step 3: nonlinear activation and element-wise multiplication in the kernel's
 * epilogue).  The weight matrix holds the two projections with their rows interleaved: row 2j
 * of q (and of w_gscale) is gate channel j, row 2j+1 is up channel j; N counts these rows and
 * must be even.  With Y the result fq_w4a8_gemm_ws would give before rounding,
 *
 *   H[m,j] = bf16( SiLU(Y[m,2j]) * Y[m,2j+1] ),   SiLU(x) = x / (1 + exp(-x)),
 *
 * computed in FP32 and rounded once.  H_bf16 is [M,N/2] row-major.  Everything else
 * (operands, workspace, status codes) is as for fq_w4a8_gemm_ws.
 */
int fq_w4a8_gemm_swiglu_ws(const uint8_t *A_fp8, const float *a_scale, const uint8_t *Wq_packed,
                           const uint8_t *w_gscale, float w_tscale, uint16_t *H_bf16,
                           int M, int N, int K, void *workspace, size_t workspace_bytes,
                           int workspace_prepared, void *stream);

/*
 * The GEMM with the residual stream added in its epilogue (Sec. 3.1.1 step 3 lists the
 * addition of activations among the epilogue operations; Fig. 1: after the attention-output and the
 * down projections):
 *
 *   Y[m,n] = bf16( GEMM[m,n] + R[m,n] ),
 *
 * the sum formed in FP32 on the unrounded GEMM result of fq_w4a8_gemm_ws and rounded once.
 * R_bf16 is [M,N] row-major bfloat16 bit patterns, finite, 16-byte aligned.  R_bf16 may be
 * Y_bf16 itself (the residual stream updated in place); any other overlap of the two arrays is
 * FQ_ERR_SHAPE.  Everything else is as for fq_w4a8_gemm_ws.
 */
int fq_w4a8_gemm_add_ws(const uint8_t *A_fp8, const float *a_scale, const uint8_t *Wq_packed,
                        const uint8_t *w_gscale, float w_tscale, const uint16_t *R_bf16,
                        uint16_t *Y_bf16, int M, int N, int K, void *workspace,
                        size_t workspace_bytes, int workspace_prepared, void *stream);

/*
 * Per-token FP8 quantisation of activations (Sec. 2.1 eq. 2: A = FP8(x / beta)).
 *
 *   beta[m] = max_k |X[m,k]| / 448 in FP32 (1 for an all-zero row);
 *   A[m,k]  = E4M3 nearest-even of the FP32 quotient X[m,k] / beta[m], saturating at +-448.
 *
 *   X_bf16 [M,K] row-major bfloat16 bit patterns, finite;  A_fp8 [M,K];  a_scale [M].
 *   K here only has to be a positive multiple of 8.
 */
int fq_quantize_act(const uint16_t *X_bf16, uint8_t *A_fp8, float *a_scale,
                    int M, int K, void *stream);

/*
 * fq_quantize_act that also prepares the workspace of the GEMM that consumes A_fp8 (see
 * fq_w4a8_gemm_ws: pass workspace_prepared = 1 there).  K must be a multiple of 128 here;
 * `workspace` must hold at least fq_w4a8_gemm_workspace_bytes(M, N, K) bytes (the size does not
 * depend on N), 16-byte aligned; FQ_ERR_MEMORY otherwise.  Where that size is 0 (M <= 64) the call
 * is fq_quantize_act and `workspace` may be NULL.
 */
int fq_quantize_act_ws(const uint16_t *X_bf16, uint8_t *A_fp8, float *a_scale, int M, int K,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Offline weight packing (Sec. 3.1: INT4 weights in groups of 128).  The paper does not
 * define a nibble order; the packed order is private to this library, laid out for the
 * gfx950 FP8 MFMA operand, and versioned by fq_layout_version().
 *
 *   q [N,K] row-major, one int8 per INT4 code in -8..7 (only the low four bits are read).
 *   fq_packed_weight_bytes(N,K) = ceil(N/32)*32 * K/2 (rows are padded to a multiple of 32
 *   with code 0); returns 0 for an invalid shape.
 *   fq_unpack_weights is the exact inverse: unpack(pack(q)) == q for every code.
 */
size_t fq_packed_weight_bytes(int N, int K);
int fq_pack_weights(const int8_t *q, uint8_t *Wq_packed, int N, int K, void *stream);
int fq_unpack_weights(const uint8_t *Wq_packed, int8_t *q, int N, int K, void *stream);

/*
 * The fused gate/up layer of fq_w4a8_gemm_swiglu_ws whose output also leaves as the FP8 input of the
 * next layer (Sec. 3.1.1 step 3, Fig. 1: the feed-forward chain without a separate pass that searches
 * every row for its largest magnitude): H_bf16 [M, N/2] as before, and H_fp8 [M, N/2] (E4M3 codes,
 * 16-byte aligned) with h_scale [M] exactly as fq_quantize_act gives them for H_bf16, bit for bit.
 * The per-token scale of eq. 2 is a maximum over a whole row, which the workgroups of all the row's
 * tiles produce, so no code can be written before every tile is done: the GEMM's epilogue raises the
 * row maxima (kept in h_scale meanwhile) with one atomic per row and tile, and a second, element-wise
 * kernel turns H_bf16 into codes.  N/2 must be a multiple of 8.  With next_workspace != NULL
 * (fq_w4a8_gemm_workspace_bytes(M, N', N/2) bytes or more, N' the next layer's width; needs M > 64 and
 * N/2 a multiple of 128, at most 16384) that kernel also prepares the workspace of a GEMM that takes
 * H_fp8 as its input (workspace_prepared = 1 there), as fq_quantize_act_ws does.  For M <= 64 the call
 * runs the fused gate/up GEMM and the plain quantiser.  Other arguments, workspace and status codes as
 * for fq_w4a8_gemm_swiglu_ws; allocates nothing, keeps no state, never synchronises.
 */
int fq_w4a8_gemm_swiglu_quant_ws(const uint8_t *A_fp8, const float *a_scale, const uint8_t *Wq_packed,
                                 const uint8_t *w_gscale, float w_tscale, uint16_t *H_bf16,
                                 uint8_t *H_fp8, float *h_scale, int M, int N, int K,
                                 void *workspace, size_t workspace_bytes, int workspace_prepared,
                                 void *next_workspace, size_t next_workspace_bytes, void *stream);

/*
 * A whole linear layer from bfloat16 activations: the quantiser of Sec. 2.1 eq. 2 followed by the
 * GEMM of Sec. 2.2 eq. 3, with the result fq_quantize_act + fq_w4a8_gemm_ws give, bit for bit.
 * For M <= 6 and K <= 4096 (decode) it is ONE kernel: every workgroup quantises the few rows of
 * X itself while its weights are on their way, no codes or scales go through memory, and no
 * workspace is needed.  Otherwise the call runs the quantiser and the GEMM one after the other
 * and keeps the codes, the row scales and the GEMM's own scratch in `workspace`
 * (fq_w4a8_linear_workspace_bytes(M,N,K) bytes, 16-byte aligned; FQ_ERR_MEMORY if it is missing
 * or too small).  X_bf16 [M,K] row-major, finite, 16-byte aligned; the other operands as for
 * fq_w4a8_gemm_ws.  Allocates nothing, keeps no state, never synchronises.
 */
size_t fq_w4a8_linear_workspace_bytes(int M, int N, int K);
int fq_w4a8_linear_ws(const uint16_t *X_bf16, const uint8_t *Wq_packed, const uint8_t *w_gscale,
                      float w_tscale, uint16_t *Y_bf16, int M, int N, int K,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Offline weight quantisation: from a bfloat16 weight matrix W [N,K] (row n = output channel,
 * column k = input channel; Y = X W^T) to the operands of the GEMM.  Typical order:
 * fq_cas_scales, fq_pts_exponent, fq_quantize_weights, fq_pack_weights; the GEMM then takes
 * w_tscale = 2^-n.  All of it works on v[n,k] = W[n,k] * lambda[k] rounded once to FP32
 * (lambda == NULL: v = W).
 *
 * fq_cas_scales -- channel-wise absmean scaling (Sec. 3.1.2, Def. 3.1):
 *   lambda[k] = target / ((1/N) * sum_n |W[n,k]|), FP64 sums, result rounded to FP32; a channel
 *   that is zero throughout keeps lambda = 1.  lambda is [K] FP32 (output); target > 0.  The
 *   caller merges 1/lambda into whatever produces the layer's input, as the paper does.
 *
 * fq_pts_exponent -- per-tensor scaling (Def. 3.2, App. C.1): the smallest n >= 0 such that
 *   (1) every non-zero |v| * 2^n is at least 7 * 2^-9, the point from which the cumulative
 *       underflow S(v * 2^n) = sum max(0, 7 * 2^-9 - |v| * 2^n) no longer falls, or
 *   (2) some element satisfies 7 * 2^(5-n) <= |v| < 7 * 2^(6-n);
 *   capped at 126 so that 2^n stays an FP32 number.  n_out is DEVICE memory of 64 bytes,
 *   16-byte aligned: its first int receives n, the rest is scratch of the call.
 *
 * fq_quantize_weights -- group-wise INT4 with an FP8 scale (Sec. 2.1 eq. 1 with b = 4, groups
 *   of 128 along K, Sec. 3.1), on v * 2^n_pts (0 <= n_pts <= 126):
 *     sigma  = max_group |v * 2^n| / 7             (FP32 division), at most 448
 *     sigma8 = E4M3 of sigma, rounded toward zero when sigma_nearest == 0 -- the cast of App. B,
 *              Lemma B.1, under which a group with max < 7 * 2^-9 gets sigma8 = 0 -- or to
 *              nearest-even when sigma_nearest != 0
 *     q      = clamp(round_half_even(v * 2^n / sigma8), -8, 7)  (FP32 division); 0 where sigma8 = 0
 *   q [N,K] int8 (the input format of fq_pack_weights; 16-byte aligned here, like lambda),
 *   w_gscale [N,K/128] E4M3 codes.  Weights are finite.
 */
int fq_cas_scales(const uint16_t *W_bf16, float target, float *lambda, int N, int K, void *stream);
int fq_pts_exponent(const uint16_t *W_bf16, const float *lambda, int *n_out, int N, int K,
                    void *stream);
int fq_quantize_weights(const uint16_t *W_bf16, const float *lambda, int n_pts, int sigma_nearest,
                        int8_t *q, uint8_t *w_gscale, int N, int K, void *stream);

/*
 * Attention operands with an INT4 key/value cache and FP8 queries ("KV4/Q8", Sec. 3.2.1: queries
 * FP8, keys and values INT4 quantised per token, each token's row having its own scaling factor;
 * Sec. 2.1: those factors are FP8; Sec. 3.1.1: the INT4 x FP8 product also computes the attention
 * scores S = Q K^T and the output O = P V).  Heads are 128 wide: one token of one head is one
 * quantisation group.  A "head" below is one key/value head of one sequence, an independent
 * problem; R is the number of query rows that attend to it (grouped-query heads, batch rows).
 *
 *   S[h,r,t] = bf16( out_scale * q_scale[h,r] * e4m3(k_scale[h,t]) * sum_c e4m3(Q[h,r,c]) * Kq[h,t,c] )
 *   O[h,r,c] = bf16( p_scale[h,r] * sum_t e4m3(P[h,r,t]) * e4m3(v_scale[h,t]) * Vq[h,t,c] )
 *
 * Both are exact up to FP32 accumulation and one rounding to bf16: in S the token's factor
 * multiplies the finished FP32 sum; in O it sits on the summation index, and the kernel forms
 * P * sigma (at most 8 significant bits) and q exactly as bf16 operands of the matrix cores.
 *
 *   fq_kv4_pack      codes [H][T][128] int8 (INT4 codes -8..7, low four bits read) -> the packed
 *                    cache, fq_kv4_packed_bytes(H, T, values) bytes, 16-byte aligned.  values = 0:
 *                    a key cache (read by fq_kv4_scores), values != 0: a value cache (stored
 *                    transposed, tokens padded to a multiple of 128; read by fq_kv4_output).
 *                    fq_kv4_unpack is the exact inverse.
 *   fq_kv4_scores    Q_fp8 [H][R][128] E4M3 codes (16-byte aligned), q_scale [H][R] FP32,
 *                    k_scale [H][T] E4M3 codes (finite), out_scale FP32 (the 1/sqrt(128) of the
 *                    scores, or any factor), S_bf16 [H][R][T].  R <= 64.
 *   fq_kv4_output    P_fp8 [H][R][ldp] E4M3 codes, the first T of each row used (ldp >= T),
 *                    p_scale [H][R] FP32, v_scale [H][T], O_bf16 [H][R][128].  R <= 32, T >= 1.
 *                    Fastest when T and ldp are multiples of 16 and P_fp8 and v_scale 16-byte
 *                    aligned (16-byte loads); any other T, ldp and alignment is served too.
 * H <= 65535.  Status codes as above; a zero H, R (or T for the scores) is a successful no-op.
 */
size_t fq_kv4_packed_bytes(int H, int T, int values);
int fq_kv4_pack(const int8_t *codes, uint8_t *packed, int H, int T, int values, void *stream);
int fq_kv4_unpack(const uint8_t *packed, int8_t *codes, int H, int T, int values, void *stream);
int fq_kv4_scores(const uint8_t *Q_fp8, const float *q_scale, const uint8_t *K_packed,
                  const uint8_t *k_scale, float out_scale, uint16_t *S_bf16,
                  int H, int R, int T, void *stream);
int fq_kv4_output(const uint8_t *P_fp8, const float *p_scale, const uint8_t *V_packed,
                  const uint8_t *v_scale, uint16_t *O_bf16, int H, int R, int T, int ldp,
                  void *stream);

/*
 * Diagnostics (used by the tests; no kernel is launched).
 *
 * fq_w4a8_gemm_plan: how fq_w4a8_gemm_ws would run an M x N x K problem on a device with `cus`
 *   compute units (0 = the current device).  `plan` is HOST memory of 8 ints:
 *     plan[0]  kernel: 0 one-thread-per-output cross-check kernel, 1 the M <= 16 kernel, 2 the
 *              M <= 64 kernel, 3 the large-M kernel, 4 / 5 / 6 the K-split kernel with 256 x 128 /
 *              128 x 64 / 64 x 64 tiles (plain GEMM and residual form; the fused gate/up form
 *              always takes the large-M or the M <= 64 kernel), its number of tiles in plan[5] and
 *              the number of workgroups that share a tile along K in plan[6]
 *     plan[1]  large-M kernel: whole tiles (256 rows x 128 channels) written with whole-row stores
 *     plan[2]  whole tiles written element by element (a ragged edge, or N not a multiple of 8)
 *     plan[3], plan[4]  the same two counts for the 128-row half tiles of the last round
 *     plan[7]  0
 * fq_test_force_kernel: "simple", "small", "large" or "ksplit" makes every GEMM entry point use that kernel
 *   where it serves the shape; "" or NULL restores the choice by M.  The environment variable
 *   FQ_FORCE_KERNEL, read once when the library is loaded, sets the initial value.  Process-wide;
 *   meant for cross-checking the kernels against each other.
 * fq_diag_stream_read: a kernel that only reads `bytes` bytes (a multiple of 16) of device memory at
 *   `src` (16-byte aligned) and leaves fq_diag_stream_read_sink_bytes() bytes of checksums in the
 *   device buffer `sink`.  The benchmark times it on the packed weights to put the small-M GEMM's
 *   rate beside that of a plain streaming read of the same bytes.
 */
int fq_w4a8_gemm_plan(int M, int N, int K, int cus, int *plan);
size_t fq_diag_stream_read_sink_bytes(void);
int fq_diag_stream_read(const void *src, size_t bytes, void *sink, void *stream);
int fq_test_force_kernel(const char *name);

/* Changes whenever the byte order written by fq_pack_weights changes. */
int fq_layout_version(void);

/* Static, NUL-terminated description of a status code. */
const char *fq_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FIREQ_H */
