/*
 * CPU oracle for the W4A8-FP linear layer of FireQ (arXiv 2505.20839).
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must compute and is
 * used by the tests, the smoke check and the benchmark's cpu_baseline leg.  It shares no
 * code, header, table or constant generator with the HIP path and must never be called
 * from the product path.
 *
 * Everything is written out the slow, direct way, in FP64, with no blocking, fusion or
 * reordering beyond what the definitions below state:
 *
 *   operand formats          Sec. 2.1 (eq. 1, eq. 2) and Sec. 3.1:
 *                            INT4 weights, groups of 128 along K, one E4M3 scale per group;
 *                            E4M3 activations with one scale per token (row).
 *   linear layer             Sec. 2.2 eq. 3:  Y = X W^T.
 *   per-tensor scale         Sec. 3.1.2, Def. 3.2: weights were scaled by delta = 2^n before
 *                            quantisation, the GEMM output is multiplied by delta^-1
 *                            (here: w_tscale).
 *   FP8 constants            App. B (Lemma B.1: smallest subnormal 2^-9) and App. C.1
 *                            (overflow threshold 1.75 * 2^8 = 448): OCP E4M3, bias 7.
 *   INT4 range               Sec. 3.1.1 step 1: the table of dequantised values runs from
 *                            -8*sigma to 7*sigma, so codes are the 16 two's-complement
 *                            values -8..7.
 *
 *   Y[m,n] = a_scale[m] * w_tscale * sum_g dec8(gscale[n,g]) * sum_{k in g} dec8(A[m,k]) * q[n,k]
 *
 *   offline quantiser        Sec. 2.1 eq. 1 (group-wise INT4), Def. 3.1 (channel-wise absmean
 *                            scaling), Def. 3.2 (per-tensor scaling; its search for n is in
 *                            pts.py beside this file, in exact integer arithmetic),
 *                            Lemma B.1 (underflow of the FP8 group scale).
 *
 * Readings of points the paper leaves open (scale applied exactly in FP64 instead of a
 * rounded FP8 look-up table; one round-to-nearest-even to bf16 at the very end; the
 * activation scale is absmax/448 in FP32; an all-zero row gets scale 1) are stated at the
 * functions that take them.
 *
 * Build:  gcc -O2 -fopenmp -shared -fPIC -o libfq_oracle.so fq_oracle.c -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define FQO_GROUP 128

/* ---------------------------------------------------------------------------------------
 * E4M3 (OCP "e4m3fn": 1 sign, 4 exponent, 3 mantissa bits, bias 7, no infinities).
 * App. B, Lemma B.1 fixes the smallest subnormal at 2^-9; App. C.1 fixes the largest
 * finite value at 1.75 * 2^8 = 448.  Codes 0x7F and 0xFF are NaN.
 * ------------------------------------------------------------------------------------- */
double fqo_e4m3_decode(uint8_t code)
{
    int sign = (code >> 7) & 1;
    int expo = (code >> 3) & 0xF;
    int mant = code & 0x7;
    double v;
    if (expo == 0xF && mant == 0x7)
        return NAN;
    if (expo == 0)
        v = ldexp((double)mant, -9);              /* subnormal: mant/8 * 2^(1-7) */
    else
        v = ldexp(1.0 + (double)mant / 8.0, expo - 7);
    return sign ? -v : v;
}

/* Round a real number to the nearest E4M3 value, ties to the code with an even mantissa,
 * saturating at +-448 (never NaN for a finite input; NaN input gives the NaN code).
 * Done by definition: scan the 127 finite non-negative codes, keep the closest.          */
uint8_t fqo_e4m3_encode_rne(double x)
{
    if (isnan(x))
        return 0x7F;
    uint8_t sign = (uint8_t)(signbit(x) ? 0x80 : 0x00);
    double a = fabs(x);
    if (a >= 448.0)
        return (uint8_t)(sign | 0x7E);
    int best = 0;
    double best_d = a;                            /* distance to code 0 (value 0) */
    for (int c = 1; c <= 0x7E; ++c) {
        double d = fabs(a - fqo_e4m3_decode((uint8_t)c));
        if (d < best_d || (d == best_d && (c & 1) == 0 && (best & 1) == 1)) {
            best = c;
            best_d = d;
        }
    }
    return (uint8_t)(sign | best);
}

/* INT4: the low four bits of `nibble` read as a two's-complement number, -8..7
 * (Sec. 2.1 eq. 1 with b = 4; Sec. 3.1.1 step 1 lists -8*sigma .. 7*sigma).              */
int fqo_int4_decode(uint8_t nibble)
{
    int v = nibble & 0xF;
    return v >= 8 ? v - 16 : v;
}

/* bfloat16 <-> real.  A bf16 is the top 16 bits of an IEEE binary32.                      */
double fqo_bf16_decode(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Nearest bf16 to a real number, ties to even, overflow to infinity (IEEE behaviour).
 * Written from the definition: bf16 has 8 significand bits, so for a normal value the
 * spacing is 2^(e-7) with e = floor(log2|x|); the exponent range is that of binary32.   */
uint16_t fqo_bf16_encode_rne(double x)
{
    if (isnan(x))
        return 0x7FC0;
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000 : 0x0000);
    double a = fabs(x);
    if (a == 0.0)
        return sign;
    if (isinf(a))
        return (uint16_t)(sign | 0x7F80);
    int e;
    (void)frexp(a, &e);                           /* a = f * 2^e, f in [0.5,1)  */
    e -= 1;                                       /* a in [2^e, 2^(e+1))        */
    if (e < -126)
        e = -126;                                 /* subnormal spacing          */
    double ulp = ldexp(1.0, e - 7);
    double n = nearbyint(a / ulp);                /* default mode: ties to even; a/ulp is exact */
    double r = n * ulp;
    if (r >= ldexp(1.0, 128))
        return (uint16_t)(sign | 0x7F80);
    float f = (float)r;                           /* exact: r has <= 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(sign | (uint16_t)(u >> 16));
}

/* Size of one bf16 unit in the last place at the magnitude of x (for tolerances).        */
double fqo_bf16_ulp(double x)
{
    double a = fabs(x);
    int e;
    if (a == 0.0 || isnan(a) || isinf(a))
        return ldexp(1.0, -126 - 7);
    (void)frexp(a, &e);
    e -= 1;
    if (e < -126)
        e = -126;
    return ldexp(1.0, e - 7);
}

/* Array forms of the two bf16 helpers above (elementwise, nothing else).                  */
void fqo_bf16_encode_rne_array(const double *x, uint16_t *out, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        out[i] = fqo_bf16_encode_rne(x[i]);
}

void fqo_bf16_ulp_array(const double *x, double *out, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        out[i] = fqo_bf16_ulp(x[i]);
}

/* ---------------------------------------------------------------------------------------
 * The W4A8-FP GEMM (Sec. 2.2 eq. 3 with the operands of Sec. 2.1 / 3.1 and the output
 * scaling of Def. 3.2):
 *
 *   A       [M,K]      E4M3 codes, row-major
 *   a_scale [M]        per-token scale (the paper's beta), FP32
 *   q       [N,K]      INT4 codes, one int8 per code holding -8..7, row-major
 *   gscale  [N,K/128]  E4M3 codes, one per (output channel, group of 128 along K)
 *   w_tscale           per-tensor factor delta^-1
 *   Y       [M,N]      FP64 result, not rounded
 *   bound   [M,N]      optional (may be NULL): the same sum with every factor replaced by
 *                      its absolute value -- the forward-error scale used by the
 *                      per-element tolerance.
 *
 * Reading: the group scale multiplies the exact group sum (the paper's kernel instead
 * rounds q*sigma to FP8 in a 16-entry table before the multiply; the benchmark spec asks
 * for the exact formula).  Order: inner sum over the 128 k of a group, times the group
 * scale, summed over groups, times the two outer scales.  Returns 0, -1 on a bad shape,
 * -2 when the temporary FP64 copies of A and gscale cannot be allocated.
 * ------------------------------------------------------------------------------------- */
int fqo_w4a8_gemm(const uint8_t *A, const float *a_scale, const int8_t *q,
                  const uint8_t *gscale, float w_tscale,
                  double *Y, double *bound, int M, int N, int K)
{
    if (M < 0 || N < 0 || K < 0 || (K % FQO_GROUP) != 0)
        return -1;
    if (M == 0 || N == 0)
        return 0;
    const int G = K / FQO_GROUP;

    /* Decode the operands once into FP64 (pure look-ups, no arithmetic on them yet). */
    double *Ad = (double *)malloc((size_t)M * K * sizeof(double));
    double *Sd = (double *)malloc((size_t)N * (G > 0 ? G : 1) * sizeof(double));
    if (!Ad || !Sd) {
        free(Ad);
        free(Sd);
        return -2;
    }
    for (size_t i = 0; i < (size_t)M * K; ++i)
        Ad[i] = fqo_e4m3_decode(A[i]);
    for (size_t i = 0; i < (size_t)N * G; ++i)
        Sd[i] = fqo_e4m3_decode(gscale[i]);

    long m;
#pragma omp parallel for schedule(static)
    for (m = 0; m < M; ++m) {
        const double outer = (double)a_scale[m] * (double)w_tscale;
        for (int n = 0; n < N; ++n) {
            double y = 0.0, b = 0.0;
            for (int g = 0; g < G; ++g) {
                const double *a = Ad + (size_t)m * K + (size_t)g * FQO_GROUP;
                const int8_t *w = q + (size_t)n * K + (size_t)g * FQO_GROUP;
                double p = 0.0;
                for (int k = 0; k < FQO_GROUP; ++k)
                    p += a[k] * (double)w[k];
                y += Sd[(size_t)n * G + g] * p;
                if (bound) {
                    double pa = 0.0;
                    for (int k = 0; k < FQO_GROUP; ++k)
                        pa += fabs(a[k]) * fabs((double)w[k]);
                    b += fabs(Sd[(size_t)n * G + g]) * pa;
                }
            }
            Y[(size_t)m * N + n] = outer * y;
            if (bound)
                bound[(size_t)m * N + n] = fabs(outer) * b;
        }
    }
    free(Ad);
    free(Sd);
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * The GEMM as the paper's own kernel forms it (Sec. 3.1.1 steps 1 and 2): per group a table of
 * 16 FP8 entries {-8 sigma, ..., 7 sigma} is built from the FP8 group scale, every INT4 weight
 * is replaced by its table entry, and the matrix unit multiplies FP8 activations with these
 * FP8 weights; no scale is applied afterwards except the two outer factors:
 *
 *   Y[m,n] = a_scale[m] * w_tscale * sum_k dec8(A[m,k]) * dec8( E4M3( q[n,k] * dec8(gscale[n,g(k)]) ) )
 *
 * NOT the parity target of the library (which applies the scale exactly, see fqo_w4a8_gemm):
 * this variant exists to measure what the table's rounding costs in accuracy.
 * Reading: the entry q * sigma (exact in FP64: 4 x 4 significant bits) is rounded to E4M3
 * nearest-even, saturating at 448; sums in FP64 (the paper accumulates in FP32).
 * ------------------------------------------------------------------------------------- */
int fqo_w4a8_gemm_lut(const uint8_t *A, const float *a_scale, const int8_t *q,
                      const uint8_t *gscale, float w_tscale, double *Y, double *B, int M, int N, int K)
{
    if (M < 0 || N < 0 || K < 0 || (K % FQO_GROUP) != 0)
        return -1;
    if (M == 0 || N == 0)
        return 0;
    const int G = K / FQO_GROUP;
    double *Wd = (double *)malloc((size_t)N * K * sizeof(double));   /* table entries, decoded */
    if (!Wd)
        return -2;
    for (size_t n = 0; n < (size_t)N; ++n) {
        for (int g = 0; g < G; ++g) {
            double table[16];                                       /* index = INT4 code + 8 */
            const double sigma = fqo_e4m3_decode(gscale[n * (size_t)G + (size_t)g]);
            for (int c = -8; c <= 7; ++c)
                table[c + 8] = fqo_e4m3_decode(fqo_e4m3_encode_rne((double)c * sigma));
            for (int k = 0; k < FQO_GROUP; ++k) {
                const size_t idx = n * (size_t)K + (size_t)(g * FQO_GROUP + k);
                Wd[idx] = table[q[idx] + 8];
            }
        }
    }
    long m;
#pragma omp parallel for schedule(static)
    for (m = 0; m < M; ++m) {
        const double outer = (double)a_scale[m] * (double)w_tscale;
        for (int n = 0; n < N; ++n) {
            double y = 0.0, b = 0.0;                                /* b: the same sum over absolute values */
            for (int k = 0; k < K; ++k) {
                const double t = fqo_e4m3_decode(A[(size_t)m * K + k]) * Wd[(size_t)n * K + k];
                y += t;
                b += fabs(t);
            }
            Y[(size_t)m * N + n] = outer * y;
            if (B)
                B[(size_t)m * N + n] = fabs(outer) * b;
        }
    }
    free(Wd);
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * The gate/up pair of a feed-forward block with the epilogue fused (Sec. 3.1.1 step 3: the
 * kernel's epilogue applies the nonlinear activation, SiLU, and the element-wise
 * multiplication):
 *
 *   H[m,j] = SiLU(Yg[m,j]) * Yu[m,j],   SiLU(x) = x / (1 + exp(-x)),
 *
 * where Yg = row 2j and Yu = row 2j+1 of the W4A8-FP GEMM above (the weight matrix holds
 * the gate and up projections with their rows interleaved; N rows give N/2 outputs).
 *
 * Reading: the paper converts the GEMM result to BF16 before the epilogue; as for the plain
 * GEMM, the task's reading is FP32/FP64 throughout and one rounding at the very end, so
 * this function applies SiLU and the product to the unrounded sums.
 *
 * bound (may be NULL) [M,N/2]: first-order bound of what errors eg, eu of the two sums do
 * to H:  |dH| <= 1.1 |Yu| eg + |SiLU(Yg)| eu  (|SiLU'| <= 1.1), evaluated with eg, eu set
 * to the absolute-value bounds of the two sums.
 * Returns 0, -1 on a bad shape (N odd included), -2 when a temporary cannot be allocated.
 * ------------------------------------------------------------------------------------- */
int fqo_w4a8_gemm_swiglu(const uint8_t *A, const float *a_scale, const int8_t *q,
                         const uint8_t *gscale, float w_tscale,
                         double *H, double *bound, int M, int N, int K)
{
    if (M < 0 || N < 0 || (N & 1) || K < 0 || (K % FQO_GROUP) != 0)
        return -1;
    if (M == 0 || N == 0)
        return 0;
    double *Y = (double *)malloc((size_t)M * N * sizeof(double));
    double *B = (double *)malloc((size_t)M * N * sizeof(double));
    if (!Y || !B) {
        free(Y);
        free(B);
        return -2;
    }
    int rc = fqo_w4a8_gemm(A, a_scale, q, gscale, w_tscale, Y, B, M, N, K);
    if (rc == 0) {
        const int J = N / 2;
        for (size_t m = 0; m < (size_t)M; ++m) {
            for (int j = 0; j < J; ++j) {
                const double g = Y[m * N + 2 * j], u = Y[m * N + 2 * j + 1];
                const double silu = g / (1.0 + exp(-g));
                H[m * J + j] = silu * u;
                if (bound)
                    bound[m * J + j] = 1.1 * fabs(u) * B[m * N + 2 * j] + fabs(silu) * B[m * N + 2 * j + 1];
            }
        }
    }
    free(Y);
    free(B);
    return rc;
}

/* ---------------------------------------------------------------------------------------
 * The GEMM with the activation addition of the epilogue (Sec. 3.1.1 step 3 lists the addition
 * of activations: the residual stream added to the output of the attention-output and the
 * down projections, Fig. 1):
 *
 *   Y[m,n] = GEMM[m,n] + R[m,n],   R [M,N] bf16 bit patterns, row-major.
 *
 * Reading: as for the other epilogues the sum is formed on the unrounded GEMM result and
 * rounded once by the caller of this function (the paper adds in BF16 after a first
 * rounding of the GEMM result).  R is exact, so the error bound is that of the GEMM.
 * Returns what fqo_w4a8_gemm returns.
 * ------------------------------------------------------------------------------------- */
int fqo_w4a8_gemm_add(const uint8_t *A, const float *a_scale, const int8_t *q,
                      const uint8_t *gscale, float w_tscale, const uint16_t *R,
                      double *Y, double *bound, int M, int N, int K)
{
    int rc = fqo_w4a8_gemm(A, a_scale, q, gscale, w_tscale, Y, bound, M, N, K);
    if (rc != 0 || M == 0 || N == 0)
        return rc;
    for (size_t m = 0; m < (size_t)M; ++m)
        for (size_t n = 0; n < (size_t)N; ++n)
            Y[m * N + n] += fqo_bf16_decode(R[m * N + n]);
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Activation quantisation (Sec. 2.1 eq. 2):  A = FP8(x / beta), one beta per token.
 *
 *   X [M,K] bf16 bit patterns -> A [M,K] E4M3 codes, a_scale [M] FP32.
 *
 * Readings (the paper gives no formula for beta and no rounding mode):
 *   beta = absmax(row) / 448 rounded to FP32 (448 = the E4M3 maximum of App. C.1);
 *   an all-zero row takes beta = 1;  the quotient x/beta is rounded to FP32 (IEEE
 *   division) and then to E4M3, nearest-even, saturating.  Inputs are finite.
 * ------------------------------------------------------------------------------------- */
int fqo_quantize_act(const uint16_t *X, uint8_t *A, float *a_scale, int M, int K)
{
    if (M < 0 || K < 0)
        return -1;
    long m;
#pragma omp parallel for schedule(static)
    for (m = 0; m < M; ++m) {
        double amax = 0.0;
        for (int k = 0; k < K; ++k) {
            double v = fabs(fqo_bf16_decode(X[(size_t)m * K + k]));
            if (v > amax)
                amax = v;
        }
        float s = (amax == 0.0) ? 1.0f : (float)(amax / 448.0);
        a_scale[m] = s;
        for (int k = 0; k < K; ++k) {
            double x = fqo_bf16_decode(X[(size_t)m * K + k]);
            float quot = (float)(x / (double)s);   /* = IEEE binary32 division of two floats */
            A[(size_t)m * K + k] = fqo_e4m3_encode_rne((double)quot);
        }
    }
    return 0;
}

/* =======================================================================================
 * Offline weight quantisation (the step that produces the GEMM's weight operands).
 * ===================================================================================== */

/* Largest E4M3 value not above |x| in magnitude (rounding toward zero), saturating at 448.
 * This is the cast Lemma B.1 (App. B) describes for the group scale: a value below the
 * smallest subnormal 2^-9 becomes 0.  By definition: scan the finite non-negative codes.  */
uint8_t fqo_e4m3_encode_rtz(double x)
{
    if (isnan(x))
        return 0x7F;
    uint8_t sign = (uint8_t)(signbit(x) ? 0x80 : 0x00);
    double a = fabs(x);
    int best = 0;
    for (int c = 1; c <= 0x7E; ++c)
        if (fqo_e4m3_decode((uint8_t)c) <= a)
            best = c;                             /* decode is increasing in c on 0..0x7E */
    return (uint8_t)(sign | best);
}

/* Channel-wise absmean scaling (Sec. 3.1.2, Def. 3.1): W is [N,K] (output channel n, input
 * channel k; Y = X W^T), Lambda is diagonal over the K input channels and scales column k,
 *
 *   lambda[k] = target / absmean_n(W[n,k]),   absmean = (1/N) sum_n |W[n,k]|.
 *
 * Reading: a column that is entirely zero has no absmean to normalise; it keeps lambda = 1.
 * W holds bf16 bit patterns.  FP64 throughout.  Returns 0, -1 on a bad shape.               */
int fqo_cas_scales(const uint16_t *W, double target, double *lambda, int N, int K)
{
    if (N <= 0 || K <= 0)
        return -1;
    for (int k = 0; k < K; ++k) {
        double s = 0.0;
        for (int n = 0; n < N; ++n)
            s += fabs(fqo_bf16_decode(W[(size_t)n * K + k]));
        lambda[k] = (s == 0.0) ? 1.0 : target / (s / (double)N);
    }
    return 0;
}

/* The scaled weight the quantiser and the per-tensor search work on: bf16 W[n,k] times the
 * FP32 lambda[k] (NULL = no channel scaling), the product rounded once to FP32.  The product
 * of a bf16 and an FP32 number has at most 32 significant bits, so the FP64 product is exact
 * and the conversion below is the single rounding.                                          */
static float fqo_scaled_weight(const uint16_t *W, const float *lambda, size_t n, int k, int K)
{
    double w = fqo_bf16_decode(W[n * (size_t)K + (size_t)k]);
    return lambda ? (float)(w * (double)lambda[k]) : (float)w;
}

void fqo_scaled_weights(const uint16_t *W, const float *lambda, float *out, int N, int K)
{
    for (size_t n = 0; n < (size_t)N; ++n)
        for (int k = 0; k < K; ++k)
            out[n * (size_t)K + (size_t)k] = fqo_scaled_weight(W, lambda, n, k, K);
}

/* Group-wise INT4 quantisation with an FP8 scale (Sec. 2.1 eq. 1 with b = 4, on groups of 128
 * consecutive k of one output channel, Sec. 3.1), applied to v = scaled weight * 2^n_pts
 * (Def. 3.2: the matrix is multiplied by delta = 2^n before quantisation):
 *
 *   sigma    = max_group |v| / 7                       FP32 division
 *   sigma8   = E4M3(sigma)                             toward zero (Lemma B.1) or nearest-even
 *   q        = clamp(round(v / dec8(sigma8)), -8, 7)   FP32 division, ties to even
 *   sigma8 = 0  ->  q = 0 for the whole group          (Lemma B.1)
 *
 * Readings: eq. 1 gives no rounding rule for the quotient (nearest, ties to even, taken here)
 * and does not say how sigma becomes FP8.  Lemma B.1 states that a sigma below 2^-9 becomes 0,
 * which holds for rounding toward zero and not for rounding to nearest (2^-10 < sigma < 2^-9
 * would round up to 2^-9); sigma_rne = 0 takes the lemma's cast, sigma_rne = 1 the
 * nearest-even cast of the usual hardware converters.  The quotient can exceed 7 when the
 * cast lowers sigma, hence the clamp to the INT4 range of eq. 1.  |v| beyond 7 * 448 saturates
 * sigma8 at 448 (App. C.1: 448 is the overflow threshold).  Inputs are finite.
 * q [N,K] int8, gscale [N,K/128] E4M3 codes.  Returns 0, -1 on a bad shape.                   */
int fqo_quantize_weights(const uint16_t *W, const float *lambda, int n_pts, int sigma_rne,
                         int8_t *q, uint8_t *gscale, int N, int K)
{
    if (N < 0 || K <= 0 || (K % FQO_GROUP) != 0 || n_pts < 0 || n_pts > 126)
        return -1;
    const int G = K / FQO_GROUP;
    for (size_t n = 0; n < (size_t)N; ++n) {
        for (int g = 0; g < G; ++g) {
            float v[FQO_GROUP];
            float vmax = 0.0f;
            for (int i = 0; i < FQO_GROUP; ++i) {
                /* times 2^n: exact unless it overflows FP32, which finite sane weights do not */
                v[i] = ldexpf(fqo_scaled_weight(W, lambda, n, g * FQO_GROUP + i, K), n_pts);
                if (fabsf(v[i]) > vmax)
                    vmax = fabsf(v[i]);
            }
            const float sigma = (float)((double)vmax / 7.0);          /* = IEEE binary32 division */
            const double sc = sigma >= 448.0f ? 448.0 : (double)sigma;
            const uint8_t code = sigma_rne ? fqo_e4m3_encode_rne(sc) : fqo_e4m3_encode_rtz(sc);
            gscale[n * (size_t)G + (size_t)g] = code;
            const double s8 = fqo_e4m3_decode(code);
            for (int i = 0; i < FQO_GROUP; ++i) {
                int c = 0;
                if (s8 > 0.0) {
                    const float quot = (float)((double)v[i] / s8);    /* = IEEE binary32 division */
                    double r = nearbyint((double)quot);               /* default mode: ties to even */
                    if (r > 7.0) r = 7.0;
                    if (r < -8.0) r = -8.0;
                    c = (int)r;
                }
                q[n * (size_t)K + (size_t)(g * FQO_GROUP + i)] = (int8_t)c;
            }
        }
    }
    return 0;
}

/* Threads the parallel loops above will use (1 when built without OpenMP).               */
int fqo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------------------------------
 * Attention operands with an INT4 key/value cache and FP8 queries (Sec. 3.2.1: queries are
 * FP8, keys and values INT4, quantised per token -- each row, one token of one head, has its own
 * scaling factor sigma; Sec. 2.1: those factors are FP8, like the weights'; Sec. 3.1.1: the
 * INT4 x FP8 product also computes S = Q K^T and O = P V).  Heads are 128 wide, so a token's
 * row of one head is exactly one quantisation group.  For every head h (an independent
 * problem; "head" here is a key/value head of one sequence, R the query rows that attend
 * to it):
 *
 *   S[h,r,t] = out_scale * q_scale[h,r] * dec8(k_scale[h,t]) * sum_c dec8(Q[h,r,c]) * Kq[h,t,c]
 *   O[h,r,c] = p_scale[h,r] * sum_t dec8(P[h,r,t]) * dec8(v_scale[h,t]) * Vq[h,t,c]
 *
 * Q, P: E4M3 codes with one FP32 scale per row (eq. 2); Kq, Vq: INT4 codes -8..7, one int8
 * each, [H][T][128]; k_scale, v_scale: E4M3 codes [H][T]; out_scale: the 1/sqrt(d) of the
 * attention scores (any FP32).  Reading: the paper does not say where the per-token factor
 * of V enters O = P V (its own kernel folds every factor into a rounded FP8 table); here it
 * multiplies each term exactly, as the group scale does in the linear layers.
 * B (may be NULL) receives the same sums over absolute values.
 * ------------------------------------------------------------------------------------- */
#define FQO_HEAD 128

int fqo_kv4_scores(const uint8_t *Q, const float *q_scale, const int8_t *Kq, const uint8_t *k_scale,
                   float out_scale, double *S, double *B, int H, int R, int T)
{
    if (H < 0 || R < 0 || T < 0)
        return -1;
    long hr;
#pragma omp parallel for schedule(static)
    for (hr = 0; hr < (long)H * R; ++hr) {
        const long h = hr / R;
        const uint8_t *qrow = Q + (size_t)hr * FQO_HEAD;
        const double outer = (double)out_scale * (double)q_scale[hr];
        for (int t = 0; t < T; ++t) {
            const int8_t *krow = Kq + ((size_t)h * T + (size_t)t) * FQO_HEAD;
            double dot = 0.0, adot = 0.0;
            for (int c = 0; c < FQO_HEAD; ++c) {
                const double term = fqo_e4m3_decode(qrow[c]) * (double)fqo_int4_decode((uint8_t)krow[c]);
                dot += term;
                adot += fabs(term);
            }
            const double sigma = fqo_e4m3_decode(k_scale[(size_t)h * T + (size_t)t]);
            S[(size_t)hr * T + (size_t)t] = outer * (sigma * dot);
            if (B)
                B[(size_t)hr * T + (size_t)t] = fabs(outer) * (fabs(sigma) * adot);
        }
    }
    return 0;
}

int fqo_kv4_output(const uint8_t *P, const float *p_scale, const int8_t *Vq, const uint8_t *v_scale,
                   double *O, double *B, int H, int R, int T)
{
    if (H < 0 || R < 0 || T < 0)
        return -1;
    long hr;
#pragma omp parallel for schedule(static)
    for (hr = 0; hr < (long)H * R; ++hr) {
        const long h = hr / R;
        const uint8_t *prow = P + (size_t)hr * T;
        for (int c = 0; c < FQO_HEAD; ++c) {
            double sum = 0.0, asum = 0.0;
            for (int t = 0; t < T; ++t) {
                const double term = fqo_e4m3_decode(prow[t]) * fqo_e4m3_decode(v_scale[(size_t)h * T + (size_t)t]) *
                                    (double)fqo_int4_decode((uint8_t)Vq[((size_t)h * T + (size_t)t) * FQO_HEAD + c]);
                sum += term;
                asum += fabs(term);
            }
            O[(size_t)hr * FQO_HEAD + c] = (double)p_scale[hr] * sum;
            if (B)
                B[(size_t)hr * FQO_HEAD + c] = fabs((double)p_scale[hr]) * asum;
        }
    }
    return 0;
}
