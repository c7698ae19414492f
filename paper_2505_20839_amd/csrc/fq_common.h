// Device-side helpers shared by the kernels of the W4A8-FP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define FQ_GROUP 128
#define FQ_LAYOUT_VERSION 2

typedef int   fq_v4i  __attribute__((ext_vector_type(4)));
typedef int   fq_v8i  __attribute__((ext_vector_type(8)));
typedef int   fq_v2i  __attribute__((ext_vector_type(2)));
typedef float fq_v16f __attribute__((ext_vector_type(16)));
typedef float fq_v4f  __attribute__((ext_vector_type(4)));
typedef float fq_v2f  __attribute__((ext_vector_type(2)));
typedef __bf16 fq_v2bf __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------------------------
// Packed weight layout (version 2), made for the B operand of v_mfma_f32_32x32x64_f8f6f4.
//
// Unit: one "block" per (tile of 32 output channels, group of 128 input channels) = 2048 bytes,
// blocks ordered [n/32][k/128].  A block is [h = 0,1][lane = 0..63][16 bytes]: `h` is the 64-wide
// half of the group that one MFMA consumes, `lane` = 32*kh + (n % 32) is the MFMA lane that needs
// the bytes, so a wave fetches one half with a single coalesced 16-byte load per lane.
// Inside the 16 bytes, byte 4*i + j holds two 4-bit codes:
//     low  nibble -> operand register i,     byte j :  k = 128*g + 64*h + 32*kh +      4*i + j
//     high nibble -> operand register 4 + i, byte j :  k = 128*g + 64*h + 32*kh + 16 + 4*i + j
// A 4-bit code is the weight with a zero point of 8:  code = q + 8  (0..15 for q = -8..7).
// Zero-extended to a byte it IS an E4M3 number: E4M3 subnormals (codes 0..7) and the first binade
// (codes 8..15) share one spacing, so byte c reads as c * 2^-9 exactly.  Unpacking is a mask and a
// shift, and the kernels compute  sum_k a_k * c_k * 2^-9  on the matrix cores and take the zero
// point out again as  - 2^-6 * sum_k a_k  per (row, group), a term that does not depend on the
// output channel.  Channels past N hold code 0.
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline size_t fq_block_offset(int nt, int g, int G) {
    return ((size_t)nt * (size_t)G + (size_t)g) * 2048u;
}

__host__ __device__ inline unsigned fq_code_from_q(int q) {       // q in -8..7 (low 4 bits used)
    q = (q << 28) >> 28;                                            // sign-extend the nibble
    return (unsigned)(q + 8);
}

__host__ __device__ inline int fq_q_from_code(unsigned code) {
    return (int)(code & 0xFu) - 8;
}

// Byte offset inside the packed buffer and nibble position (0 = low, 1 = high) of weight (n, k).
__host__ __device__ inline size_t fq_weight_byte(int n, int k, int G, int* hi) {
    int nt = n >> 5, n32 = n & 31;
    int g = k >> 7, kk = k & 127;
    int h = kk >> 6, kh = (kk >> 5) & 1, b = kk & 31;
    *hi = b >> 4;
    int ij = b & 15;
    return fq_block_offset(nt, g, G) + (size_t)h * 1024u + (size_t)(kh * 32 + n32) * 16u + (size_t)ij;
}

#ifdef __HIPCC__
// E4M3 byte of -2^-6: an all-(-2^-6) B operand turns an MFMA into the zero-point term
// -2^-6 * sum_k a_k, delivered in every output column.
#define FQ_ZP_BYTES 0x88888888

// One 16-byte packed chunk -> the 8 operand registers of one MFMA half (bytes c * 2^-9).
__device__ __forceinline__ fq_v8i fq_unpack_chunk(fq_v4i w) {
    fq_v8i r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        unsigned u = (unsigned)w[i];
        r[i]     = (int)(u & 0x0F0F0F0Fu);
        r[4 + i] = (int)((u >> 4) & 0x0F0F0F0Fu);
    }
    return r;
}

// OCP E4M3 byte -> float (exact), done with integer operations (no table, handles subnormals).
__device__ __forceinline__ float fq_e4m3_to_float(unsigned b) {
    unsigned sign = (b & 0x80u) << 24;
    unsigned em = b & 0x7Fu;
    float mag;
    if (em < 8u) mag = (float)em * 0.001953125f;                    // subnormal: m * 2^-9
    else         mag = __uint_as_float((em << 20) + 0x3C000000u);   // (e + 120) << 23 | m << 20
    return __uint_as_float(__float_as_uint(mag) | sign);
}

// SiLU(g) * u in FP32 (fused gate/up epilogue, Sec. 3.1.1 step 3): g / (1 + e^-g) * u with the
// hardware exponential and reciprocal (about 2 ulp of FP32 each, far below the bf16 step of the
// result); a very negative g gives e^-g = inf, 1 / inf = 0 and the result 0.
__device__ __forceinline__ float fq_silu_mul(float g, float u) {
    return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
}

// ---- activation quantisation (Sec. 2.1 eq. 2), shared by the quantiser kernel and the fused linear ----
// The two bf16 halves of a word as floats.
__device__ __forceinline__ float fq_bf16_hi(unsigned w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ float fq_bf16_lo(unsigned w) { return __uint_as_float(w << 16); }

// x / s.  FAST: from rcp = 1 / s with one exact residual step; the E4M3 code of the result equals that
// of the IEEE quotient for every finite bf16 x with |x| <= 448 * s and s in [2^-60, 2^60] (checked
// exhaustively by a host program); otherwise the full division.  FAST is a template argument so that
// the choice is made once per row (fq_scale_is_fast), not per element.
template <bool FAST>
__device__ __forceinline__ float fq_quotient(float x, float s, float rcp) {
    if (!FAST) return x / s;
    const float q = x * rcp;
    const float e = fmaf(-q, s, x);
    return copysignf(fmaf(e, rcp, q), x);
}

__device__ __forceinline__ bool fq_scale_is_fast(float s) { return s >= 0x1p-60f && s <= 0x1p60f; }

// Four quotients -> four E4M3 codes (nearest even, saturating at +-448 instead of becoming NaN).
template <bool FAST>
__device__ __forceinline__ unsigned fq_quant4(float a, float b, float c, float d, float s, float rcp) {
    a = fminf(fmaxf(fq_quotient<FAST>(a, s, rcp), -448.f), 448.f);
    b = fminf(fmaxf(fq_quotient<FAST>(b, s, rcp), -448.f), 448.f);
    c = fminf(fmaxf(fq_quotient<FAST>(c, s, rcp), -448.f), 448.f);
    d = fminf(fmaxf(fq_quotient<FAST>(d, s, rcp), -448.f), 448.f);
    int r = 0;
    r = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, r, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, r, true);
    return (unsigned)r;
}

// The eight bf16 of a 16-byte chunk -> eight E4M3 codes.
template <bool FAST>
__device__ __forceinline__ fq_v2i fq_quant8(fq_v4i v, float s, float rcp) {
    fq_v2i o;
    o[0] = (int)fq_quant4<FAST>(fq_bf16_lo(v[0]), fq_bf16_hi(v[0]), fq_bf16_lo(v[1]), fq_bf16_hi(v[1]), s, rcp);
    o[1] = (int)fq_quant4<FAST>(fq_bf16_lo(v[2]), fq_bf16_hi(v[2]), fq_bf16_lo(v[3]), fq_bf16_hi(v[3]), s, rcp);
    return o;
}

// float -> bf16 bits, round to nearest even (finite or infinite input; NaN not expected).
__device__ __forceinline__ unsigned fq_float_to_bf16(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
#endif
