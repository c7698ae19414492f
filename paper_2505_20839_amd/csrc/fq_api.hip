// C entry points of the W4A8-FP library: argument validation, kernel choice, launch.
// Declarations and the contract of every call are in include/fireq.h.
#include "../../include/fireq.h"
#include "fq_common.h"
#include "fq_kernels.h"

#include <cstdlib>
#include <cstring>
#include <atomic>
#include <mutex>

// Scratch of fq_w4a8_gemm_static: one array per GPU the library runs on, part of the code object, held
// until the process ends.  In host code the name is only a handle for hipGetSymbolAddress.
#define FQ_STATIC_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char scratch[FQ_STATIC_SCRATCH_BYTES];

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int after_launch() { return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_LAUNCH; }

enum class GemmKernel { Auto, Simple, Large, Small, KSplit };

// FQ_FORCE_KERNEL=simple|large|small overrides the choice (tests use it to cross-check kernels).
GemmKernel parse_kernel(const char* e) {
    if (!e || !*e) return GemmKernel::Auto;
    if (!std::strcmp(e, "simple")) return GemmKernel::Simple;
    if (!std::strcmp(e, "large")) return GemmKernel::Large;
    if (!std::strcmp(e, "small")) return GemmKernel::Small;
    if (!std::strcmp(e, "ksplit")) return GemmKernel::KSplit;
    return GemmKernel::Auto;
}

// The environment is read when the library is loaded; fq_test_force_kernel changes the choice later.
std::atomic<int> g_forced{static_cast<int>(parse_kernel(std::getenv("FQ_FORCE_KERNEL")))};

GemmKernel forced_kernel() { return static_cast<GemmKernel>(g_forced.load(std::memory_order_relaxed)); }

// The GEMM kernels address every operand through 32-bit buffer offsets: each of A, the packed
// weights, the group scales and the workspace must stay below 4 GiB, and a band of 256 output rows too.
bool gemm_operands_addressable(int M, int N, int K) {
    const unsigned long long lim = 0xFFFFFF00ull, m = (unsigned long long)M, n = (unsigned long long)N,
                             k = (unsigned long long)K, g = k / FQ_GROUP;
    return m * k < lim && ((n + 31) / 32) * 32 * k / 2 < lim && n * g < lim && 256ull * n * 2 < lim &&
           (unsigned long long)fq_gemm_large_workspace_bytes(M, K) < lim;
}

// Argument checks shared by the GEMM entry points (M == 0 is valid and needs no pointers).
int check_gemm_args(const void* A, const void* a_scale, const void* W, const void* gs, const void* Y,
                    int M, int N, int K) {
    if (M < 0 || N < 0 || K <= 0 || (K % FQ_GROUP) != 0) return FQ_ERR_SHAPE;
    if (M == 0) return FQ_OK;
    if (N == 0) return FQ_ERR_SHAPE;
    if (!A || !a_scale || !W || !gs || !Y) return FQ_ERR_NULL;
    if (!aligned16(A) || !aligned16(W) || !aligned16(gs) || !aligned16(Y)) return FQ_ERR_ALIGN;
    if (!gemm_operands_addressable(M, N, K)) return FQ_ERR_SHAPE;
    return FQ_OK;
}

// Large also stands for the K-split kernel, which shares its workspace: ksplit_choice picks between the two.
GemmKernel choose_kernel(int M) {
    const GemmKernel k = forced_kernel();
    if (k == GemmKernel::KSplit) return GemmKernel::Large;
    return k != GemmKernel::Auto ? k : (M <= 64 ? GemmKernel::Small : GemmKernel::Large);
}

// 0: the large-M kernel's own tiles; 1, 2: a shape of the K-split kernel (never with the fused gate/up epilogue).
// Forcing "large" keeps the large-M kernel, forcing "ksplit" takes the K-split kernel wherever it can run.
int ksplit_choice(int M, int N, int K, bool swiglu) {
    const GemmKernel k = forced_kernel();
    if (swiglu || k == GemmKernel::Large || k == GemmKernel::Simple || k == GemmKernel::Small) return 0;
    if (k == GemmKernel::KSplit) return (K / FQ_GROUP >= 8) ? (M <= 512 ? 2 : 1) : 0;
    return fq_gemm_ksplit_choice(M, N, K, fq_device_cus());
}

// The top of 16 < M <= 64: the K-split kernel on 64 x 64 tiles instead of the M <= 64 kernel (never when a kernel is forced,
// never with the fused gate/up epilogue)
bool ksplit64_choice(int M, int N, int K, bool swiglu) {
    return !swiglu && forced_kernel() == GemmKernel::Auto && fq_gemm_ksplit64_serves(M, N, K, fq_device_cus());
}

}  // namespace

extern "C" {

int fq_layout_version(void) { return FQ_LAYOUT_VERSION; }

const char* fq_status_string(int status) {
    switch (status) {
        case FQ_OK: return "ok";
        case FQ_ERR_NULL: return "a required pointer is NULL";
        case FQ_ERR_SHAPE: return "invalid shape (sizes must be non-negative, K a positive multiple of 128)";
        case FQ_ERR_ALIGN: return "a base pointer is not 16-byte aligned";
        case FQ_ERR_LAUNCH: return "the HIP runtime rejected the kernel launch";
        case FQ_ERR_MEMORY: return "workspace missing or too small (fq_w4a8_gemm_static: the problem needs more than the "
                                   "built-in scratch holds), or the library could not allocate its own";
        default: return "unknown status";
    }
}

size_t fq_packed_weight_bytes(int N, int K) {
    if (N <= 0 || K <= 0 || (K % FQ_GROUP) != 0) return 0;
    return (size_t)((N + 31) / 32) * 32u * (size_t)K / 2u;
}

int fq_pack_weights(const int8_t* q, uint8_t* Wq_packed, int N, int K, void* stream) {
    if (N < 0 || K <= 0 || (K % FQ_GROUP) != 0) return FQ_ERR_SHAPE;
    if (N == 0) return FQ_OK;
    if (!q || !Wq_packed) return FQ_ERR_NULL;
    if (!aligned16(Wq_packed)) return FQ_ERR_ALIGN;
    fq_launch_pack(q, Wq_packed, N, K, static_cast<hipStream_t>(stream));
    return after_launch();
}

int fq_unpack_weights(const uint8_t* Wq_packed, int8_t* q, int N, int K, void* stream) {
    if (N < 0 || K <= 0 || (K % FQ_GROUP) != 0) return FQ_ERR_SHAPE;
    if (N == 0) return FQ_OK;
    if (!q || !Wq_packed) return FQ_ERR_NULL;
    if (!aligned16(Wq_packed)) return FQ_ERR_ALIGN;
    fq_launch_unpack(Wq_packed, q, N, K, static_cast<hipStream_t>(stream));
    return after_launch();
}

int fq_quantize_act(const uint16_t* X_bf16, uint8_t* A_fp8, float* a_scale, int M, int K, void* stream) {
    if (M < 0 || K <= 0 || (K % 8) != 0) return FQ_ERR_SHAPE;
    if (M == 0) return FQ_OK;
    if (!X_bf16 || !A_fp8 || !a_scale) return FQ_ERR_NULL;
    if (!aligned16(X_bf16) || !aligned16(A_fp8)) return FQ_ERR_ALIGN;
    if (((size_t)K * 2u) % 16u != 0 || ((size_t)K % 8u) != 0) return FQ_ERR_SHAPE;
    fq_launch_quantize(X_bf16, A_fp8, a_scale, M, K, static_cast<hipStream_t>(stream));
    return after_launch();
}

int fq_cas_scales(const uint16_t* W_bf16, float target, float* lambda, int N, int K, void* stream) {
    if (N <= 0 || K <= 0 || !(target > 0.f)) return FQ_ERR_SHAPE;
    if (!W_bf16 || !lambda) return FQ_ERR_NULL;
    fq_launch_cas_scales(W_bf16, target, lambda, N, K, static_cast<hipStream_t>(stream));
    return after_launch();
}

int fq_pts_exponent(const uint16_t* W_bf16, const float* lambda, int* n_out, int N, int K, void* stream) {
    if (N <= 0 || K <= 0 || (K % FQ_GROUP) != 0) return FQ_ERR_SHAPE;
    if (!W_bf16 || !n_out) return FQ_ERR_NULL;
    if (!aligned16(W_bf16) || !aligned16(n_out)) return FQ_ERR_ALIGN;
    fq_launch_pts_exponent(W_bf16, lambda, n_out, N, K, static_cast<hipStream_t>(stream));
    return after_launch();
}

int fq_quantize_weights(const uint16_t* W_bf16, const float* lambda, int n_pts, int sigma_nearest,
                        int8_t* q, uint8_t* w_gscale, int N, int K, void* stream) {
    if (N < 0 || K <= 0 || (K % FQ_GROUP) != 0 || n_pts < 0 || n_pts > 126) return FQ_ERR_SHAPE;
    if (N == 0) return FQ_OK;
    if (!W_bf16 || !q || !w_gscale) return FQ_ERR_NULL;
    if (!aligned16(W_bf16) || !aligned16(q) || (lambda && !aligned16(lambda))) return FQ_ERR_ALIGN;
    fq_launch_quantize_weights(W_bf16, lambda, n_pts, sigma_nearest != 0, q, w_gscale, N, K,
                               static_cast<hipStream_t>(stream));
    return after_launch();
}

int fq_test_force_kernel(const char* name) {
    g_forced.store(static_cast<int>(parse_kernel(name)), std::memory_order_relaxed);
    return FQ_OK;
}

size_t fq_diag_stream_read_sink_bytes(void) { return (size_t)fq_stream_read_blocks() * sizeof(unsigned); }

int fq_diag_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
    if (bytes == 0) return FQ_OK;
    if (!src || !sink) return FQ_ERR_NULL;
    if (!aligned16(src) || (bytes & 15u) != 0) return FQ_ERR_ALIGN;
    fq_launch_stream_read(src, bytes, static_cast<unsigned*>(sink), static_cast<hipStream_t>(stream));
    return after_launch();
}

int fq_w4a8_gemm_plan(int M, int N, int K, int cus, int* plan) {
    if (M <= 0 || N <= 0 || K <= 0 || (K % FQ_GROUP) != 0 || cus < 0) return FQ_ERR_SHAPE;
    if (!plan) return FQ_ERR_NULL;
    for (int i = 0; i < 8; ++i) plan[i] = 0;
    const GemmKernel k = choose_kernel(M);
    plan[0] = k == GemmKernel::Simple ? 0 : k == GemmKernel::Small ? (M <= 16 ? 1 : 2) : 3;
    if (k == GemmKernel::Small && forced_kernel() == GemmKernel::Auto &&
        fq_gemm_ksplit64_serves(M, N, K, cus > 0 ? cus : fq_device_cus())) {
        plan[0] = 6;
        plan[5] = (N + 63) / 64;
        plan[6] = 1;
    }
    if (k == GemmKernel::Large) {
        const int c = cus > 0 ? cus : fq_device_cus();
        const GemmKernel f = forced_kernel();
        const int ks = f == GemmKernel::Large ? 0
                     : f == GemmKernel::KSplit ? ((K / FQ_GROUP >= 8) ? (M <= 512 ? 2 : 1) : 0)
                                               : fq_gemm_ksplit_choice(M, N, K, c);
        if (ks != 0) {
            plan[0] = 3 + ks;
            plan[5] = ks == 1 ? ((M + 255) / 256) * ((N + 127) / 128) : ((M + 127) / 128) * ((N + 63) / 64);
            plan[6] = fq_gemm_ksplit_slices(ks, M, N, K, c);
        } else {
            fq_gemm_large_plan(M, N, c, plan + 1);
        }
    }
    return FQ_OK;
}

size_t fq_w4a8_gemm_workspace_bytes(int M, int N, int K) {
    if (M <= 0 || N <= 0 || K <= 0 || (K % FQ_GROUP) != 0) return 0;
    if (choose_kernel(M) != GemmKernel::Large) return 0;
    // (the fused gate/up epilogue never takes the K-split kernel and leaves the partial tiles unused)
    return fq_gemm_large_workspace_bytes(M, K) +
           fq_gemm_ksplit_partial_bytes(ksplit_choice(M, N, K, false), M, N, K, fq_device_cus());
}

int fq_quantize_act_ws(const uint16_t* X_bf16, uint8_t* A_fp8, float* a_scale, int M, int K,
                       void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || K <= 0 || (K % FQ_GROUP) != 0) return FQ_ERR_SHAPE;
    if (M == 0) return FQ_OK;
    if (!X_bf16 || !A_fp8 || !a_scale) return FQ_ERR_NULL;
    if (!aligned16(X_bf16) || !aligned16(A_fp8)) return FQ_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (choose_kernel(M) != GemmKernel::Large) {          // that GEMM takes no workspace: the plain quantiser
        fq_launch_quantize(X_bf16, A_fp8, a_scale, M, K, s);
        return after_launch();
    }
    if (!workspace || workspace_bytes < fq_gemm_large_workspace_bytes(M, K)) return FQ_ERR_MEMORY;
    if (!aligned16(workspace)) return FQ_ERR_ALIGN;
    if (fq_quantize_can_write_zero_point(K)) {
        fq_launch_quantize_zp(X_bf16, A_fp8, a_scale, M, K, workspace, s);
    } else {                                              // very long rows: two kernels
        fq_launch_quantize(X_bf16, A_fp8, a_scale, M, K, s);
        fq_launch_zero_point(A_fp8, workspace, M, K, s);
    }
    return after_launch();
}

namespace {

int gemm_ws(const uint8_t* A_fp8, const float* a_scale, const uint8_t* Wq_packed, const uint8_t* w_gscale,
            float w_tscale, uint16_t* out, int M, int N, int K, void* workspace, size_t workspace_bytes,
            int workspace_prepared, bool swiglu, const uint16_t* R, bool with_residual, void* stream) {
    const int rc = check_gemm_args(A_fp8, a_scale, Wq_packed, w_gscale, out, M, N, K);
    if (rc != FQ_OK) return rc;
    if (swiglu && (N & 1)) return FQ_ERR_SHAPE;
    if (M == 0) return FQ_OK;
    if (with_residual) {
        if (!R) return FQ_ERR_NULL;
        if (!aligned16(R)) return FQ_ERR_ALIGN;
        if (R != out) {                                   // the very same array is fine, a shifted overlap is not
            const uintptr_t r0 = reinterpret_cast<uintptr_t>(R), y0 = reinterpret_cast<uintptr_t>(out);
            const uintptr_t bytes = (uintptr_t)M * (uintptr_t)N * 2u;
            if (r0 < y0 + bytes && y0 < r0 + bytes) return FQ_ERR_SHAPE;
        }
    }
    const size_t need = fq_w4a8_gemm_workspace_bytes(M, N, K);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return FQ_ERR_MEMORY;
        if (!aligned16(workspace)) return FQ_ERR_ALIGN;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (choose_kernel(M)) {
        case GemmKernel::Simple:
            fq_launch_gemm_simple(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, out, M, N, K, swiglu, R, s);
            break;
        case GemmKernel::Small:
            if (ksplit64_choice(M, N, K, swiglu))
                fq_launch_gemm_ksplit64(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, out, M, N, K, R, s);
            else if (!fq_launch_gemm_small(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, out, M, N, K, swiglu, R, s))
                fq_launch_gemm_simple(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, out, M, N, K, swiglu, R, s);
            break;
        default: {
            const int ks = ksplit_choice(M, N, K, swiglu);
            if (ks != 0)
                fq_launch_gemm_ksplit(ks, A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, out, M, N, K, workspace,
                                      workspace_prepared != 0, R, s);
            else
                fq_launch_gemm_large(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, out, M, N, K, workspace,
                                     workspace_prepared != 0, swiglu, R, s);
            break;
        }
    }
    return after_launch();
}

}  // namespace

int fq_w4a8_gemm_ws(const uint8_t* A_fp8, const float* a_scale, const uint8_t* Wq_packed,
                    const uint8_t* w_gscale, float w_tscale, uint16_t* Y_bf16,
                    int M, int N, int K, void* workspace, size_t workspace_bytes, int workspace_prepared,
                    void* stream) {
    return gemm_ws(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, Y_bf16, M, N, K, workspace, workspace_bytes,
                   workspace_prepared, false, nullptr, false, stream);
}

int fq_w4a8_gemm_add_ws(const uint8_t* A_fp8, const float* a_scale, const uint8_t* Wq_packed,
                        const uint8_t* w_gscale, float w_tscale, const uint16_t* R_bf16, uint16_t* Y_bf16,
                        int M, int N, int K, void* workspace, size_t workspace_bytes, int workspace_prepared,
                        void* stream) {
    return gemm_ws(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, Y_bf16, M, N, K, workspace, workspace_bytes,
                   workspace_prepared, false, R_bf16, true, stream);
}

int fq_w4a8_gemm_swiglu_ws(const uint8_t* A_fp8, const float* a_scale, const uint8_t* Wq_packed,
                           const uint8_t* w_gscale, float w_tscale, uint16_t* H_bf16,
                           int M, int N, int K, void* workspace, size_t workspace_bytes, int workspace_prepared,
                           void* stream) {
    return gemm_ws(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, H_bf16, M, N, K, workspace, workspace_bytes,
                   workspace_prepared, true, nullptr, false, stream);
}

int fq_w4a8_gemm_swiglu_quant_ws(const uint8_t* A_fp8, const float* a_scale, const uint8_t* Wq_packed,
                                 const uint8_t* w_gscale, float w_tscale, uint16_t* H_bf16,
                                 uint8_t* H_fp8, float* h_scale, int M, int N, int K,
                                 void* workspace, size_t workspace_bytes, int workspace_prepared,
                                 void* next_workspace, size_t next_workspace_bytes, void* stream) {
    const int rc = check_gemm_args(A_fp8, a_scale, Wq_packed, w_gscale, H_bf16, M, N, K);
    if (rc != FQ_OK) return rc;
    if (N & 1) return FQ_ERR_SHAPE;
    if (M == 0) return FQ_OK;
    const int NH = N / 2;
    if ((NH % 8) != 0) return FQ_ERR_SHAPE;               // the quantiser works on whole 16-byte chunks of a row
    if (!H_fp8 || !h_scale) return FQ_ERR_NULL;
    if (!aligned16(H_fp8)) return FQ_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // zero-point terms for a GEMM that takes H_fp8 as its input: only where that GEMM has a workspace and the
    // quantiser can write them (rows of at most 16384 codes, whole groups)
    const bool next_large = next_workspace != nullptr && choose_kernel(M) == GemmKernel::Large &&
                            (NH % FQ_GROUP) == 0 && fq_quantize_can_write_zero_point(NH);
    if (next_workspace) {
        if (!next_large) return FQ_ERR_SHAPE;
        if (next_workspace_bytes < fq_gemm_large_workspace_bytes(M, NH)) return FQ_ERR_MEMORY;
        if (!aligned16(next_workspace)) return FQ_ERR_ALIGN;
    }
    const bool fused = choose_kernel(M) == GemmKernel::Large;
    const size_t need = fq_w4a8_gemm_workspace_bytes(M, N, K);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return FQ_ERR_MEMORY;
        if (!aligned16(workspace)) return FQ_ERR_ALIGN;
    }
    if (fused) {
        fq_launch_fill_zero(reinterpret_cast<unsigned*>(h_scale), M, s);   // the row maxima start at zero
        fq_launch_gemm_large(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, H_bf16, M, N, K, workspace,
                             workspace_prepared != 0, true, nullptr, s, false, reinterpret_cast<unsigned*>(h_scale));
        fq_launch_quantize_known(H_bf16, H_fp8, h_scale, M, NH, next_workspace, s);
        return after_launch();
    }
    // M <= 64 (or a kernel forced from outside): the fused gate/up GEMM, then the plain quantiser
    const int g = fq_w4a8_gemm_swiglu_ws(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, H_bf16, M, N, K, workspace,
                                         workspace_bytes, workspace_prepared, stream);
    if (g != FQ_OK) return g;
    fq_launch_quantize(H_bf16, H_fp8, h_scale, M, NH, s);
    return after_launch();
}

namespace {

inline size_t round16(size_t v) { return (v + 15u) & ~(size_t)15u; }

// one kernel for the whole layer: small M, short K, and no kernel forced from outside
bool linear_is_fused(int M, int K) {
    const GemmKernel k = forced_kernel();
    return (k == GemmKernel::Auto || k == GemmKernel::Small) && fq_linear_small_serves(M, K);
}

}  // namespace

size_t fq_w4a8_linear_workspace_bytes(int M, int N, int K) {
    if (M <= 0 || N <= 0 || K <= 0 || (K % FQ_GROUP) != 0) return 0;
    if (linear_is_fused(M, K)) return 0;
    return round16((size_t)M * (size_t)K) + round16((size_t)M * sizeof(float)) + fq_w4a8_gemm_workspace_bytes(M, N, K);
}

int fq_w4a8_linear_ws(const uint16_t* X_bf16, const uint8_t* Wq_packed, const uint8_t* w_gscale, float w_tscale,
                      uint16_t* Y_bf16, int M, int N, int K, void* workspace, size_t workspace_bytes, void* stream) {
    // the GEMM's checks, with X in the place of the codes (same alignment rule, twice the bytes)
    const int rc = check_gemm_args(X_bf16, X_bf16, Wq_packed, w_gscale, Y_bf16, M, N, K);
    if (rc != FQ_OK || M == 0) return rc;
    if ((unsigned long long)M * (unsigned long long)K * 2ull >= 0xFFFFFF00ull) return FQ_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (linear_is_fused(M, K)) {
        if (fq_launch_linear_small(X_bf16, nullptr, Wq_packed, w_gscale, w_tscale, Y_bf16, M, N, K, s)) return after_launch();
        return FQ_ERR_LAUNCH;                             // (the predicate and the launcher agree; not reached)
    }
    const size_t need = fq_w4a8_linear_workspace_bytes(M, N, K);
    if (!workspace || workspace_bytes < need) return FQ_ERR_MEMORY;
    if (!aligned16(workspace)) return FQ_ERR_ALIGN;
    uint8_t* A = static_cast<uint8_t*>(workspace);
    float* a_scale = reinterpret_cast<float*>(A + round16((size_t)M * (size_t)K));
    uint8_t* gemm_ws = reinterpret_cast<uint8_t*>(a_scale) + round16((size_t)M * sizeof(float));
    const size_t gemm_ws_bytes = fq_w4a8_gemm_workspace_bytes(M, N, K);
    int q;
    if (gemm_ws_bytes > 0) q = fq_quantize_act_ws(X_bf16, A, a_scale, M, K, gemm_ws, gemm_ws_bytes, stream);
    else                   q = fq_quantize_act(X_bf16, A, a_scale, M, K, stream);
    if (q != FQ_OK) return q;
    return fq_w4a8_gemm_ws(A, a_scale, Wq_packed, w_gscale, w_tscale, Y_bf16, M, N, K, gemm_ws, gemm_ws_bytes,
                           gemm_ws_bytes > 0 ? 1 : 0, stream);
}

int fq_w4a8_gemm_lut(const uint8_t* A_fp8, const float* a_scale, const uint8_t* Wq_packed,
                     const uint8_t* w_gscale, float w_tscale, uint16_t* Y_bf16,
                     int M, int N, int K, void* stream) {
    const int rc = check_gemm_args(A_fp8, a_scale, Wq_packed, w_gscale, Y_bf16, M, N, K);
    if (rc != FQ_OK || M == 0) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (forced_kernel() == GemmKernel::Simple)
        fq_launch_gemm_simple(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, Y_bf16, M, N, K, false, nullptr, s, true);
    else
        fq_launch_gemm_large(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, Y_bf16, M, N, K, nullptr, true, false, nullptr, s,
                             true);
    return after_launch();
}

size_t fq_kv4_packed_bytes(int H, int T, int values) {
    if (H <= 0 || T <= 0) return 0;
    return (size_t)H * (values ? fq_kv4_value_bytes(T) : fq_kv4_key_bytes(T));
}

int fq_kv4_pack(const int8_t* codes, uint8_t* packed, int H, int T, int values, void* stream) {
    if (H < 0 || T < 0) return FQ_ERR_SHAPE;
    if (H == 0 || T == 0) return FQ_OK;
    if (!codes || !packed) return FQ_ERR_NULL;
    if (!aligned16(packed)) return FQ_ERR_ALIGN;
    if (fq_kv4_packed_bytes(1, T, values) >= 0xFFFFFF00ull || H > 65535) return FQ_ERR_SHAPE;
    fq_launch_kv4_pack(codes, packed, H, T, values != 0, static_cast<hipStream_t>(stream));
    return after_launch();
}

int fq_kv4_unpack(const uint8_t* packed, int8_t* codes, int H, int T, int values, void* stream) {
    if (H < 0 || T < 0) return FQ_ERR_SHAPE;
    if (H == 0 || T == 0) return FQ_OK;
    if (!codes || !packed) return FQ_ERR_NULL;
    if (!aligned16(packed)) return FQ_ERR_ALIGN;
    if (fq_kv4_packed_bytes(1, T, values) >= 0xFFFFFF00ull || H > 65535) return FQ_ERR_SHAPE;
    fq_launch_kv4_unpack(packed, codes, H, T, values != 0, static_cast<hipStream_t>(stream));
    return after_launch();
}

int fq_kv4_scores(const uint8_t* Q_fp8, const float* q_scale, const uint8_t* K_packed, const uint8_t* k_scale,
                  float out_scale, uint16_t* S_bf16, int H, int R, int T, void* stream) {
    if (H < 0 || R < 0 || T < 0 || R > 64 || H > 65535) return FQ_ERR_SHAPE;
    if (H == 0 || R == 0 || T == 0) return FQ_OK;
    if (!Q_fp8 || !q_scale || !K_packed || !k_scale || !S_bf16) return FQ_ERR_NULL;
    if (!aligned16(Q_fp8) || !aligned16(K_packed)) return FQ_ERR_ALIGN;
    if (fq_kv4_key_bytes(T) >= 0xFFFFFF00ull) return FQ_ERR_SHAPE;
    fq_launch_kv4_scores(Q_fp8, q_scale, K_packed, k_scale, out_scale, S_bf16, H, R, T, static_cast<hipStream_t>(stream));
    return after_launch();
}

int fq_kv4_output(const uint8_t* P_fp8, const float* p_scale, const uint8_t* V_packed, const uint8_t* v_scale,
                  uint16_t* O_bf16, int H, int R, int T, int ldp, void* stream) {
    if (H < 0 || R < 0 || T < 0 || R > 32 || ldp < T) return FQ_ERR_SHAPE;
    if (H == 0 || R == 0) return FQ_OK;
    if (T == 0) return FQ_ERR_SHAPE;                      // an empty sum: nothing to attend to
    if (!P_fp8 || !p_scale || !V_packed || !v_scale || !O_bf16) return FQ_ERR_NULL;
    if (!aligned16(V_packed)) return FQ_ERR_ALIGN;
    if (fq_kv4_value_bytes(T) >= 0xFFFFFF00ull) return FQ_ERR_SHAPE;
    fq_launch_kv4_output(P_fp8, p_scale, V_packed, v_scale, O_bf16, H, R, T, ldp, static_cast<hipStream_t>(stream));
    return after_launch();
}

size_t fq_w4a8_gemm_static_max_workspace(void) { return FQ_STATIC_SCRATCH_BYTES; }

int fq_w4a8_gemm_static(const uint8_t* A_fp8, const float* a_scale, const uint8_t* Wq_packed,
                        const uint8_t* w_gscale, float w_tscale, uint16_t* Y_bf16,
                        int M, int N, int K, void* stream) {
    const int rc = check_gemm_args(A_fp8, a_scale, Wq_packed, w_gscale, Y_bf16, M, N, K);
    if (rc != FQ_OK || M == 0) return rc;
    const size_t need = fq_w4a8_gemm_workspace_bytes(M, N, K);
    if (need > FQ_STATIC_SCRATCH_BYTES) return FQ_ERR_MEMORY;
    // the device address of this GPU's copy of the array, looked up once per device
    static std::mutex m;
    static void* ptr[FQ_MAX_DEVICES];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= FQ_MAX_DEVICES) {
        (void)hipGetLastError();
        return FQ_ERR_LAUNCH;
    }
    void* ws;
    {
        std::lock_guard<std::mutex> lock(m);
        if (!ptr[dev]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
                (void)hipGetLastError();
                return FQ_ERR_MEMORY;
            }
            ptr[dev] = p;
        }
        ws = ptr[dev];
    }
    // every byte of the scratch this call reads is written by this call first (the zero-point pre-pass
    // fills all units of all M rows), so nothing needs clearing between calls
    return fq_w4a8_gemm_ws(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, Y_bf16, M, N, K, ws, FQ_STATIC_SCRATCH_BYTES, 0,
                           stream);
}

int fq_w4a8_gemm(const uint8_t* A_fp8, const float* a_scale, const uint8_t* Wq_packed,
                 const uint8_t* w_gscale, float w_tscale, uint16_t* Y_bf16,
                 int M, int N, int K, void* stream) {
    const int rc = check_gemm_args(A_fp8, a_scale, Wq_packed, w_gscale, Y_bf16, M, N, K);
    if (rc != FQ_OK || M == 0) return rc;
    // the library's own workspace: one grow-only device buffer, shared by every call of the process
    // (the mutex keeps the bookkeeping whole when several host threads call; the kernels of overlapping
    // calls still share the buffer, as the header says)
    static std::mutex ws_mutex;
    static void* ws = nullptr;
    static size_t ws_bytes = 0;
    const size_t need = fq_w4a8_gemm_workspace_bytes(M, N, K);
    std::lock_guard<std::mutex> lock(ws_mutex);
    if (need > ws_bytes) {
        if (ws) (void)hipFree(ws);
        ws = nullptr;
        ws_bytes = 0;
        if (hipMalloc(&ws, need) != hipSuccess) {
            (void)hipGetLastError();
            return FQ_ERR_MEMORY;
        }
        ws_bytes = need;
    }
    return fq_w4a8_gemm_ws(A_fp8, a_scale, Wq_packed, w_gscale, w_tscale, Y_bf16, M, N, K, ws, ws_bytes, 0, stream);
}

}  // extern "C"
