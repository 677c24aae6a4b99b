// Shared declarations of the gfx950 MoE-layer library (internal; the public
// interface is include/moe.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "moe.h"

namespace moe {

typedef unsigned short bf16_t;   // bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
    return __uint_as_float(((unsigned)v) << 16);
}
// round to nearest, ties to even (v_cvt_pk_bf16_f32 on gfx950)
typedef __bf16 hw_bf16x2 __attribute__((ext_vector_type(2)));
typedef float hw_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    return __builtin_bit_cast(bf16_t, (__bf16)f);
}
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    hw_f32x2 v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, hw_bf16x2));
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float ld(const float* p) { return *p; }
    static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// eight consecutive elements <-> eight floats (16 bytes of bf16, 32 bytes of float)
template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* o) {
        uint4 u = *reinterpret_cast<const uint4*>(p);
        unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = __uint_as_float(w[i] << 16);
            o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float* v) {
        uint4 u;
        u.x = pack_bf16x2(v[0], v[1]); u.y = pack_bf16x2(v[2], v[3]);
        u.z = pack_bf16x2(v[4], v[5]); u.w = pack_bf16x2(v[6], v[7]);
        *reinterpret_cast<uint4*>(p) = u;
    }
};
template <> struct Vec8<float> {
    static __device__ __forceinline__ void load(const float* p, float* o) {
        float4 a = *reinterpret_cast<const float4*>(p);
        float4 b = *reinterpret_cast<const float4*>(p + 4);
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
        o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
    static __device__ __forceinline__ void store(float* p, const float* v) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
};

// Eight consecutive elements as they come from memory; converted when used, so that a
// loop can request the next ones before it works on the current ones.
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> {
    uint4 u;
    __device__ __forceinline__ void load(const bf16_t* p) { u = *reinterpret_cast<const uint4*>(p); }
    __device__ __forceinline__ void zero() { u = make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ void to_float(float* o) const {
        const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = __uint_as_float(w[i] << 16);
            o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};
template <> struct Raw8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float* p) {
        a = *reinterpret_cast<const float4*>(p);
        b = *reinterpret_cast<const float4*>(p + 4);
    }
    __device__ __forceinline__ void zero() { a = make_float4(0, 0, 0, 0); b = a; }
    __device__ __forceinline__ void to_float(float* o) const {
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
        o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
};

// GeLU in its erf form, z * Phi(z), and its derivative Phi(z) + z * phi(z).
// erf is evaluated with the five-term rational approximation of Abramowitz &
// Stegun 7.1.26 (absolute error below 1.5e-7, far inside the float32 tolerance),
// which shares its exp(-x^2) with the normal density phi: about twenty
// instructions for value and derivative together.
__device__ __forceinline__ void gelu_both_f(float z, float* g, float* dg) {
    const float x = fabsf(z) * 0.70710678118654752440f;
    const float t = __frcp_rn(fmaf(0.3275911f, x, 1.0f));
    const float ex = __expf(-x * x);                       // = exp(-z^2 / 2)
    float p = fmaf(t, 1.061405429f, -1.453152027f);
    p = fmaf(t, p, 1.421413741f);
    p = fmaf(t, p, -0.284496736f);
    p = fmaf(t, p, 0.254829592f);
    const float erf_abs = fmaf(-p * t, ex, 1.0f);
    const float cdf = fmaf(copysignf(0.5f, z), erf_abs, 0.5f);
    *g = z * cdf;
    *dg = fmaf(z * 0.39894228040143267794f, ex, cdf);
}
__device__ __forceinline__ float gelu_f(float z) {
    float g, dg;
    gelu_both_f(z, &g, &dg);
    return g;
}

// The same two functions for bfloat16 storage, where every result is rounded to 8 bits of
// mantissa anyway: Phi(z) ~ 1 / (1 + exp(-z (a + b z^2))), the logistic form of the usual tanh
// approximation with a, b refitted to the erf form (absolute error of z*Phi below 2.8e-4, of
// the derivative below 8.8e-4, against half a bfloat16 unit of 2e-3 at magnitude one).  Two
// transcendental instructions (v_exp_f32, and v_rcp_f32 as it is: a correctly rounded
// reciprocal costs ten more) and a handful of multiply-adds instead of the rational erf.
__device__ __forceinline__ void gelu_both_fast_f(float z, float* g, float* dg) {
    constexpr float A = 1.60031416f, B = 0.06940179f, LOG2E = 1.44269504088896340736f;
    const float z2 = z * z;
    const float arg = z * fmaf(z2, -B * LOG2E, -A * LOG2E);        // -z (a + b z^2) log2(e)
    const float s = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(arg));   // exp2(+inf) = inf gives s = 0
    const float gz = z * s;
    *g = gz;
    // d/dz [z s(u)] = s + z s (1 - s) u',  u = z (a + b z^2),  u' = a + 3 b z^2
    *dg = fmaf(gz * (1.0f - s), fmaf(z2, 3.0f * B, A), s);
}
__device__ __forceinline__ float gelu_fast_f(float z) {
    constexpr float A = 1.60031416f, B = 0.06940179f, LOG2E = 1.44269504088896340736f;
    const float arg = z * fmaf(z * z, -B * LOG2E, -A * LOG2E);
    return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(arg));
}

struct Dims {
    int T, M, H, E, k, n, Tp, Cp, Rp;
    int dtype, reuse;
    int overwrite;   // weight gradients are overwritten (first partition stores) instead of accumulated
    int renorm;      // combine weights are renormalised over the token's k choices
    int fuse;        // forward's first GEMM gathers its rows from the token-major input
    int G;           // partitions per weight-gradient GEMM in backward (>= 1)
    int free_cus;    // compute units the persistent GEMM grids leave to other streams
    int fcomb;       // k = 1: the second expert GEMM writes its weighted rows straight into y
    size_t es;   // element size in bytes
};

// Validates cfg and fills Dims.  Host.
moe_status make_dims(const moe_config* cfg, Dims* d);
moe_status check_part(const Dims& d, int part);

// Remembers where a HIP call failed; moe_last_error() returns the text.
void note_hip_error(hipError_t e, const char* file, int line);
#define MOE_CHECK_LAUNCH() do { hipError_t _e = hipGetLastError(); \
    if (_e != hipSuccess) { ::moe::note_hip_error(_e, __FILE__, __LINE__); return MOE_ERR_HIP; } } while (0)
#define HIP_TRY(expr) do { hipError_t _e = (expr); \
    if (_e != hipSuccess) { ::moe::note_hip_error(_e, __FILE__, __LINE__); return MOE_ERR_HIP; } } while (0)
#define MOE_TRY(expr) do { moe_status _s = (expr); if (_s != MOE_OK) return _s; } while (0)

enum LaunchClass { LC_GEMM = 0, LC_PERMUTE = 1, LC_OTHER = 2 };
void count_launch(LaunchClass c, int n = 1);

// Optional per-kernel timing with HIP events on the launching stream (off by
// default; moe_profile_enable).  Kinds index the table in moe_profile_read.
enum ProfKind {
    PK_GEMM_FWD1 = 0,    // T_DI W1 -> gelu            (NN, GeLU epilogue)
    PK_GEMM_NN = 1,      // A W2 -> T_DO, and the recomputation of T_M (NN, plain store)
    PK_GEMM_DGELU = 2,   // dDO W2^T with the GeLU-backward epilogue (NT)
    PK_GEMM_DGRAD = 3,   // dZ W1^T -> dDI                (NT, plain store)
    PK_GEMM_WGRAD = 4,   // both weight gradients         (TN, float accumulate)
    PK_DISPATCH = 5, PK_COMBINE = 6, PK_DISPATCH_BWD = 7, PK_ROUTE = 8, PK_SLOTS = 9, PK_GATE_BWD = 10,
    PK_COUNT = 11
};
struct ProfScope {
    int idx; hipStream_t s;
    ProfScope(int kind, hipStream_t stream);
    ~ProfScope();
};

// ---- grouped GEMM interface (gemm_bf16.hip / gemm_f32.hip) -------------------
// Three operand layouts, all per expert e with r = counts[e] valid rows:
//   NN: C[r,N] = A[r,K] * B[K,N]         A rows K-contiguous, B rows N-contiguous
//   NT: C[r,N] = A[r,K] * B[N,K]^T       both K-contiguous
//   TN: C[Mo,N] (+)= A[r,Mo]^T * B[r,N]  reduction over the r valid rows
enum GemmLayout { GEMM_NN = 0, GEMM_NT = 1, GEMM_TN = 2 };
enum GemmEpilogue {
    EPI_STORE = 0,      // C = acc                       (element type)
    EPI_GELU = 1,       // Z = acc (optional), A = gelu(Z)
    EPI_DGELU = 2,      // dZ = w*acc*gelu'(Z), Z <- w*gelu(Z), dw_part = <gelu(Z), acc>
    EPI_ACCUM_F32 = 3,  // C(float) += acc
    EPI_STORE_F32 = 4,  // C(float) = acc (also where the reduction is empty)
    EPI_SCATTER = 5     // C[c_rows[row]] = slot_w[row] * acc: rows leave for one matrix of c_row_limit rows
};

struct GemmArgs {
    const void* A; const void* B; void* C;
    long long a_estride, b_estride, c_estride;   // elements between experts
    int lda, ldb, ldc;
    const int* a_rows;    // NN / NT only, may be NULL: row r of expert e is row a_rows[e*Cp + r] of A
                          // (A is then one matrix of a_row_limit rows for all experts; a_estride unused)
    int a_row_limit;
    const int* counts;    // [E] valid rows of this partition
    int E, Cp;            // experts, max rows per expert
    int Mo;               // TN only: output rows
    int N, K;             // K unused for TN (K = counts[e])
    // TN only: reduce over the rows of k_segs partitions in one launch (0 or 1: one).  Partition sg of
    // the group has its counts at counts[sg*E + e] and its operands a_sstride / b_sstride elements
    // after those of the partition before.  bf16 GEMM, at most 8.
    int k_segs;
    long long a_sstride, b_sstride;
    int free_cus;         // bf16: compute units the persistent grid leaves free
    const int* c_rows;    // EPI_SCATTER: [E*Cp] output row of each expert row (C is then one matrix for all
    int c_row_limit;      //   experts, of c_row_limit rows; c_estride unused); slot_w gives the row weights
    // epilogue operands
    void* Z;              // EPI_GELU: optional pre-activation out; EPI_DGELU: in/out
    int ldz;              // row stride of Z (elements); expert stride is Cp*ldz
    const float* slot_w;  // EPI_DGELU: [E*Cp] row weights
    float* dw_part;       // EPI_DGELU: [E*Cp, dw_parts] or NULL
    int dw_parts;
};

inline int gemm_prof_kind(int lay, int epi) {
    if (epi == EPI_GELU) return PK_GEMM_FWD1;
    if (epi == EPI_DGELU) return PK_GEMM_DGELU;
    if (epi == EPI_ACCUM_F32 || epi == EPI_STORE_F32) return PK_GEMM_WGRAD;
    if (epi == EPI_SCATTER) return PK_GEMM_NN;
    return lay == GEMM_NN ? PK_GEMM_NN : PK_GEMM_DGRAD;
}

moe_status gemm_bf16(GemmLayout lay, GemmEpilogue epi, const GemmArgs& a, hipStream_t s);
moe_status gemm_f32(GemmLayout lay, GemmEpilogue epi, const GemmArgs& a, hipStream_t s);
int gemm_bf16_dw_parts(int H);   // column blocks the DGELU epilogue reports per row
int gemm_f32_dw_parts(int H);


// ---- one partition's expert FFN (ffn.hip) ---------------------------------------
// rows != NULL: DI is the token-major input [T, M] and rows[part] maps expert rows to its rows
// y_rows != NULL (k = 1): the second GEMM writes slot_w * row into y[y_rows[...]] instead of DO
moe_status ffn_fwd(const Dims& d, int part, const void* DI, const int* rows, const int* counts,
                   const void* W1, const void* W2, void* Z, void* A, void* DO, hipStream_t s,
                   const int* y_rows = nullptr, const float* slot_w = nullptr, void* y = nullptr);
moe_status ffn_bwd(const Dims& d, int part, int recompute, const void* DI, void* Z, const void* dDO,
                   const int* counts, const float* slot_w, const void* W1, const void* W2,
                   void* dZ, void* dDI, float* dW1, float* dW2, float* dw_part, hipStream_t s);
// its two halves: everything but the weight gradients of one partition, and the weight gradients of
// nparts consecutive partitions at once
moe_status ffn_bwd_main(const Dims& d, int part, int recompute, const void* DI, void* Z, const void* dDO,
                        const int* counts, const float* slot_w, const void* W1, const void* W2,
                        void* dZ, void* dDI, float* dw_part, hipStream_t s);
moe_status ffn_wgrad(const Dims& d, int part, int nparts, int store, const void* DI, const void* A, const void* dDO,
                     const void* dZ, long long strideM, long long strideH, const int* counts,
                     float* dW1, float* dW2, hipStream_t s);

// k = 1 with the fused combine: rows of y of dropped tokens <- 0 (permute.hip)
moe_status zero_dropped(const Dims& d, const int* slot, void* y, hipStream_t s);

}  // namespace moe
