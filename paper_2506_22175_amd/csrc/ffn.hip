// Expert FFN of one partition, forward and backward, as grouped GEMMs over the
// local experts (Section II-B2: T_DI -> T_M -> T_DO through two linear layers
// and one activation; Section III-B: backward is symmetric; Table II: 2 GEMM
// units forward, 4 backward, 5 with recomputation of T_M).
#include "common.h"

namespace moe {

static moe_status run_gemm(const Dims& d, GemmLayout lay, GemmEpilogue epi, const GemmArgs& a, hipStream_t s) {
    return d.dtype == MOE_F32 ? gemm_f32(lay, epi, a, s) : gemm_bf16(lay, epi, a, s);
}

static GemmArgs base_args(const Dims& d, const int* counts_p) {
    GemmArgs a = {};
    a.counts = counts_p;
    a.E = d.E;
    a.Cp = d.Cp;
    a.free_cus = d.free_cus;
    return a;
}

moe_status ffn_fwd(const Dims& d, int part, const void* DI, const int* rows, const int* counts,
                   const void* W1, const void* W2, void* Z, void* A, void* DO, hipStream_t s,
                   const int* y_rows, const float* slot_w, void* y) {
    const int* cp = counts + (size_t)part * d.E;
    // T_M = T_DI W1 ; A = gelu(T_M)
    GemmArgs a = base_args(d, cp);
    a.A = DI; a.lda = d.M; a.a_estride = (long long)d.Cp * d.M;
    if (rows) { a.a_rows = rows + (size_t)part * d.Rp; a.a_row_limit = d.T; a.a_estride = 0; }
    a.B = W1; a.ldb = d.H; a.b_estride = (long long)d.M * d.H;
    a.C = A; a.ldc = d.H; a.c_estride = (long long)d.Cp * d.H;
    a.N = d.H; a.K = d.M;
    a.Z = Z; a.ldz = d.H;
    MOE_TRY(run_gemm(d, GEMM_NN, EPI_GELU, a, s));
    // T_DO = A W2
    GemmArgs b = base_args(d, cp);
    b.A = A; b.lda = d.H; b.a_estride = (long long)d.Cp * d.H;
    b.B = W2; b.ldb = d.M; b.b_estride = (long long)d.H * d.M;
    b.C = DO; b.ldc = d.M; b.c_estride = (long long)d.Cp * d.M;
    b.N = d.M; b.K = d.H;
    if (y_rows) {
        // one choice per token: a kept row is its token's whole output, weighted (Fig. 1: T_DO -> T_O with
        // no T_DO in between)
        b.C = y; b.c_estride = 0;
        b.c_rows = y_rows + (size_t)part * d.Rp; b.c_row_limit = d.T;
        b.slot_w = slot_w + (size_t)part * d.Rp;
        return run_gemm(d, GEMM_NN, EPI_SCATTER, b, s);
    }
    return run_gemm(d, GEMM_NN, EPI_STORE, b, s);
}

moe_status ffn_bwd_main(const Dims& d, int part, int recompute, const void* DI, void* Z, const void* dDO,
                        const int* counts, const float* slot_w, const void* W1, const void* W2,
                        void* dZ, void* dDI, float* dw_part, hipStream_t s) {
    const int* cp = counts + (size_t)part * d.E;
    const long long eM = (long long)d.Cp * d.M, eH = (long long)d.Cp * d.H, wMH = (long long)d.M * d.H;
    if (recompute) {
        // T_M again from T_DI (Section III-D: the overwritten T_M is restored by recomputation)
        GemmArgs a = base_args(d, cp);
        a.A = DI; a.lda = d.M; a.a_estride = eM;
        a.B = W1; a.ldb = d.H; a.b_estride = wMH;
        a.C = Z; a.ldc = d.H; a.c_estride = eH;
        a.N = d.H; a.K = d.M;
        MOE_TRY(run_gemm(d, GEMM_NN, EPI_STORE, a, s));
    }
    {   // G = dDO W2^T ; dZ = w G gelu'(Z) ; Z <- w gelu(Z) ; dw_part = <gelu(Z), G>
        GemmArgs a = base_args(d, cp);
        a.A = dDO; a.lda = d.M; a.a_estride = eM;
        a.B = W2; a.ldb = d.M; a.b_estride = wMH;
        a.C = dZ; a.ldc = d.H; a.c_estride = eH;
        a.N = d.H; a.K = d.M;
        a.Z = Z; a.ldz = d.H;
        a.slot_w = slot_w + (size_t)part * d.Rp;
        a.dw_part = dw_part;
        a.dw_parts = d.dtype == MOE_F32 ? gemm_f32_dw_parts(d.H) : gemm_bf16_dw_parts(d.H);
        MOE_TRY(run_gemm(d, GEMM_NT, EPI_DGELU, a, s));
    }
    {   // dDI = dZ W1^T
        GemmArgs a = base_args(d, cp);
        a.A = dZ; a.lda = d.H; a.a_estride = eH;
        a.B = W1; a.ldb = d.H; a.b_estride = wMH;
        a.C = dDI; a.ldc = d.M; a.c_estride = eM;
        a.N = d.M; a.K = d.H;
        MOE_TRY(run_gemm(d, GEMM_NT, EPI_STORE, a, s));
    }
    return MOE_OK;
}

// Both weight gradients over the rows of `nparts` consecutive partitions starting at `part`, whose
// buffers lie strideM (T_DI, dT_DO) and strideH (weighted activations, dT_M) elements apart.  The
// reduction over a partition's rows and the sum over partitions are one GEMM, so the float gradients
// are read and written once per group instead of once per partition.
moe_status ffn_wgrad(const Dims& d, int part, int nparts, int store, const void* DI, const void* A, const void* dDO,
                     const void* dZ, long long strideM, long long strideH, const int* counts,
                     float* dW1, float* dW2, hipStream_t s) {
    const long long eM = (long long)d.Cp * d.M, eH = (long long)d.Cp * d.H, wMH = (long long)d.M * d.H;
    // the float GEMM reduces one partition per launch
    const int per_launch = d.dtype == MOE_F32 ? 1 : nparts;
    for (int q = 0; q < nparts; q += per_launch) {
        const int* cp = counts + (size_t)(part + q) * d.E;
        const GemmEpilogue epi = (store && q == 0) ? EPI_STORE_F32 : EPI_ACCUM_F32;
        const size_t oM = (size_t)q * strideM * d.es, oH = (size_t)q * strideH * d.es;
        {   // dW2[e] += (w gelu(Z))^T dDO
            GemmArgs a = base_args(d, cp);
            a.A = (const char*)A + oH; a.lda = d.H; a.a_estride = eH; a.Mo = d.H;
            a.B = (const char*)dDO + oM; a.ldb = d.M; a.b_estride = eM;
            a.C = dW2; a.ldc = d.M; a.c_estride = wMH;
            a.N = d.M;
            a.k_segs = per_launch; a.a_sstride = strideH; a.b_sstride = strideM;
            MOE_TRY(run_gemm(d, GEMM_TN, epi, a, s));
        }
        {   // dW1[e] += DI^T dZ
            GemmArgs a = base_args(d, cp);
            a.A = (const char*)DI + oM; a.lda = d.M; a.a_estride = eM; a.Mo = d.M;
            a.B = (const char*)dZ + oH; a.ldb = d.H; a.b_estride = eH;
            a.C = dW1; a.ldc = d.H; a.c_estride = wMH;
            a.N = d.H;
            a.k_segs = per_launch; a.a_sstride = strideM; a.b_sstride = strideH;
            MOE_TRY(run_gemm(d, GEMM_TN, epi, a, s));
        }
    }
    return MOE_OK;
}

moe_status ffn_bwd(const Dims& d, int part, int recompute, const void* DI, void* Z, const void* dDO,
                   const int* counts, const float* slot_w, const void* W1, const void* W2,
                   void* dZ, void* dDI, float* dW1, float* dW2, float* dw_part, hipStream_t s) {
    MOE_TRY(ffn_bwd_main(d, part, recompute, DI, Z, dDO, counts, slot_w, W1, W2, dZ, dDI, dw_part, s));
    return ffn_wgrad(d, part, 1, d.overwrite && part == 0, DI, Z, dDO, dZ, 0, 0, counts, dW1, dW2, s);
}

}  // namespace moe

using namespace moe;

extern "C" moe_status moe_dw_parts(const moe_config* cfg, int32_t* parts) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    if (!parts) return MOE_ERR_NULL;
    *parts = d.dtype == MOE_F32 ? gemm_f32_dw_parts(d.H) : gemm_bf16_dw_parts(d.H);
    return MOE_OK;
}

extern "C" moe_status moe_expert_ffn_fwd(const moe_config* cfg, int32_t part, const void* DI, const int32_t* counts,
                                         const void* W1, const void* W2, void* Z, void* A, void* DO, void* stream) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    MOE_TRY(check_part(d, part));
    if (!DI || !counts || !W1 || !W2 || !A || !DO) return MOE_ERR_NULL;
    return ffn_fwd(d, part, DI, nullptr, counts, W1, W2, Z, A, DO, (hipStream_t)stream);
}

extern "C" moe_status moe_expert_ffn_fwd_gather(const moe_config* cfg, int32_t part, const void* x, const int32_t* rows,
                                                const int32_t* counts, const void* W1, const void* W2,
                                                void* Z, void* A, void* DO, void* stream) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    MOE_TRY(check_part(d, part));
    if (!x || !rows || !counts || !W1 || !W2 || !A || !DO) return MOE_ERR_NULL;
    return ffn_fwd(d, part, x, rows, counts, W1, W2, Z, A, DO, (hipStream_t)stream);
}

extern "C" moe_status moe_expert_ffn_bwd(const moe_config* cfg, int32_t part, int32_t recompute,
                                         const void* DI, void* Z, const void* dDO, const int32_t* counts,
                                         const float* slot_w, const void* W1, const void* W2,
                                         void* dZ, void* dDI, float* dW1, float* dW2, float* dw_part, void* stream) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    MOE_TRY(check_part(d, part));
    if (!DI || !Z || !dDO || !counts || !slot_w || !W1 || !W2 || !dZ || !dDI || !dW1 || !dW2) return MOE_ERR_NULL;
    return ffn_bwd(d, part, recompute, DI, Z, dDO, counts, slot_w, W1, W2, dZ, dDI, dW1, dW2, dw_part,
                   (hipStream_t)stream);
}
