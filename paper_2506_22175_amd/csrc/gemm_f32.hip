// float32 grouped GEMM for the expert FFN (the two linear layers of an expert,
// Section II-B2, and their gradients).  Plain FMA arithmetic in float, LDS-tiled;
// this path exists for the float32 workload, whose tolerance rules out reduced
// precision inputs.  One workgroup computes a 64x64 tile of one expert.
#include "common.h"
#include "epilogue.h"

namespace moe {

constexpr int F_BM = 64, F_BN = 64, F_BK = 16, F_THREADS = 256;

// A(m,k) = A[m*a_rs + k*a_cs], B(k,n) = B[k*b_rs + n*b_cs]
template <int LAY, int EPI>
__global__ __launch_bounds__(F_THREADS) void gemm_f32_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    __shared__ float As[F_BK][F_BM + 4];
    __shared__ float Bs[F_BK][F_BN + 4];
    const int e = blockIdx.z;
    const int tm = blockIdx.y, tn = blockIdx.x;
    const int rows = g.counts[e];
    int Mdim, Kdim;
    long long a_rs, a_cs, b_rs, b_cs;
    if (LAY == GEMM_TN) { Mdim = g.Mo; Kdim = rows; a_rs = 1; a_cs = g.lda; b_rs = g.ldb; b_cs = 1; }
    else if (LAY == GEMM_NN) { Mdim = rows; Kdim = g.K; a_rs = g.lda; a_cs = 1; b_rs = g.ldb; b_cs = 1; }
    else { Mdim = rows; Kdim = g.K; a_rs = g.lda; a_cs = 1; b_rs = 1; b_cs = g.ldb; }
    const int m0 = tm * F_BM, n0 = tn * F_BN;
    if (m0 >= Mdim) return;
    const float* A = (const float*)g.A + (size_t)e * g.a_estride;
    const float* B = (const float*)g.B + (size_t)e * g.b_estride;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;

    for (int k0 = 0; k0 < Kdim; k0 += F_BK) {
        // 64x16 elements of A and of B: four each per thread
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int idx = tid + q * F_THREADS;
            int kk, mm;
            if (LAY == GEMM_TN) { mm = idx & 63; kk = idx >> 6; } else { kk = idx & 15; mm = idx >> 4; }
            float v = 0.0f;
            if (m0 + mm < Mdim && k0 + kk < Kdim) {
                if (LAY != GEMM_TN && g.a_rows)       // gathered rows: one matrix for all experts
                    v = ((const float*)g.A)[(size_t)g.a_rows[(size_t)e * g.Cp + m0 + mm] * a_rs + (size_t)(k0 + kk) * a_cs];
                else
                    v = A[(size_t)(m0 + mm) * a_rs + (size_t)(k0 + kk) * a_cs];
            }
            As[kk][mm] = v;
            int kb, nn;
            if (LAY == GEMM_NT) { kb = idx & 15; nn = idx >> 4; } else { nn = idx & 63; kb = idx >> 6; }
            float w = 0.0f;
            if (n0 + nn < g.N && k0 + kb < Kdim) w = B[(size_t)(k0 + kb) * b_rs + (size_t)(n0 + nn) * b_cs];
            Bs[kb][nn] = w;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < F_BK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty + 16 * i];
            float4 bv = *reinterpret_cast<const float4*>(&Bs[kk][tx * 4]);
            b[0] = bv.x; b[1] = bv.y; b[2] = bv.z; b[3] = bv.w;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    EpiCtx<float> c;
    c.ldc = g.ldc; c.ldz = g.ldz;
    c.C = EPI == EPI_SCATTER ? (float*)g.C : (float*)g.C + (size_t)e * g.c_estride;
    c.Cf = c.C;
    c.out_rows = g.c_rows ? g.c_rows + (size_t)e * g.Cp : nullptr;
    c.Z = g.Z ? (float*)g.Z + (size_t)e * g.Cp * g.ldz : nullptr;
    c.w = g.slot_w ? g.slot_w + (size_t)e * g.Cp : nullptr;
    const int n = n0 + tx * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = m0 + ty + 16 * i;
        float dot = 0.0f;
        if (r < Mdim && n < g.N) dot = epilogue4<float, EPI>(c, r, n, acc[i]);
        if (EPI == EPI_DGELU && g.dw_part) {
            // the 16 threads of a row are consecutive lanes
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, 64);
            if (tx == 0 && r < Mdim) g.dw_part[((size_t)e * g.Cp + r) * g.dw_parts + tn] = dot;
        }
    }
}

int gemm_f32_dw_parts(int H) { return (H + F_BN - 1) / F_BN; }

template <int LAY>
static moe_status launch_f32(GemmEpilogue epi, const GemmArgs& a, hipStream_t s) {
    const int Mmax = (LAY == GEMM_TN) ? a.Mo : a.Cp;
    const int tiles_m = (Mmax + F_BM - 1) / F_BM, tiles_n = (a.N + F_BN - 1) / F_BN;
    dim3 grid(tiles_n, tiles_m, a.E), block(F_THREADS);
    ProfScope ps(gemm_prof_kind(LAY, epi), s);
    switch (epi) {
        case EPI_STORE: hipLaunchKernelGGL((gemm_f32_kernel<LAY, EPI_STORE>), grid, block, 0, s, a, tiles_m, tiles_n); break;
        case EPI_GELU: hipLaunchKernelGGL((gemm_f32_kernel<LAY, EPI_GELU>), grid, block, 0, s, a, tiles_m, tiles_n); break;
        case EPI_DGELU: hipLaunchKernelGGL((gemm_f32_kernel<LAY, EPI_DGELU>), grid, block, 0, s, a, tiles_m, tiles_n); break;
        case EPI_ACCUM_F32: hipLaunchKernelGGL((gemm_f32_kernel<LAY, EPI_ACCUM_F32>), grid, block, 0, s, a, tiles_m, tiles_n); break;
        case EPI_STORE_F32: hipLaunchKernelGGL((gemm_f32_kernel<LAY, EPI_STORE_F32>), grid, block, 0, s, a, tiles_m, tiles_n); break;
        case EPI_SCATTER: hipLaunchKernelGGL((gemm_f32_kernel<LAY, EPI_SCATTER>), grid, block, 0, s, a, tiles_m, tiles_n); break;
    }
    count_launch(LC_GEMM);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

moe_status gemm_f32(GemmLayout lay, GemmEpilogue epi, const GemmArgs& a, hipStream_t s) {
    if (a.dw_part && a.dw_parts != gemm_f32_dw_parts(a.N)) return MOE_ERR_SHAPE;
    if (a.a_rows && (lay == GEMM_TN || a.a_row_limit <= 0)) return MOE_ERR_UNSUPPORTED;
    if (epi == EPI_SCATTER && (lay == GEMM_TN || !a.c_rows || !a.slot_w || a.c_row_limit <= 0)) return MOE_ERR_UNSUPPORTED;
    if (lay == GEMM_NN) return launch_f32<GEMM_NN>(epi, a, s);
    if (lay == GEMM_NT) return launch_f32<GEMM_NT>(epi, a, s);
    return launch_f32<GEMM_TN>(epi, a, s);
}

}  // namespace moe
