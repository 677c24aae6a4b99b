// Dispatch (S), combine (R) and their backward counterparts for one partition.
// In the paper S and R are the two All-to-All exchanges of expert parallelism
// (Fig. 1, Section II-A); on one GPU they are local row permutations between the
// token-ordered tensors T_I / T_O and the expert-contiguous T_DI / T_DO.  They
// are bound by HBM: every kernel moves whole rows with 16-byte accesses, one
// wavefront per token, and reads each token row once however many experts it
// goes to.
#include "common.h"

namespace moe {

constexpr int PERM_THREADS = 256;
constexpr int PERM_WAVES = PERM_THREADS / 64;

// 16-byte row accesses; NT = non-temporal (the row is read or written once per kernel)
typedef unsigned u32x4_hw __attribute__((ext_vector_type(4)));
template <bool NT> __device__ __forceinline__ uint4 ld_row(const uint4* p) {
    if (NT) {
        u32x4_hw v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_hw*>(p));
        return make_uint4(v[0], v[1], v[2], v[3]);
    }
    return *p;
}
template <bool NT> __device__ __forceinline__ void st_row(uint4* p, const uint4& u) {
    if (NT) {
        u32x4_hw v = {u.x, u.y, u.z, u.w};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4_hw*>(p));
    } else {
        *p = u;
    }
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// DI[slot[t,j]] = src[t]; optionally dw[t,j] = <src[t], saved[slot[t,j]]>.
// U = 16-byte units per row.
template <typename T, bool WITH_DW>
__global__ __launch_bounds__(PERM_THREADS) void dispatch_kernel(
    const T* __restrict__ src, const int* __restrict__ slot, T* __restrict__ dst,
    const T* __restrict__ saved, float* __restrict__ dw, int t_begin, int t_count, int M, int k) {
    const int lane = threadIdx.x & 63;
    const int tl = blockIdx.x * PERM_WAVES + (threadIdx.x >> 6);
    if (tl >= t_count) return;
    const int t = t_begin + tl;
    constexpr int EPU = 16 / sizeof(T);            // elements per 16-byte unit
    const int U = M / EPU;
    int s[8];
    for (int j = 0; j < k; ++j) s[j] = slot[(size_t)t * k + j];
    const uint4* in = reinterpret_cast<const uint4*>(src + (size_t)t * M);
    float dot[8];
    if (WITH_DW) for (int j = 0; j < k; ++j) dot[j] = 0.0f;
    for (int c0 = 0; c0 < U; c0 += 256) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int c = c0 + u * 64 + lane;
            if (c < U) v[u] = ld_row<true>(in + c);
        }
        for (int j = 0; j < k; ++j) {
            if (s[j] < 0) continue;
            uint4* out = reinterpret_cast<uint4*>(dst + (size_t)s[j] * M);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                int c = c0 + u * 64 + lane;
                if (c < U) {
                    st_row<false>(out + c, v[u]);
                    if (WITH_DW) {
                        uint4 o = reinterpret_cast<const uint4*>(saved + (size_t)s[j] * M)[c];
                        const T* a = reinterpret_cast<const T*>(&v[u]);
                        const T* b = reinterpret_cast<const T*>(&o);
#pragma unroll
                        for (int i = 0; i < EPU; ++i) dot[j] = fmaf(Elem<T>::ld(a + i), Elem<T>::ld(b + i), dot[j]);
                    }
                }
            }
        }
    }
    if (WITH_DW) {
        for (int j = 0; j < k; ++j) {
            float d = wave_sum(dot[j]);
            if (lane == 0) dw[(size_t)t * k + j] = s[j] >= 0 ? d : 0.0f;
        }
    }
}

// 16 bytes <-> floats (8 bf16 or 4 float)
template <typename T> struct Unit;
template <> struct Unit<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void to_float(const uint4& u, float* o) {
        const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = __uint_as_float(w[i] << 16);
            o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ uint4 from_float(const float* v) {
        return make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
    }
};
template <> struct Unit<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void to_float(const uint4& u, float* o) {
        o[0] = __uint_as_float(u.x); o[1] = __uint_as_float(u.y); o[2] = __uint_as_float(u.z); o[3] = __uint_as_float(u.w);
    }
    static __device__ __forceinline__ uint4 from_float(const float* v) {
        return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
    }
};

// y[t] = sum_j w[t,j] * DO[slot[t,j]]  (float accumulation, ascending j).  One wavefront per
// token; four 16-byte units per lane are in flight per source row.
template <typename T>
__global__ __launch_bounds__(PERM_THREADS) void combine_kernel(
    const T* __restrict__ DO, const int* __restrict__ slot, const float* __restrict__ w,
    T* __restrict__ y, int t_begin, int t_count, int M, int k) {
    const int lane = threadIdx.x & 63;
    const int tl = blockIdx.x * PERM_WAVES + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (tl >= t_count) return;
    const int t = t_begin + tl;
    constexpr int N = Unit<T>::N;
    const int U = M / N;
    int s[8];
    float ws[8];
    for (int j = 0; j < k; ++j) { s[j] = slot[(size_t)t * k + j]; ws[j] = w[(size_t)t * k + j]; }
    uint4* out = reinterpret_cast<uint4*>(y + (size_t)t * M);
    for (int c0 = 0; c0 < U; c0 += 256) {
        float acc[4][N];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < N; ++i) acc[u][i] = 0.0f;
        for (int j = 0; j < k; ++j) {
            if (s[j] < 0) continue;
            const uint4* in = reinterpret_cast<const uint4*>(DO + (size_t)s[j] * M);
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * 64 + lane;
                v[u] = c < U ? ld_row<true>(in + c) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float r[N];
                Unit<T>::to_float(v[u], r);
#pragma unroll
                for (int i = 0; i < N; ++i) acc[u][i] = fmaf(ws[j], r[i], acc[u][i]);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * 64 + lane;
            if (c < U) st_row<false>(out + c, Unit<T>::from_float(acc[u]));
        }
    }
}

// One choice per token and the combine fused into the second expert GEMM: a dropped token has no row
// that would write its output, so its row of y is zeroed here.  One wavefront per token.
template <typename T>
__global__ __launch_bounds__(PERM_THREADS) void zero_dropped_kernel(const int* __restrict__ slot, T* __restrict__ y,
                                                                    int Ttot, int M) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * PERM_WAVES + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (t >= Ttot || slot[t] >= 0) return;
    const int U = M / Unit<T>::N;
    uint4* out = reinterpret_cast<uint4*>(y + (size_t)t * M);
    for (int c = lane; c < U; c += 64) out[c] = make_uint4(0, 0, 0, 0);
}

// dx[t] = sum_j dDI[slot[t,j]] + dL[t,:] Wg^T with the gate matrix transposed into LDS as
// float (no conversion per token); a wavefront takes two tokens at a time, so each LDS read
// feeds two tokens, and workgroups walk over the tokens.  Row e of W_g^T is stored so that the
// 16 bytes a lane reads are contiguous across lanes: element d = unit*N + 4*h + r sits at
// e*M + h*(M/N)*4 + unit*4 + r (N = elements of the storage type per 16-byte unit).
constexpr int DXF_THREADS = 1024;
constexpr int DXF_WAVES = DXF_THREADS / 64;
template <typename T>
__global__ __launch_bounds__(DXF_THREADS) void dispatch_bwd_f32lds_kernel(
    const T* __restrict__ dDI, const int* __restrict__ slot, const float* __restrict__ dL,
    const T* __restrict__ Wg, T* __restrict__ dx, int t_begin, int t_count, int M, int E, int k) {
    extern __shared__ __attribute__((aligned(16))) char dxb_smem[];
    float* wgt = reinterpret_cast<float*>(dxb_smem);
    constexpr int N = Unit<T>::N;
    constexpr int NH = N / 4;
    const int U = M / N;
#pragma unroll 8
    for (int q = threadIdx.x; q < M * E; q += DXF_THREADS) {
        const int e = q / M, d = q - e * M;
        const int unit = d / N, h = (d % N) >> 2, r = d & 3;
        wgt[e * M + h * U * 4 + unit * 4 + r] = Elem<T>::ld(Wg + (size_t)d * E + e);
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    for (int tl = 2 * (blockIdx.x * DXF_WAVES + wid); tl < t_count; tl += 2 * gridDim.x * DXF_WAVES) {
        const int ntok = min(2, t_count - tl);
        for (int c0 = 0; c0 < U; c0 += 256) {
            float acc[2][4][N];
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int i = 0; i < N; ++i) acc[a][u][i] = 0.0f;
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                if (a >= ntok) continue;
                const int t = t_begin + tl + a;
                for (int j = 0; j < k; ++j) {
                    const int sj = slot[(size_t)t * k + j];
                    if (sj < 0) continue;
                    const uint4* in = reinterpret_cast<const uint4*>(dDI + (size_t)sj * M);
                    uint4 v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int c = c0 + u * 64 + lane;
                        v[u] = c < U ? in[c] : make_uint4(0, 0, 0, 0);
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        float r[N];
                        Unit<T>::to_float(v[u], r);
#pragma unroll
                        for (int i = 0; i < N; ++i) acc[a][u][i] += r[i];
                    }
                }
            }
            const float* g0 = dL + (size_t)(t_begin + tl) * E;
            const float* g1 = dL + (size_t)(t_begin + tl + ntok - 1) * E;     // the same token again when only one is left
            for (int e = 0; e < E; ++e) {
                const float ge0 = g0[e], ge1 = g1[e];
                const float* wrow = wgt + (size_t)e * M;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = c0 + u * 64 + lane;
                    if (c < U) {
#pragma unroll
                        for (int h = 0; h < NH; ++h) {
                            const float4 w4 = *reinterpret_cast<const float4*>(wrow + h * U * 4 + c * 4);
                            const float w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                acc[0][u][4 * h + r] = fmaf(ge0, w[r], acc[0][u][4 * h + r]);
                                acc[1][u][4 * h + r] = fmaf(ge1, w[r], acc[1][u][4 * h + r]);
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                if (a >= ntok) continue;
                uint4* out = reinterpret_cast<uint4*>(dx + (size_t)(t_begin + tl + a) * M);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = c0 + u * 64 + lane;
                    if (c < U) out[c] = Unit<T>::from_float(acc[a][u]);
                }
            }
        }
    }
}

// dx[t] = sum_j dDI[slot[t,j]] + dL[t,:] Wg^T for bfloat16 storage, with the gate term on the
// matrix cores.  A lane owns eight consecutive columns (a wavefront 512, so every row access is
// a coalesced 1 KB), and its gate weights are the second operand of
// v_mfma_f32_4x4x4_16B_bf16: that instruction multiplies sixteen independent 4x4 blocks, block
// b = lane/4, D_b[i][j] += sum_k A_b[i][k] B_b[k][j], lane 4b+j holding column j of B_b and of
// D_b (rows i in its four result registers) and lane 4b+i holding row i of A_b.  With
// A_b[i][k] = dL[token i][expert 4g+k] (the same four tokens in every block) and
// B_b[k][j] = Wg[column of lane 4b+j][expert 4g+k], one instruction per column and expert
// group gives a lane the gate term of four tokens at one of its columns, at 1/8 of the issue
// slots of float FMAs.  dL is split into two bfloat16 terms (hi + lo), which keeps 16 bits of
// its mantissa; Wg is bfloat16 already.  The kernel is bound by the latency of its row reads,
// so it is built for many wavefronts: the gate weights stay in LDS (read again every round)
// rather than in 64 registers, which lets four wavefronts per SIMD run.
typedef short bf16x4_hw __attribute__((ext_vector_type(4)));
typedef float f32x4_hw __attribute__((ext_vector_type(4)));
constexpr int DXM_TOK = 16;          // tokens per token group
constexpr int DXM_CT = 64;           // column threads of a workgroup: one wavefront, 512 columns
constexpr int DXM_TG = 8;            // token groups per workgroup, one wavefront each (they share the gate weights in LDS)
template <int EG>                    // expert groups of four: E <= 4*EG
__global__ __launch_bounds__(DXM_CT * DXM_TG, 2) void dispatch_bwd_mfma_kernel(
    const bf16_t* __restrict__ dDI, const int* __restrict__ slot, const float* __restrict__ dL,
    const bf16_t* __restrict__ Wg, bf16_t* __restrict__ dx, int t_begin, int t_count, int M, int E, int k) {
    const int ct = threadIdx.x % DXM_CT;                       // column thread
    const int tg = __builtin_amdgcn_readfirstlane(threadIdx.x / DXM_CT);
    const int c = (blockIdx.x * DXM_CT + ct) * 8;
    const bool c_ok = c < M;                       // lanes beyond the row still feed the A operand
    const int lane = threadIdx.x & 63;
    const int tl0 = min((blockIdx.y * DXM_TG + tg) * DXM_TOK, t_count);
    const int tl1 = min(tl0 + DXM_TOK, t_count);
    // The slots of the group's (token, choice) pairs, one per lane (two registers cover 16 tokens x 8
    // choices); a pair's slot is then broadcast from its lane, which costs no memory access per row.
    const int nsl = (tl1 - tl0) * k;
    const int* sl0 = slot + (size_t)(t_begin + tl0) * k;
    const int sv0 = lane < nsl ? sl0[lane] : -1;
    const int sv1 = lane + 64 < nsl ? sl0[lane + 64] : -1;
    const int cc = c_ok ? c : 0;
    // rows of four tokens, choices j0 and j0 + 1: eight 16-byte reads in flight per lane, no branch
    // around them (a missing row is read from row 0 and replaced by zeros)
    auto request = [&](int tb, int j0, uint4 (&raw)[4][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int i = (tb - tl0 + u) * k + j0 + jj;
                const int s0 = __builtin_amdgcn_readlane(sv0, i & 63), s1 = __builtin_amdgcn_readlane(sv1, i & 63);
                const int sj = (tb + u < tl1 && j0 + jj < k) ? (i < 64 ? s0 : s1) : -1;
                const uint4 v = ld_row<true>(reinterpret_cast<const uint4*>(dDI + (size_t)max(sj, 0) * M + cc));
                raw[u][jj] = sj >= 0 ? v : make_uint4(0, 0, 0, 0);
            }
    };
    // gate gradients of this lane's token (tb + lane%4) for the A operand
    auto request_dl = [&](int tb, float4 (&dl)[EG]) {
        const int ta = tb + (lane & 3);
#pragma unroll
        for (int g = 0; g < EG; ++g) {
            dl[g] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (ta < tl1) {
                const float* row = dL + (size_t)(t_begin + ta) * E + 4 * g;
                if (E == 4 * EG) {
                    dl[g] = *reinterpret_cast<const float4*>(row);
                } else {
                    if (4 * g + 0 < E) dl[g].x = row[0];
                    if (4 * g + 1 < E) dl[g].y = row[1];
                    if (4 * g + 2 < E) dl[g].z = row[2];
                    if (4 * g + 3 < E) dl[g].w = row[3];
                }
            }
        }
    };
    // Gate weights of this workgroup's columns into LDS with coalesced 16-byte reads.  A lane's
    // piece (64*EG bytes: 8 columns x 4*EG experts) is padded by 16 bytes so that the reads of a
    // wavefront spread over all banks.  The weights are staged before the first rows are requested:
    // an LDS write waits for every load issued before it, and the rows take several times longer
    // to arrive than the weights.
    extern __shared__ __attribute__((aligned(16))) char dxm_smem[];
    constexpr int CHUNK = 64 * EG;
    constexpr int PITCH = CHUNK + 16;
    const int c_base = blockIdx.x * DXM_CT * 8;
    const int ncols = min(DXM_CT * 8, M - c_base);
    const int pieces = ncols * EG / 2;             // 16-byte pieces of the slice: at most two per thread
    static_assert(DXM_CT * 8 * 4 / 2 <= 2 * DXM_CT * DXM_TG, "two pieces per thread cover the slice");
    const bool whole = E == 4 * EG;
    uint4 piece[2];
    if (whole) {
        const uint4* src = reinterpret_cast<const uint4*>(Wg + (size_t)c_base * E);
#pragma unroll
        for (int i = 0; i < 2; ++i) piece[i] = src[min((int)threadIdx.x + i * DXM_CT * DXM_TG, pieces - 1)];
    }
    if (whole) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int q = threadIdx.x + i * DXM_CT * DXM_TG;
            const int byte = q * 16;
            if (q < pieces) *reinterpret_cast<uint4*>(dxm_smem + (byte / CHUNK) * PITCH + byte % CHUNK) = piece[i];
        }
    } else {
        for (int q = threadIdx.x; q < ncols * 4 * EG; q += DXM_CT * DXM_TG) {
            const int col = q / (4 * EG), e = q % (4 * EG);
            const bf16_t v = e < E ? Wg[(size_t)(c_base + col) * E + e] : (bf16_t)0;
            *reinterpret_cast<bf16_t*>(dxm_smem + (col / 8) * PITCH + (col % 8) * 8 * EG + e * 2) = v;
        }
    }
    uint4 raw[4][2];
    float4 dl[EG];
    request_dl(tl0, dl);
    request(tl0, 0, raw);
    __syncthreads();
    for (int tb = tl0; tb < tl1; tb += 4) {
        if (tb > tl0) {
            request_dl(tb, dl);
            request(tb, 0, raw);
        }
        bf16x4_hw a_hi[EG], a_lo[EG];
#pragma unroll
        for (int g = 0; g < EG; ++g) {
            const float v[4] = {dl[g].x, dl[g].y, dl[g].z, dl[g].w};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bf16_t h = f32_to_bf16(v[r]);
                a_hi[g][r] = (short)h;
                a_lo[g][r] = (short)f32_to_bf16(v[r] - bf16_to_f32(h));
            }
        }
        f32x4_hw gate[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) gate[i] = f32x4_hw{0.0f, 0.0f, 0.0f, 0.0f};
        int my_off = ct * PITCH;                   // opaque: the compiler must not keep the weights in registers
        asm volatile("" : "+v"(my_off));
#pragma unroll
        for (int g = 0; g < EG; ++g)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bf16x4_hw w = *reinterpret_cast<const bf16x4_hw*>(dxm_smem + my_off + (i * EG + g) * 8);
                gate[i] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_hi[g], w, gate[i], 0, 0, 0);
                gate[i] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_lo[g], w, gate[i], 0, 0, 0);
            }
        float acc[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float r0[8], r1[8];
            Unit<bf16_t>::to_float(raw[u][0], r0);
            Unit<bf16_t>::to_float(raw[u][1], r1);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[u][i] = gate[i][u] + (r0[i] + r1[i]);
        }
        for (int j0 = 2; j0 < k; j0 += 2) {            // further choices (k > 2)
            request(tb, j0, raw);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float r0[8], r1[8];
                Unit<bf16_t>::to_float(raw[u][0], r0);
                Unit<bf16_t>::to_float(raw[u][1], r1);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[u][i] += r0[i] + r1[i];
            }
        }
        if (c_ok) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (tb + u < tl1)
                    st_row<false>(reinterpret_cast<uint4*>(dx + (size_t)(t_begin + tb + u) * M + c), Unit<bf16_t>::from_float(acc[u]));
        }
    }
}

// dx[t] = sum_j dDI[slot[t,j]] + dL[t,:] Wg^T.  A thread owns eight columns and
// keeps their gate weights in registers across TOKB tokens.
constexpr int DXB_TOK = 32;
template <typename T, int EC>
__global__ __launch_bounds__(PERM_THREADS) void dispatch_bwd_kernel(
    const T* __restrict__ dDI, const int* __restrict__ slot, const float* __restrict__ dL,
    const T* __restrict__ Wg, T* __restrict__ dx, int t_begin, int t_count, int M, int E, int k) {
    const int c = (blockIdx.x * PERM_THREADS + threadIdx.x) * 8;
    if (c >= M) return;
    float wg[8][EC];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < EC; ++e) wg[i][e] = e < E ? Elem<T>::ld(Wg + (size_t)(c + i) * E + e) : 0.0f;
    const int tl0 = blockIdx.y * DXB_TOK;
    const int tl1 = min(tl0 + DXB_TOK, t_count);
    // four tokens per round so that their row reads are in flight together
    for (int tb = tl0; tb < tl1; tb += 4) {
        float acc[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[u][i] = 0.0f;
            const int tl = tb + u;
            if (tl >= tl1) continue;
            const int t = t_begin + tl;
            for (int j = 0; j < k; ++j) {
                int s = slot[(size_t)t * k + j];
                if (s < 0) continue;
                float r[8];
                Vec8<T>::load(dDI + (size_t)s * M + c, r);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[u][i] += r[i];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int tl = tb + u;
            if (tl >= tl1) continue;
            const int t = t_begin + tl;
            for (int e0 = 0; e0 < E; e0 += EC) {
#pragma unroll
                for (int e = 0; e < EC; ++e) {
                    if (e0 + e < E) {
                        float g = dL[(size_t)t * E + e0 + e];
                        if (E <= EC) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) acc[u][i] = fmaf(g, wg[i][e], acc[u][i]);
                        } else {
#pragma unroll
                            for (int i = 0; i < 8; ++i)
                                acc[u][i] = fmaf(g, Elem<T>::ld(Wg + (size_t)(c + i) * E + e0 + e), acc[u][i]);
                        }
                    }
                }
            }
            Vec8<T>::store(dx + (size_t)t * M + c, acc[u]);
        }
    }
}

// ---- gate backward ------------------------------------------------------------
//
// dL[t,e] = p[t,e] * (dp[t,e] - sum_e' dp[t,e'] p[t,e']) with dp nonzero only at the chosen
// experts (the softmax Jacobian applied to the combine-weight gradients), then
// dWg += x^T dL.  A workgroup of 256 threads prepares dL for a block of DWG_TOK tokens, four
// lanes per token.
constexpr int DWG_TOK = 64;
constexpr int DWG_EMAX = 64;
constexpr int DWG_LD = DWG_EMAX + 4;     // floats per row of the block's LDS tile

// Combine-weight gradients of the block's (token, choice) pairs into sdw[ti*k + j]: either given,
// or the fixed-order sum of the GEMM epilogue's column-block partial sums (four lanes per pair).
// A thread has at most DWG_TOK*8*4/256 = 8 pairs; their slots are all requested before the first
// row of partial sums is read.
__device__ __forceinline__ void gate_block_dw(
    float* sdw, const int* __restrict__ slot, const float* __restrict__ dw, const float* __restrict__ dw_part,
    int parts, int t_first, int nt, int k) {
    constexpr int NI = DWG_TOK * 8 * 4 / PERM_THREADS;
    const int total = nt * k * 4;
    const int sub = threadIdx.x & 3;
    int sl[NI];
    float given[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int q = threadIdx.x + i * PERM_THREADS;
        const size_t at = (size_t)t_first * k + (q >> 2);          // pairs of the block are consecutive
        sl[i] = (q < total && dw_part) ? slot[at] : -1;
        given[i] = (q < total && !dw_part && sub == 0) ? dw[at] : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int q = threadIdx.x + i * PERM_THREADS;
        if (q >= total) break;                                     // uniform over the four lanes of a pair
        float v = given[i];
        if (sl[i] >= 0) {
            const float* row = dw_part + (size_t)sl[i] * parts;
            if ((parts & 3) == 0) {
                // lane `sub` of the pair takes every fourth group of four partial sums, all
                // requested before the first is added (fixed order: groups ascending, then the lanes)
                const int ngrp = parts >> 2;
                for (int g0 = sub; g0 < ngrp; g0 += 32) {
                    float4 q4[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        q4[u] = (g0 + 4 * u < ngrp) ? *reinterpret_cast<const float4*>(row + 4 * (g0 + 4 * u))
                                                    : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
                    for (int u = 0; u < 8; ++u) v += (q4[u].x + q4[u].y) + (q4[u].z + q4[u].w);
                }
            } else {
                const int per = (parts + 3) >> 2;
                const int c1 = min(parts, (sub + 1) * per);
                for (int c = sub * per; c < c1; ++c) v += row[c];
            }
        }
        v += __shfl_xor(v, 1, 64);
        v += __shfl_xor(v, 2, 64);
        if (sub == 0) sdw[q >> 2] = v;
    }
}

// The block's logits (nt rows of E floats, contiguous in memory) into the LDS tile; a thread's
// loads (at most DWG_TOK*DWG_EMAX/256 = 16 floats) are all requested before the first is written.
__device__ __forceinline__ void gate_block_logits(float (*tile)[DWG_LD], const float* __restrict__ logits,
                                                  int t_first, int nt, int E) {
    const float* src = logits + (size_t)t_first * E;
    if ((E & 3) == 0 && (((size_t)t_first * E) & 3) == 0) {
        constexpr int NI = DWG_TOK * DWG_EMAX / 4 / PERM_THREADS;
        const int E4 = E >> 2, total = nt * E4;
        float4 v[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int q = threadIdx.x + i * PERM_THREADS;
            v[i] = q < total ? reinterpret_cast<const float4*>(src)[q] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int q = threadIdx.x + i * PERM_THREADS;
            if (q < total) *reinterpret_cast<float4*>(&tile[q / E4][4 * (q % E4)]) = v[i];
        }
    } else {
        for (int q = threadIdx.x; q < nt * E; q += PERM_THREADS) tile[q / E][q % E] = src[q];
    }
}

// The experts chosen by the token of this thread (thread / 4 within the block), -1 beyond k or past the
// last token; requested first so that the read is over by the time gate_block_dl needs it.
__device__ __forceinline__ void gate_block_ids(int (&ids)[8], const int* __restrict__ topk_idx, int t_first, int nt, int k) {
    const int ti = threadIdx.x >> 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) ids[j] = (ti < nt && j < k) ? topk_idx[(size_t)(t_first + ti) * k + j] : -1;
}

// dL of the block's tokens, four lanes per token (lane `sub` takes experts sub, sub+4, ...; maxima and
// sums are folded over the four lanes).  The LDS tile holds the logits on entry and dL on return, with
// zeros in the rows of missing tokens and in columns E .. E16-1 (E16 = E rounded up to 16).  dL also
// goes to global memory, and, if dLt is given, as two bfloat16 terms (hi + lo, 16 bits of mantissa)
// to dLt[(e/16)*32 + e%16][token] and dLt[(e/16)*32 + 16 + e%16][token], rows of tp_pad tokens.
__device__ __forceinline__ void gate_block_dl(
    float (*tile)[DWG_LD], const float* sdw, const int (&ids)[8], float* __restrict__ dL,
    bf16_t* __restrict__ dLt, int tp_pad, int t_first, int tl0, int nt, int E, int k, int renorm) {
    const int ti = threadIdx.x >> 2, sub = threadIdx.x & 3;
    const int E16 = (E + 15) & ~15;
    const bool live = ti < nt;
    const int t = t_first + ti;
    float* row = tile[ti];
    float mx = -INFINITY;
    if (live)
        for (int e = sub; e < E; e += 4) mx = fmaxf(mx, row[e]);
    mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
    float g[8], pc[8];                  // gradient and exp(logit - max) of the chosen experts
    float den = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        g[j] = 0.0f; pc[j] = 0.0f;
        if (live && j < k) {
            g[j] = sdw[ti * k + j];
            pc[j] = expf(row[ids[j]] - mx);
            den += pc[j];
        }
    }
    if (!renorm) {
        float sum = 0.0f;
        if (live)
            for (int e = sub; e < E; e += 4) sum += expf(row[e] - mx);
        sum += __shfl_xor(sum, 1, 64);
        sum += __shfl_xor(sum, 2, 64);
        den = sum;
    }
    // (renormalised weights are a softmax over the chosen logits only: dL_e = w_j (dw_j - sum_j' dw_j' w_j')
    // for a chosen e, zero otherwise)
    const float inv = 1.0f / den;
    float inner = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) inner = fmaf(g[j], pc[j] * inv, inner);
    for (int e = sub; e < E16; e += 4) {
        float v = 0.0f;
        if (live && e < E) {
            float dp = 0.0f;
            bool chosen = false;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (ids[j] == e) { dp = g[j]; chosen = true; }
            if (!renorm) v = expf(row[e] - mx) * inv * (dp - inner);
            else if (chosen) v = expf(row[e] - mx) * inv * (dp - inner);
            dL[(size_t)t * E + e] = v;
        }
        row[e] = v;
        if (dLt) {
            const bf16_t hi = f32_to_bf16(v);
            const bf16_t lo = f32_to_bf16(v - bf16_to_f32(hi));
            bf16_t* col = dLt + ((size_t)((e >> 4) * 32 + (e & 15)) * tp_pad + tl0 + ti);
            col[0] = hi;
            col[(size_t)16 * tp_pad] = lo;
        }
    }
}

// One workgroup takes DWG_TOK tokens: first dL of those tokens (to global memory for the
// dispatch-backward kernel, and to LDS), then part[b][d][e] = sum over the tokens of
// x[t,d] * dL[t,e] in float FMAs, each thread owning eight columns d.
template <typename T>
__global__ __launch_bounds__(PERM_THREADS) void gate_bwd_kernel(
    const T* __restrict__ x, const float* __restrict__ logits, const int* __restrict__ topk_idx,
    const int* __restrict__ slot, const float* __restrict__ dw, const float* __restrict__ dw_part, int parts,
    float* __restrict__ dL, float* __restrict__ part, int t_begin, int t_count, int M, int E, int k, int renorm) {
    __shared__ __attribute__((aligned(16))) float sdl[DWG_TOK][DWG_LD];
    __shared__ float sdw[DWG_TOK * 8];
    const int tl0 = blockIdx.y * DWG_TOK;
    const int nt = min(DWG_TOK, t_count - tl0);
    int ids[8];
    gate_block_ids(ids, topk_idx, t_begin + tl0, nt, k);
    gate_block_logits(sdl, logits, t_begin + tl0, nt, E);
    gate_block_dw(sdw, slot, dw, dw_part, parts, t_begin + tl0, nt, k);
    __syncthreads();
    gate_block_dl(sdl, sdw, ids, dL, nullptr, 0, t_begin + tl0, tl0, nt, E, k, renorm);
    __syncthreads();
    for (int c = threadIdx.x * 8; c < M; c += PERM_THREADS * 8) {
        for (int e0 = 0; e0 < E; e0 += 16) {
            const int ne = min(16, E - e0);
            float acc[8][16];
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][e] = 0.0f;
            // Four token rows at a time, in two register sets in turn: the next four rows are
            // requested before the current four are used, with no branch between request and use.
            // Tokens past the end are clamped to the last one; their rows of sdl are zero.
            auto request = [&](Raw8<T>* r, int i0) {
#pragma unroll
                for (int u = 0; u < 4; ++u) r[u].load(x + (size_t)(t_begin + tl0 + min(i0 + u, nt - 1)) * M + c);
            };
            auto use = [&](const Raw8<T>* r, int i0) {
                float xv[4][8];
#pragma unroll
                for (int u = 0; u < 4; ++u) r[u].to_float(xv[u]);
                // the gradients of token u+1 are read from LDS while token u is multiplied
                float4 g4[2][4];
#pragma unroll
                for (int v = 0; v < 4; ++v) g4[0][v] = *reinterpret_cast<const float4*>(&sdl[i0][e0 + 4 * v]);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (u + 1 < 4) {
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            g4[(u + 1) & 1][v] = *reinterpret_cast<const float4*>(&sdl[i0 + u + 1][e0 + 4 * v]);
                    }
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float4 gq = g4[u & 1][v];
                        const float gd[4] = {gq.x, gq.y, gq.z, gq.w};
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4)
#pragma unroll
                            for (int q = 0; q < 8; ++q) acc[q][4 * v + r4] = fmaf(xv[u][q], gd[r4], acc[q][4 * v + r4]);
                    }
                }
            };
            static_assert(DWG_TOK % 8 == 0, "the loop below walks over sdl in steps of eight rows");
            Raw8<T> ca[4], cb[4];
            request(ca, 0);
            for (int i0 = 0; i0 < nt; i0 += 8) {
                // (the barriers keep the instruction scheduler from sinking the requests to their uses)
                request(cb, i0 + 4);
                __builtin_amdgcn_sched_barrier(0);
                use(ca, i0);
                __builtin_amdgcn_sched_barrier(0);
                request(ca, i0 + 8);
                __builtin_amdgcn_sched_barrier(0);
                use(cb, i0 + 4);
                __builtin_amdgcn_sched_barrier(0);
            }
            float* out = part + ((size_t)blockIdx.y * M + c) * E + e0;
            if (ne == 16 && (E & 3) == 0) {
#pragma unroll
                for (int q = 0; q < 8; ++q)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        *reinterpret_cast<float4*>(out + (size_t)q * E + 4 * v) =
                            make_float4(acc[q][4 * v], acc[q][4 * v + 1], acc[q][4 * v + 2], acc[q][4 * v + 3]);
            } else {
#pragma unroll
                for (int q = 0; q < 8; ++q)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (e < ne) out[(size_t)q * E + e] = acc[q][e];
            }
        }
    }
}


// bfloat16 storage: dL of one block of tokens per workgroup, to global memory in float (for the
// dispatch-backward kernel) and transposed as hi + lo bfloat16 terms (for the kernel below).
__global__ __launch_bounds__(PERM_THREADS) void gate_dl_kernel(
    const float* __restrict__ logits, const int* __restrict__ topk_idx, const int* __restrict__ slot,
    const float* __restrict__ dw, const float* __restrict__ dw_part, int parts, float* __restrict__ dL,
    bf16_t* __restrict__ dLt, int tp_pad, int t_begin, int t_count, int E, int k, int renorm) {
    __shared__ __attribute__((aligned(16))) float sdl[DWG_TOK][DWG_LD];
    __shared__ float sdw[DWG_TOK * 8];
    const int tl0 = blockIdx.x * DWG_TOK;
    const int nt = max(0, min(DWG_TOK, t_count - tl0));
    int ids[8];
    gate_block_ids(ids, topk_idx, t_begin + tl0, nt, k);
    gate_block_logits(sdl, logits, t_begin + tl0, nt, E);
    gate_block_dw(sdw, slot, dw, dw_part, parts, t_begin + tl0, nt, k);
    __syncthreads();
    gate_block_dl(sdl, sdw, ids, dL, dLt, tp_pad, t_begin + tl0, tl0, nt, E, k, renorm);
}

// part[s][d][e] = sum over the tokens of chunk s of x[t,d] * dL[t,e] on the matrix cores
// (bfloat16 storage).  The tokens are the reduction dimension of v_mfma_f32_32x32x16_bf16, and
// both operands want eight consecutive tokens in a lane: dL comes transposed from the kernel
// above; of x a lane reads one dword (two neighbouring columns) from each of eight token rows
// - every such read covers whole 128-byte lines of two rows - and splits them into the operand
// of the even and of the odd columns.  A wavefront owns 64 columns and a chunk of TC tokens;
// the first operand holds 32 columns of dL^T: sixteen experts' hi terms and their lo terms, so that
// hi and lo products land in accumulator registers q and q + 8 of the same lane.
// (The kernel is written for CPL = 2, 4 or 8 columns per lane; wider reads with fewer, fatter
// wavefronts measured no faster - 26-29 us for gate backward of 16384 x 2048 in every shape - and
// need more partial sums, so two it is.)
constexpr int DWG_CPL = 2;
typedef __bf16 gate_bf16x8 __attribute__((ext_vector_type(8)));
typedef float gate_f32x16 __attribute__((ext_vector_type(16)));
template <int W> struct GateWords;            // W dwords of a token row
template <> struct GateWords<1> { typedef unsigned type; static __device__ __forceinline__ unsigned word(const unsigned& v, int) { return v; } };
template <> struct GateWords<2> { typedef uint2 type; static __device__ __forceinline__ unsigned word(const uint2& v, int i) { return i == 0 ? v.x : v.y; } };
template <> struct GateWords<4> { typedef uint4 type; static __device__ __forceinline__ unsigned word(const uint4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; } };
template <int EB, int CPL>           // expert blocks of sixteen: E <= 16*EB; columns per lane
__global__ __launch_bounds__(PERM_THREADS) void gate_dwg_mfma_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ dLt, float* __restrict__ part,
    int t_begin, int t_count, int tp_pad, int M, int E, int S, int TC) {
    constexpr int U = (EB * CPL <= 4) ? 4 : 2;      // MFMA steps of 16 tokens requested together
    constexpr int BT = 16 * U;
    constexpr int W = CPL / 2;
    typedef typename GateWords<W>::type row_t;
    const int lane = threadIdx.x & 63, r = lane & 31, g = lane >> 5;
    const int ncb = (M + 32 * CPL - 1) / (32 * CPL);
    const int w = blockIdx.x * PERM_WAVES + (threadIdx.x >> 6);
    const int cb = w % ncb, s = w / ncb;
    if (s >= S) return;
    const int t0 = s * TC, t1 = min(t0 + TC, tp_pad);
    const int c = cb * 32 * CPL + CPL * r;
    const row_t* xcol = reinterpret_cast<const row_t*>(x + (size_t)t_begin * M + min(c, M - CPL));
    const size_t row_units = (size_t)(M / CPL);
    struct Blk { row_t xa[U][8]; uint4 b[U][EB]; };
    // tokens past the partition are clamped to its last one (their dL is zero); a block past the
    // chunk is requested from the last block of the buffer and never used
    auto request = [&](Blk& q, int tb) {
        tb = min(tb, tp_pad - BT);
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                q.xa[u][j] = xcol[(size_t)min(tb + 16 * u + 8 * g + j, t_count - 1) * row_units];
#pragma unroll
            for (int eb = 0; eb < EB; ++eb)
                q.b[u][eb] = *reinterpret_cast<const uint4*>(dLt + ((size_t)(eb * 32 + r) * tp_pad + tb + 16 * u + 8 * g));
        }
    };
    gate_f32x16 acc[CPL][EB];
#pragma unroll
    for (int p = 0; p < CPL; ++p)
#pragma unroll
        for (int eb = 0; eb < EB; ++eb)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[p][eb][q] = 0.0f;
    auto use = [&](const Blk& q) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int p = 0; p < CPL; ++p) {
                // column p of the lane over its eight tokens: the low or the high halves of word p/2
                unsigned o[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const unsigned a = GateWords<W>::word(q.xa[u][2 * i], p >> 1), b2 = GateWords<W>::word(q.xa[u][2 * i + 1], p >> 1);
                    o[i] = (p & 1) ? ((a >> 16) | (b2 & 0xffff0000u)) : ((a & 0xffffu) | (b2 << 16));
                }
                const gate_bf16x8 x8 = __builtin_bit_cast(gate_bf16x8, make_uint4(o[0], o[1], o[2], o[3]));
#pragma unroll
                for (int eb = 0; eb < EB; ++eb)
                    acc[p][eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(gate_bf16x8, q.b[u][eb]), x8,
                                                                         acc[p][eb], 0, 0, 0);
            }
    };
    Blk ka, kb;
    request(ka, t0);
    for (int tb = t0; tb < t1; tb += 2 * BT) {
        // (the barriers keep the instruction scheduler from sinking the requests to their uses)
        request(kb, tb + BT);
        __builtin_amdgcn_sched_barrier(0);
        use(ka);
        __builtin_amdgcn_sched_barrier(0);
        request(ka, tb + 2 * BT);
        __builtin_amdgcn_sched_barrier(0);
        if (tb + BT < t1) use(kb);
        __builtin_amdgcn_sched_barrier(0);
    }
    // Accumulator register q of lane (r, g) belongs to column r of the x operand and to row
    // 8*(q/4) + 4*g + q%4 of dL^T: rows 0-15 are the hi terms of sixteen experts, rows 16-31 their lo terms.
    if (c >= M) return;
#pragma unroll
    for (int p = 0; p < CPL; ++p) {
        float* out = part + ((size_t)s * M + c + p) * E;
#pragma unroll
        for (int eb = 0; eb < EB; ++eb)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int e0 = 16 * eb + 8 * h + 4 * g;
                float v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = acc[p][eb][4 * h + i] + acc[p][eb][4 * h + i + 8];
                if ((E & 3) == 0) {
                    if (e0 < E) *reinterpret_cast<float4*>(out + e0) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (e0 + i < E) out[e0 + i] = v[i];
                }
            }
    }
}

// dWg[i] += sum_b part[b][i]: 32 consecutive outputs per workgroup, eight threads per output
// each taking every eighth partial block, then a fixed-order sum of the eight.
__global__ __launch_bounds__(256) void gate_dwg_reduce_kernel(
    const float* __restrict__ part, float* __restrict__ dWg, int nblk, int ME, int store) {
    __shared__ float red[8][32];
    const int col = threadIdx.x & 31, sl = threadIdx.x >> 5;
    const int i = blockIdx.x * 32 + col;
    float s = 0.0f;
    if (i < ME)
        for (int b = sl; b < nblk; b += 8) s += part[(size_t)b * ME + i];
    red[sl][col] = s;
    __syncthreads();
    if (sl == 0 && i < ME) {
        float tot = 0.0f;
#pragma unroll
        for (int q = 0; q < 8; ++q) tot += red[q][col];
        dWg[i] = store ? tot : dWg[i] + tot;
    }
}

template <typename T>
static moe_status dispatch_t(const Dims& d, int part, const void* src, const int* slot, void* DI,
                             const void* saved, float* dw, hipStream_t s) {
    dim3 grid((d.Tp + PERM_WAVES - 1) / PERM_WAVES);
    ProfScope ps(PK_DISPATCH, s);
    if (saved && dw)
        hipLaunchKernelGGL((dispatch_kernel<T, true>), grid, dim3(PERM_THREADS), 0, s, (const T*)src, slot,
                           (T*)DI, (const T*)saved, dw, part * d.Tp, d.Tp, d.M, d.k);
    else
        hipLaunchKernelGGL((dispatch_kernel<T, false>), grid, dim3(PERM_THREADS), 0, s, (const T*)src, slot,
                           (T*)DI, (const T*)nullptr, (float*)nullptr, part * d.Tp, d.Tp, d.M, d.k);
    count_launch(LC_PERMUTE);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

template <typename T>
static moe_status dispatch_bwd_t(const Dims& d, int part, const void* dDI, const int* slot, const float* dL,
                                 const void* Wg, void* dx, hipStream_t s) {
    if (sizeof(T) == 2 && d.E <= 16) {      // more experts: the gate weights no longer fit a lane's registers
        dim3 grid((d.M / 8 + DXM_CT - 1) / DXM_CT, (d.Tp + DXM_TOK * DXM_TG - 1) / (DXM_TOK * DXM_TG));
#define LAUNCH_DXM(EG) do { \
        const int lds = DXM_CT * (64 * EG + 16); \
        static bool attr_done = false; \
        if (!attr_done) { \
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(dispatch_bwd_mfma_kernel<EG>), \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, lds)); \
            attr_done = true; \
        } \
        hipLaunchKernelGGL((dispatch_bwd_mfma_kernel<EG>), grid, dim3(DXM_CT * DXM_TG), lds, s, \
        (const bf16_t*)dDI, slot, dL, (const bf16_t*)Wg, (bf16_t*)dx, part * d.Tp, d.Tp, d.M, d.E, d.k); } while (0)
        ProfScope ps(PK_DISPATCH_BWD, s);
        if (d.E <= 4) LAUNCH_DXM(1);
        else if (d.E <= 8) LAUNCH_DXM(2);
        else LAUNCH_DXM(4);
#undef LAUNCH_DXM
        count_launch(LC_PERMUTE);
        MOE_CHECK_LAUNCH();
        return MOE_OK;
    }
    const size_t wg_float_bytes = (size_t)d.M * d.E * sizeof(float);
    if (wg_float_bytes <= 128 * 1024) {
        auto kern = dispatch_bwd_f32lds_kernel<T>;
        static size_t attr_bytes = 0;                 // largest size asked for so far
        if (wg_float_bytes > attr_bytes) {
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)wg_float_bytes));
            attr_bytes = wg_float_bytes;
        }
        int blocks = (d.Tp + 2 * DXF_WAVES - 1) / (2 * DXF_WAVES);
        const int cap = wg_float_bytes > 64 * 1024 ? 256 : 512;      // workgroups that fit the chip at once
        if (blocks > cap) blocks = cap;
        ProfScope ps(PK_DISPATCH_BWD, s);
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(DXF_THREADS), wg_float_bytes, s, (const T*)dDI, slot, dL,
                           (const T*)Wg, (T*)dx, part * d.Tp, d.Tp, d.M, d.E, d.k);
        count_launch(LC_PERMUTE);
        MOE_CHECK_LAUNCH();
        return MOE_OK;
    }
    dim3 grid((d.M / 8 + PERM_THREADS - 1) / PERM_THREADS, (d.Tp + DXB_TOK - 1) / DXB_TOK);
#define LAUNCH_DXB(EC) hipLaunchKernelGGL((dispatch_bwd_kernel<T, EC>), grid, dim3(PERM_THREADS), 0, s, \
        (const T*)dDI, slot, dL, (const T*)Wg, (T*)dx, part * d.Tp, d.Tp, d.M, d.E, d.k)
    ProfScope ps(PK_DISPATCH_BWD, s);
    if (d.E <= 4) LAUNCH_DXB(4);
    else if (d.E <= 8) LAUNCH_DXB(8);
    else LAUNCH_DXB(16);
#undef LAUNCH_DXB
    count_launch(LC_PERMUTE);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

// Shape of the bfloat16 gate-backward: token chunks of the matrix-core kernel and the two regions of
// the scratch buffer (partial sums [S][M][E] float, then dL^T [EB*32][tp_pad] bfloat16).
struct GateMfmaPlan { int tp_pad, EB, ncb, S, TC; size_t dlt_off, bytes; };
static GateMfmaPlan gate_mfma_plan(const Dims& d) {
    GateMfmaPlan g;
    g.tp_pad = (d.Tp + DWG_TOK - 1) / DWG_TOK * DWG_TOK;
    g.EB = (d.E + 15) / 16;
    g.ncb = (d.M + 32 * DWG_CPL - 1) / (32 * DWG_CPL);
    const int blocks = g.tp_pad / 64;
    int S = 1024 / g.ncb;                     // about one wavefront per SIMD: more of them were slower
    S = S < 1 ? 1 : (S > blocks ? blocks : S);
    g.TC = (blocks + S - 1) / S * 64;
    g.S = (g.tp_pad + g.TC - 1) / g.TC;
    g.dlt_off = ((size_t)g.S * d.M * d.E * sizeof(float) + 255) / 256 * 256;
    g.bytes = g.dlt_off + (size_t)g.EB * 32 * g.tp_pad * sizeof(bf16_t);
    return g;
}

static void launch_dwg_reduce(const Dims& d, int part, const void* scratch, float* dWg, int nblk, hipStream_t s) {
    const int ME = d.M * d.E;
    hipLaunchKernelGGL(gate_dwg_reduce_kernel, dim3((ME + 31) / 32), dim3(256), 0, s,
                       (const float*)scratch, dWg, nblk, ME, (d.overwrite && part == 0) ? 1 : 0);
}

template <typename T>
static moe_status gate_bwd_t(const Dims& d, int part, const void* x, const float* logits, const int* idx,
                             const int* slot, const float* dw, const float* dw_part, int parts,
                             float* dL, float* dWg, void* scratch, hipStream_t s) {
    ProfScope ps(PK_GATE_BWD, s);
    if constexpr (sizeof(T) == 2) {
        const GateMfmaPlan g = gate_mfma_plan(d);
        bf16_t* dLt = reinterpret_cast<bf16_t*>((char*)scratch + g.dlt_off);
        hipLaunchKernelGGL(gate_dl_kernel, dim3(g.tp_pad / DWG_TOK), dim3(PERM_THREADS), 0, s, logits, idx, slot, dw,
                           dw_part, parts, dL, dLt, g.tp_pad, part * d.Tp, d.Tp, d.E, d.k, d.renorm);
        MOE_CHECK_LAUNCH();
        const dim3 grid((g.ncb * g.S + PERM_WAVES - 1) / PERM_WAVES);
#define LAUNCH_DWG(EB) hipLaunchKernelGGL((gate_dwg_mfma_kernel<EB, DWG_CPL>), grid, dim3(PERM_THREADS), 0, s, (const bf16_t*)x, \
                           dLt, (float*)scratch, part * d.Tp, d.Tp, g.tp_pad, d.M, d.E, g.S, g.TC)
        if (g.EB == 1) LAUNCH_DWG(1);
        else if (g.EB == 2) LAUNCH_DWG(2);
        else LAUNCH_DWG(4);
#undef LAUNCH_DWG
        MOE_CHECK_LAUNCH();
        launch_dwg_reduce(d, part, scratch, dWg, g.S, s);
        count_launch(LC_OTHER, 3);
        MOE_CHECK_LAUNCH();
        return MOE_OK;
    } else {
        const int nblk = (d.Tp + DWG_TOK - 1) / DWG_TOK;
        hipLaunchKernelGGL((gate_bwd_kernel<T>), dim3(1, nblk), dim3(PERM_THREADS), 0, s, (const T*)x, logits, idx,
                           slot, dw, dw_part, parts, dL, (float*)scratch, part * d.Tp, d.Tp, d.M, d.E, d.k, d.renorm);
        MOE_CHECK_LAUNCH();
        launch_dwg_reduce(d, part, scratch, dWg, nblk, s);
        count_launch(LC_OTHER, 2);
        MOE_CHECK_LAUNCH();
        return MOE_OK;
    }
}

}  // namespace moe

using namespace moe;

extern "C" moe_status moe_dispatch(const moe_config* cfg, int32_t part, const void* src, const int32_t* slot,
                                   void* DI, const void* dO_saved, float* dw, void* stream) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    MOE_TRY(check_part(d, part));
    if (!src || !slot || !DI) return MOE_ERR_NULL;
    if (d.dtype == MOE_F32) return dispatch_t<float>(d, part, src, slot, DI, dO_saved, dw, (hipStream_t)stream);
    return dispatch_t<bf16_t>(d, part, src, slot, DI, dO_saved, dw, (hipStream_t)stream);
}

extern "C" moe_status moe_combine(const moe_config* cfg, int32_t part, const void* DO, const int32_t* slot,
                                  const float* topk_w, void* y, void* stream) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    MOE_TRY(check_part(d, part));
    if (!DO || !slot || !topk_w || !y) return MOE_ERR_NULL;
    dim3 grid((d.Tp + PERM_WAVES - 1) / PERM_WAVES);
    hipStream_t s = (hipStream_t)stream;
    ProfScope ps(PK_COMBINE, s);
    if (d.dtype == MOE_F32)
        hipLaunchKernelGGL((combine_kernel<float>), grid, dim3(PERM_THREADS), 0, s, (const float*)DO, slot,
                           topk_w, (float*)y, part * d.Tp, d.Tp, d.M, d.k);
    else
        hipLaunchKernelGGL((combine_kernel<bf16_t>), grid, dim3(PERM_THREADS), 0, s, (const bf16_t*)DO, slot,
                           topk_w, (bf16_t*)y, part * d.Tp, d.Tp, d.M, d.k);
    count_launch(LC_PERMUTE);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

namespace moe {
moe_status zero_dropped(const Dims& d, const int* slot, void* y, hipStream_t s) {
    dim3 grid((d.T + PERM_WAVES - 1) / PERM_WAVES);
    if (d.dtype == MOE_F32)
        hipLaunchKernelGGL((zero_dropped_kernel<float>), grid, dim3(PERM_THREADS), 0, s, slot, (float*)y, d.T, d.M);
    else
        hipLaunchKernelGGL((zero_dropped_kernel<bf16_t>), grid, dim3(PERM_THREADS), 0, s, slot, (bf16_t*)y, d.T, d.M);
    count_launch(LC_OTHER);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}
}  // namespace moe

extern "C" moe_status moe_dispatch_bwd(const moe_config* cfg, int32_t part, const void* dDI, const int32_t* slot,
                                       const float* dL, const void* Wg, void* dx, void* stream) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    MOE_TRY(check_part(d, part));
    if (!dDI || !slot || !dL || !Wg || !dx) return MOE_ERR_NULL;
    if (d.dtype == MOE_F32) return dispatch_bwd_t<float>(d, part, dDI, slot, dL, Wg, dx, (hipStream_t)stream);
    return dispatch_bwd_t<bf16_t>(d, part, dDI, slot, dL, Wg, dx, (hipStream_t)stream);
}

extern "C" moe_status moe_gate_scratch_bytes(const moe_config* cfg, size_t* bytes) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    if (!bytes) return MOE_ERR_NULL;
    *bytes = d.dtype == MOE_BF16 ? gate_mfma_plan(d).bytes
                                 : (size_t)((d.Tp + DWG_TOK - 1) / DWG_TOK) * d.M * d.E * sizeof(float);
    return MOE_OK;
}

extern "C" moe_status moe_gate_bwd(const moe_config* cfg, int32_t part, const void* x, const float* logits,
                                   const int32_t* topk_idx, const int32_t* slot, const float* dw,
                                   const float* dw_part, float* dL, float* dWg, void* scratch, void* stream) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    MOE_TRY(check_part(d, part));
    if (!x || !logits || !topk_idx || !slot || !dL || !dWg || !scratch) return MOE_ERR_NULL;
    if (!dw && !dw_part) return MOE_ERR_NULL;
    int parts = 0;
    MOE_TRY(moe_dw_parts(cfg, &parts));
    if (d.dtype == MOE_F32)
        return gate_bwd_t<float>(d, part, x, logits, topk_idx, slot, dw, dw_part, parts, dL, dWg, scratch,
                                 (hipStream_t)stream);
    return gate_bwd_t<bf16_t>(d, part, x, logits, topk_idx, slot, dw, dw_part, parts, dL, dWg, scratch,
                              (hipStream_t)stream);
}
