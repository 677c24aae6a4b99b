// Gate of the MoE layer: float logits in a fixed summation order, softmax over
// all experts, top-k on the logits (Sections II-B2 and IV-A of the paper: a
// linear gate with E*M parameters and a top-k choice; the paper itself uses
// k = 1).  One wavefront handles TB tokens at a time; the gate weights sit in
// LDS as float, laid out so that every lane reads its own bank.
//
// Summation order (the same order is written out in the CPU oracle, which
// shares no code with this file): element d of a token row belongs to lane
// (d / 8) mod 64; a lane folds its elements in ascending d with one fused
// multiply-add each, starting from +0; the 64 lane sums are folded pairwise
// with offsets 32, 16, 8, 4, 2, 1; the bias is added last.
#include "common.h"

namespace moe {

// Pairwise folding of NV values per lane across the 64 lanes.  While more than
// one value is left, the two lanes of a pair split the values between them
// (each keeps one half and adds the partner's copy of that half); the sums are
// the same ones a full butterfly would produce, since a + b == b + a exactly.
// On return v[0] of lane l is the total of value index l >> (6 - log2 NV0).
template <int NV, int OFF>
__device__ __forceinline__ void fold_lanes(float* v, int lane) {
    if constexpr (OFF >= 1) {
        if constexpr (NV > 1) {
            constexpr int HALF = NV / 2;
            const bool upper = (lane & OFF) != 0;
#pragma unroll
            for (int i = 0; i < HALF; ++i) {
                float send = upper ? v[i] : v[i + HALF];
                float keep = upper ? v[i + HALF] : v[i];
                float recv = __shfl_xor(send, OFF, 64);
                v[i] = keep + recv;
            }
            fold_lanes<HALF, OFF / 2>(v, lane);
        } else {
            v[0] = v[0] + __shfl_xor(v[0], OFF, 64);
            fold_lanes<1, OFF / 2>(v, lane);
        }
    }
}

constexpr int ROUTE_THREADS = 512;
constexpr int ROUTE_WAVES = ROUTE_THREADS / 64;

// softmax over E logits and the k largest of them; runs in one lane per token
__device__ __forceinline__ void softmax_topk(const float* lg, int E, int k, int renorm, int* idx_out, float* w_out) {
    float mx = -INFINITY;
    for (int e = 0; e < E; ++e) mx = fmaxf(mx, lg[e]);
    float sum = 0.0f;
    for (int e = 0; e < E; ++e) sum += expf(lg[e] - mx);
    unsigned long long taken = 0ull;
    for (int j = 0; j < k; ++j) {
        int best = -1;
        float bv = 0.0f;
        for (int e = 0; e < E; ++e) {
            if ((taken >> e) & 1ull) continue;
            float v = lg[e];
            if (v != v) v = -INFINITY;           // NaN orders as -inf
            if (best < 0 || v > bv) { best = e; bv = v; }
        }
        taken |= 1ull << best;
        idx_out[j] = best;
        w_out[j] = expf(lg[best] - mx);
    }
    // weights: the chosen probabilities, or those divided by their sum over the k choices
    float den = sum;
    if (renorm) {
        den = 0.0f;
        for (int j = 0; j < k; ++j) den += w_out[j];
    }
    for (int j = 0; j < k; ++j) w_out[j] = w_out[j] / den;
}

// EP = E rounded up to a power of two (>= 4); TB tokens per wavefront, TB*EP <= 64.
// MC = gate-weight rows held in LDS at a time (multiple of 512, or >= M).
template <typename T, int EP, int TB>
__global__ __launch_bounds__(ROUTE_THREADS) void route_kernel(
    const T* __restrict__ x, const T* __restrict__ Wg, const float* __restrict__ bias,
    float* __restrict__ logits, int* __restrict__ topk_idx, float* __restrict__ topk_w,
    int Ttot, int M, int E, int k, int MC, int renorm) {
    extern __shared__ float smem[];
    float* wl = smem;                               // [MC/8 ... ] see index below
    float* lg = smem + (size_t)MC * EP;             // [ROUTE_WAVES][TB][EP]
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int ngroups = (Ttot + ROUTE_WAVES * TB - 1) / (ROUTE_WAVES * TB);
    const int nchunks = (M + MC - 1) / MC;
    constexpr int E4 = EP / 4;

    for (int g = blockIdx.x; g < ngroups; g += gridDim.x) {
        const int t0 = (g * ROUTE_WAVES + wid) * TB;
        float acc[TB * EP];
#pragma unroll
        for (int i = 0; i < TB * EP; ++i) acc[i] = 0.0f;

        for (int ch = 0; ch < nchunks; ++ch) {
            const int c0 = ch * MC;
            if (nchunks > 1 || g == (int)blockIdx.x) {
                __syncthreads();
                // LDS element of (row dl, expert e): span = dl/512, lane l = (dl/8)%64, i = dl%8
                //   index = ((((span*8 + i) * E4 + e/4) * 64 + l) * 4 + e%4
                if (EP % 8 == 0 && E == EP && (reinterpret_cast<unsigned long long>(Wg) & 15ull) == 0) {
                    // eight experts of one row per load, several loads in flight per thread
                    constexpr int G = EP / 8 > 0 ? EP / 8 : 1;
#pragma unroll 4
                    for (int q = tid; q < MC * G; q += ROUTE_THREADS) {
                        const int dl = q / G, e0 = (q % G) * 8;
                        const int d = c0 + dl;
                        float v[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
                        if (d < M) Vec8<T>::load(Wg + (size_t)d * E + e0, v);
                        const int span = dl >> 9, l = (dl >> 3) & 63, i = dl & 7;
                        float* dst = wl + ((((span * 8 + i) * E4 + (e0 >> 2)) * 64 + l) << 2);
                        *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                        *reinterpret_cast<float4*>(dst + 256) = make_float4(v[4], v[5], v[6], v[7]);
                    }
                } else {
                    for (int q = tid; q < MC * EP; q += ROUTE_THREADS) {
                        int dl = q / EP, e = q % EP;
                        int d = c0 + dl;
                        float v = 0.0f;
                        if (d < M && e < E) v = Elem<T>::ld(Wg + (size_t)d * E + e);
                        int span = dl >> 9, l = (dl >> 3) & 63, i = dl & 7;
                        wl[((((span * 8 + i) * E4 + (e >> 2)) * 64 + l) << 2) + (e & 3)] = v;
                    }
                }
                __syncthreads();
            }
            const int nspan = (min(MC, M - c0) + 511) / 512;
            // token elements of the next span are requested before the current span is multiplied
            Raw8<T> xr[TB], xn[TB];
            auto fetch = [&](int sp, Raw8<T>* r) {
                const int d0 = c0 + sp * 512 + lane * 8;
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    if (d0 < M && t0 + tb < Ttot) r[tb].load(x + (size_t)(t0 + tb) * M + d0);
                    else r[tb].zero();
                }
            };
            fetch(0, xr);
            for (int sp = 0; sp < nspan; ++sp) {
                const int d0 = c0 + sp * 512 + lane * 8;
                if (sp + 1 < nspan) fetch(sp + 1, xn);
                if (d0 < M) {
                    float xs[TB][8];
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) xr[tb].to_float(xs[tb]);
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
#pragma unroll
                        for (int e4 = 0; e4 < E4; ++e4) {
                            float4 wv = *reinterpret_cast<const float4*>(
                                wl + ((((sp * 8 + i) * E4 + e4) * 64 + lane) << 2));
#pragma unroll
                            for (int tb = 0; tb < TB; ++tb) {
                                float* a = acc + tb * EP + e4 * 4;
                                a[0] = __builtin_fmaf(xs[tb][i], wv.x, a[0]);
                                a[1] = __builtin_fmaf(xs[tb][i], wv.y, a[1]);
                                a[2] = __builtin_fmaf(xs[tb][i], wv.z, a[2]);
                                a[3] = __builtin_fmaf(xs[tb][i], wv.w, a[3]);
                            }
                        }
                    }
                }
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) xr[tb] = xn[tb];
            }
        }

        fold_lanes<TB * EP, 32>(acc, lane);
        // lane l now holds value index vi = l >> SH in acc[0]; vi = tb*EP + e
        constexpr int NV = TB * EP;
        constexpr int SH = (NV == 64) ? 0 : (NV == 32) ? 1 : (NV == 16) ? 2 : (NV == 8) ? 3 : (NV == 4) ? 4 : 5;
        {
            const int vi = lane >> SH;
            const int e = vi % EP;
            if ((lane & ((1 << SH) - 1)) == 0 && e < E) {
                float v = acc[0];
                if (bias) v = v + bias[e];
                lg[(wid * TB) * EP + vi] = v;
            }
        }
        __syncthreads();
        if (lane < TB && t0 + lane < Ttot) {
            const int t = t0 + lane;
            const float* my = lg + (wid * TB + lane) * EP;
            for (int e = 0; e < E; ++e) logits[(size_t)t * E + e] = my[e];
            int ids[8];
            float ws[8];
            softmax_topk(my, E, k, renorm, ids, ws);
            for (int j = 0; j < k; ++j) {
                topk_idx[(size_t)t * k + j] = ids[j];
                topk_w[(size_t)t * k + j] = ws[j];
            }
        }
    }
}

template <typename T, int EP, int TB>
static moe_status launch_route(const Dims& d, const void* x, const void* Wg, const float* bias,
                               float* logits, int* idx, float* w, hipStream_t s) {
    // Gate-weight rows held in LDS at a time.  If the whole matrix fits in 128 KB of
    // floats it is loaded once per workgroup, which then walks over many token groups;
    // otherwise it is streamed through LDS in 64 KB pieces for every token group.
    const int Mpad = ((d.M + 511) / 512) * 512;
    int MC = (32768 / EP) / 512 * 512;
    if (Mpad <= MC) MC = Mpad;
    else {
        MC = (16384 / EP) / 512 * 512;
        if (MC < 512) MC = 512;
    }
    size_t lds = ((size_t)MC * EP + (size_t)ROUTE_WAVES * TB * EP) * sizeof(float);
    auto kern = route_kernel<T, EP, TB>;
    static size_t attr_bytes = 0;                     // largest size asked for so far (per instantiation)
    if (lds > attr_bytes) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
        attr_bytes = lds;
    }
    int ngroups = (d.T + ROUTE_WAVES * TB - 1) / (ROUTE_WAVES * TB);
    const int cap = lds > 80 * 1024 ? 256 : 512;      // one or two workgroups per CU fit
    int grid = ngroups < cap ? ngroups : cap;
    ProfScope ps(PK_ROUTE, s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(ROUTE_THREADS), lds, s,
                       (const T*)x, (const T*)Wg, bias, logits, idx, w, d.T, d.M, d.E, d.k, MC, d.renorm);
    count_launch(LC_OTHER);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

template <typename T>
static moe_status route_dispatch(const Dims& d, const void* x, const void* Wg, const float* bias,
                                 float* logits, int* idx, float* w, hipStream_t s) {
    if (d.E <= 4) return launch_route<T, 4, 8>(d, x, Wg, bias, logits, idx, w, s);
    if (d.E <= 8) return launch_route<T, 8, 8>(d, x, Wg, bias, logits, idx, w, s);
    if (d.E <= 16) return launch_route<T, 16, 4>(d, x, Wg, bias, logits, idx, w, s);
    if (d.E <= 32) return launch_route<T, 32, 2>(d, x, Wg, bias, logits, idx, w, s);
    return launch_route<T, 64, 1>(d, x, Wg, bias, logits, idx, w, s);
}

}  // namespace moe

extern "C" moe_status moe_route(const moe_config* cfg, const void* x, const void* Wg, const float* gate_bias,
                                float* logits, int32_t* topk_idx, float* topk_w, void* stream) {
    moe::Dims d;
    MOE_TRY(moe::make_dims(cfg, &d));
    if (!x || !Wg || !logits || !topk_idx || !topk_w) return MOE_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (d.dtype == MOE_F32) return moe::route_dispatch<float>(d, x, Wg, gate_bias, logits, topk_idx, topk_w, s);
    return moe::route_dispatch<moe::bf16_t>(d, x, Wg, gate_bias, logits, topk_idx, topk_w, s);
}
