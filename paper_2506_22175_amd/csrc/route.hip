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

// softmax over E logits and the k largest of them; runs in one lane per token.  The row (EP floats in
// LDS, 16-byte aligned, E of them valid) is taken into registers first, so that nothing below waits on LDS;
// idx_out and w_out are the token's k places in global memory.
template <int EP>
__device__ __forceinline__ void softmax_topk(const float* lg, int E, int k, int renorm, int* idx_out, float* w_out) {
    float v[EP];
#pragma unroll
    for (int e4 = 0; e4 < EP / 4; ++e4) {
        const float4 q = *reinterpret_cast<const float4*>(lg + 4 * e4);
        v[4 * e4] = q.x; v[4 * e4 + 1] = q.y; v[4 * e4 + 2] = q.z; v[4 * e4 + 3] = q.w;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < EP; ++e)
        if (e < E) mx = fmaxf(mx, v[e]);
    float sum = 0.0f;
#pragma unroll
    for (int e = 0; e < EP; ++e)
        if (e < E) sum += expf(v[e] - mx);
    // the k largest logits in descending order, ties to the lower index; emit(j, expert, its logit)
    auto pick = [&](auto&& emit) __attribute__((always_inline)) {
        unsigned long long taken = 0ull;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            float bv = 0.0f, braw = 0.0f;
#pragma unroll
            for (int e = 0; e < EP; ++e) {
                if (e < E && !((taken >> e) & 1ull)) {
                    const float o = (v[e] != v[e]) ? -INFINITY : v[e];       // NaN orders as -inf
                    if (best < 0 || o > bv) { best = e; bv = o; braw = v[e]; }
                }
            }
            taken |= 1ull << best;
            emit(j, best, braw);
        }
    };
    // weights: the chosen probabilities, or those divided by their sum over the k choices
    float den = sum;
    if (renorm) {
        den = 0.0f;
        pick([&](int, int, float raw) __attribute__((always_inline)) { den += expf(raw - mx); });
    }
    pick([&](int j, int best, float raw) __attribute__((always_inline)) {
        idx_out[j] = best;
        w_out[j] = expf(raw - mx) / den;
    });
}

// Eight consecutive elements of a token row through a buffer descriptor: a lane past the end of
// the descriptor gets zeros, so the loads sit in straight-line code and stay in flight while
// the previous elements are multiplied.
template <typename T> struct RowLoad;
template <> struct RowLoad<bf16_t> {
    static __device__ __forceinline__ void load(Raw8<bf16_t>& r, __amdgpu_buffer_rsrc_t rs, unsigned off) {
        r.u = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));
    }
};
template <> struct RowLoad<float> {
    static __device__ __forceinline__ void load(Raw8<float>& r, __amdgpu_buffer_rsrc_t rs, unsigned off) {
        r.a = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));
        r.b = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rs, off + 16u, 0, 0));
    }
};

// tokens whose logits a wavefront keeps in LDS before it ranks them (1 KB of LDS per padded expert
// for the workgroup; with 64 experts half as many, so that 512 gate-weight rows still fit beside them)
template <int EP> struct RouteHeld { static constexpr int N = EP >= 64 ? 16 : 32; };

// EP = E rounded up to a power of two (>= 4); TB tokens per wavefront, TB*EP <= 64.
// MC = gate-weight rows held in LDS at a time (multiple of 512, or >= M).
//
// A wavefront multiplies TB tokens at a time (a group) and parks their logits in LDS; once
// RouteHeld tokens are parked, or its groups are done, one lane per token does softmax and
// top-k, so that the serial part runs once for many tokens instead of once per group.
template <typename T, int EP, int TB>
__global__ __launch_bounds__(ROUTE_THREADS) void route_kernel(
    const T* __restrict__ x, const T* __restrict__ Wg, const float* __restrict__ bias,
    float* __restrict__ logits, int* __restrict__ topk_idx, float* __restrict__ topk_w,
    int Ttot, int M, int E, int k, int MC, int renorm) {
    extern __shared__ float smem[];
    float* wl = smem;                               // [MC/8 ... ] see index below
    float* lg = smem + (size_t)MC * EP;             // [ROUTE_WAVES][HELD][EP]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform, and visibly so
    const int ngroups = (Ttot + ROUTE_WAVES * TB - 1) / (ROUTE_WAVES * TB);
    const int nchunks = (M + MC - 1) / MC;
    constexpr int E4 = EP / 4;
    constexpr unsigned ES = sizeof(T);
    constexpr int HELD = RouteHeld<EP>::N;
    float* mylg = lg + (size_t)wid * HELD * EP;
    int held = 0, held_g0 = 0;                      // parked tokens, and the group of the first of them

    // softmax and top-k of the parked tokens: token q of the wavefront belongs to group
    // held_g0 + (q / TB) * gridDim.x
    auto rank_held = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (lane < held) {
            const int gq = held_g0 + (lane / TB) * (int)gridDim.x;
            const int t = (gq * ROUTE_WAVES + wid) * TB + lane % TB;
            if (t < Ttot) {
                const float* my = mylg + lane * EP;
                if (E == EP) {
#pragma unroll
                    for (int e4 = 0; e4 < EP / 4; ++e4)
                        *reinterpret_cast<float4*>(logits + (size_t)t * E + 4 * e4) = *reinterpret_cast<const float4*>(my + 4 * e4);
                } else {
                    for (int e = 0; e < E; ++e) logits[(size_t)t * E + e] = my[e];
                }
                softmax_topk<EP>(my, E, k, renorm, topk_idx + (size_t)t * k, topk_w + (size_t)t * k);
            }
        }
        __builtin_amdgcn_wave_barrier();
        held = 0;
    };

    // the TB token rows of group g as one descriptor; rows past the last token read as zeros
    auto rows_of = [&](int g) __attribute__((always_inline)) {
        const int t0 = (g * ROUTE_WAVES + wid) * TB;
        const int nt = min(TB, Ttot - t0);
        const T* base = x + (size_t)(nt > 0 ? t0 : 0) * M;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(base), 0,
                                                 nt > 0 ? (int)((size_t)nt * M * ES) : 0, 0x00020000);
    };
    // elements d0 .. d0+7 of the TB rows (a lane with d0 >= M reads something it never uses)
    auto fetch = [&](__amdgpu_buffer_rsrc_t rs, int d0, Raw8<T>* r) __attribute__((always_inline)) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
            RowLoad<T>::load(r[tb], rs, (unsigned)(((size_t)tb * M + d0) * ES));
    };

    // gate-weight rows c0 .. c0+MC-1 into LDS (whole workgroup; barriers before and after).
    // between() runs after the weights have been requested and before they are written to LDS:
    // an LDS write waits for every load issued before it, so the first token rows are requested there.
    auto stage_weights = [&](int c0, auto&& between) __attribute__((always_inline)) {
        __syncthreads();
        // LDS element of (row dl, expert e): span = dl/512, lane l = (dl/8)%64, i = dl%8
        //   index = ((((span*8 + i) * E4 + e/4) * 64 + l) * 4 + e%4
        if (EP % 8 == 0 && E == EP && (reinterpret_cast<unsigned long long>(Wg) & 15ull) == 0) {
            // eight experts of one row per load; a thread's loads (at most eight: MC*EP <= 32768) are all
            // in flight before the first is converted
            constexpr int G = EP / 8 > 0 ? EP / 8 : 1;
            constexpr int NP = 32768 / 8 / ROUTE_THREADS;
            Raw8<T> wr[NP];
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int q = tid + i * ROUTE_THREADS;
                const int d = c0 + q / G;
                if (q < MC * G && d < M) wr[i].load(Wg + (size_t)d * E + (q % G) * 8);
                else wr[i].zero();
            }
            between();
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int q = tid + i * ROUTE_THREADS;
                if (q < MC * G) {
                    const int dl = q / G, e0 = (q % G) * 8;
                    float v[8];
                    wr[i].to_float(v);
                    const int span = dl >> 9, l = (dl >> 3) & 63, i8 = dl & 7;
                    float* dst = wl + ((((span * 8 + i8) * E4 + (e0 >> 2)) * 64 + l) << 2);
                    *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                    *reinterpret_cast<float4*>(dst + 256) = make_float4(v[4], v[5], v[6], v[7]);
                }
            }
        } else {
            between();
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
    };

    // acc += the 8 elements of each of the TB rows times the gate weights of LDS span sp; the
    // weights of element i+1 are read from LDS while element i is multiplied
    auto multiply_span = [&](float* acc, const Raw8<T>* xr, int sp) __attribute__((always_inline)) {
        float xs[TB][8];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) xr[tb].to_float(xs[tb]);
        float4 wv[2][E4];
        const float* wsp = wl + (((sp * 8) * E4 * 64 + lane) << 2);
#pragma unroll
        for (int e4 = 0; e4 < E4; ++e4) wv[0][e4] = *reinterpret_cast<const float4*>(wsp + ((e4 * 64) << 2));
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (i + 1 < 8) {
#pragma unroll
                for (int e4 = 0; e4 < E4; ++e4)
                    wv[(i + 1) & 1][e4] = *reinterpret_cast<const float4*>(wsp + ((((i + 1) * E4 + e4) * 64) << 2));
            }
#pragma unroll
            for (int e4 = 0; e4 < E4; ++e4) {
                const float4 w4 = wv[i & 1][e4];
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    float* a = acc + tb * EP + e4 * 4;
                    a[0] = __builtin_fmaf(xs[tb][i], w4.x, a[0]);
                    a[1] = __builtin_fmaf(xs[tb][i], w4.y, a[1]);
                    a[2] = __builtin_fmaf(xs[tb][i], w4.z, a[2]);
                    a[3] = __builtin_fmaf(xs[tb][i], w4.w, a[3]);
                }
            }
        }
    };

    // fold the lane sums of group g, add the bias, park the logits; rank once enough are parked
    auto finish_group = [&](float* acc, int g) __attribute__((always_inline)) {
        fold_lanes<TB * EP, 32>(acc, lane);
        // lane l now holds value index vi = l >> SH in acc[0]; vi = tb*EP + e
        constexpr int NV = TB * EP;
        constexpr int SH = (NV == 64) ? 0 : (NV == 32) ? 1 : (NV == 16) ? 2 : (NV == 8) ? 3 : (NV == 4) ? 4 : 5;
        if (held == 0) held_g0 = g;
        const int vi = lane >> SH;
        const int e = vi % EP;
        if ((lane & ((1 << SH) - 1)) == 0 && e < E) {
            float v = acc[0];
            if (bias) v = v + bias[e];
            mylg[held * EP + vi] = v;
        }
        held += TB;
        if (held + TB > HELD) rank_held();
    };

    float acc[TB * EP];
#pragma unroll
    for (int i = 0; i < TB * EP; ++i) acc[i] = 0.0f;
    const int d_lane = lane * 8;

    if (nchunks == 1) {
        // The whole gate matrix stays in LDS.  Token elements are requested one span ahead of the
        // multiplications, across group boundaries, into two register sets in turn; past the last
        // group the descriptor is empty and the requests cost nothing.
        const int nspan = (M + 511) / 512;
        int rg = blockIdx.x, rsp = 0;               // the span to request next
        auto request = [&](Raw8<T>* r) __attribute__((always_inline)) {
            fetch(rows_of(rg), rsp * 512 + d_lane, r);
            if (++rsp == nspan) { rsp = 0; rg += gridDim.x; }
        };
        Raw8<T> xa[TB], xb[TB];
        stage_weights(0, [&]() __attribute__((always_inline)) { request(xa); });
        int g = blockIdx.x, sp = 0;                 // the span to multiply next
        auto multiply = [&](const Raw8<T>* cur) __attribute__((always_inline)) {
            if (sp * 512 + d_lane < M) multiply_span(acc, cur, sp);
            if (++sp == nspan) {
                finish_group(acc, g);
#pragma unroll
                for (int i = 0; i < TB * EP; ++i) acc[i] = 0.0f;
                sp = 0;
                g += gridDim.x;
            }
            return g < ngroups;
        };
        for (;;) {
            // (the barriers keep the instruction scheduler from sinking the requests to their uses)
            request(xb);
            __builtin_amdgcn_sched_barrier(0);
            if (!multiply(xa)) break;
            request(xa);
            __builtin_amdgcn_sched_barrier(0);
            if (!multiply(xb)) break;
        }
    } else {
        // The gate matrix passes through LDS in pieces of MC rows for every group of tokens.
        for (int g = blockIdx.x; g < ngroups; g += gridDim.x) {
            const __amdgpu_buffer_rsrc_t rs = rows_of(g);
            for (int ch = 0; ch < nchunks; ++ch) {
                const int c0 = ch * MC;
                stage_weights(c0, []() {});
                const int nspan = (min(MC, M - c0) + 511) / 512;
                for (int sp = 0; sp < nspan; ++sp) {
                    const int d0 = c0 + sp * 512 + d_lane;
                    Raw8<T> xr[TB];
                    fetch(rs, d0, xr);
                    if (d0 < M) multiply_span(acc, xr, sp);
                }
            }
            finish_group(acc, g);
#pragma unroll
            for (int i = 0; i < TB * EP; ++i) acc[i] = 0.0f;
        }
    }
    if (held > 0) rank_held();
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
    size_t lds = ((size_t)MC * EP + (size_t)ROUTE_WAVES * RouteHeld<EP>::N * EP) * sizeof(float);
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
