// Epilogues of the expert GEMMs, applied to four consecutive output columns of
// one row while the accumulators are still in registers.  The activation is
// exact GeLU and the stored middle tensor T_M is the pre-activation, so that
// backward can form both gelu(Z) and gelu'(Z) from it (Section II-B2 treats the
// activation as in place; Section III-D recomputes T_M from T_DI).
#pragma once
#include "common.h"

namespace moe {

template <typename T> struct Vec4;
template <> struct Vec4<float> {
    static __device__ __forceinline__ void load(const float* p, float* o) {
        float4 a = *reinterpret_cast<const float4*>(p);
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    }
    static __device__ __forceinline__ void store(float* p, const float* v) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
    static __device__ __forceinline__ float round(float v) { return v; }
};
template <> struct Vec4<bf16_t> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* o) {
        uint2 u = *reinterpret_cast<const uint2*>(p);
        o[0] = __uint_as_float(u.x << 16); o[1] = __uint_as_float(u.x & 0xffff0000u);
        o[2] = __uint_as_float(u.y << 16); o[3] = __uint_as_float(u.y & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float* v) {
        uint2 u;
        u.x = pack_bf16x2(v[0], v[1]);
        u.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2*>(p) = u;
    }
    static __device__ __forceinline__ float round(float v) { return bf16_to_f32(f32_to_bf16(v)); }
};

// Per-launch view of the epilogue operands for one expert.
template <typename T>
struct EpiCtx {
    T* C;            // output rows of this expert (ldc)
    float* Cf;       // EPI_ACCUM_F32 output
    T* Z;            // pre-activation rows of this expert (ldz), may be null for EPI_GELU
    const float* w;  // slot weights of this expert's rows
    int ldc, ldz;
    const int* out_rows;   // EPI_SCATTER: output row of each of this expert's rows; C is then the whole output
};

// v: four accumulators of row r, columns n..n+3 (all in range).  Returns this
// thread's contribution to <gelu(Z_r), acc_r> for EPI_DGELU, else 0.
template <typename T, int EPI>
__device__ __forceinline__ float epilogue4(const EpiCtx<T>& c, int r, int n, const float* v) {
    if constexpr (EPI == EPI_STORE) {
        Vec4<T>::store(c.C + (size_t)r * c.ldc + n, v);
        return 0.0f;
    } else if constexpr (EPI == EPI_GELU) {
        float z[4], a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { z[i] = Vec4<T>::round(v[i]); a[i] = gelu_f(z[i]); }
        if (c.Z) Vec4<T>::store(c.Z + (size_t)r * c.ldz + n, z);
        Vec4<T>::store(c.C + (size_t)r * c.ldc + n, a);
        return 0.0f;
    } else if constexpr (EPI == EPI_DGELU) {
        float z[4], dz[4], a[4];
        Vec4<T>::load(c.Z + (size_t)r * c.ldz + n, z);
        const float w = c.w[r];
        float dot = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float g, dg;
            gelu_both_f(z[i], &g, &dg);
            dot = fmaf(g, v[i], dot);
            a[i] = w * g;
            dz[i] = w * v[i] * dg;
        }
        Vec4<T>::store(c.C + (size_t)r * c.ldc + n, dz);
        Vec4<T>::store(c.Z + (size_t)r * c.ldz + n, a);
        return dot;
    } else if constexpr (EPI == EPI_SCATTER) {
        const float w = c.w[r];
        const float o[4] = {w * v[0], w * v[1], w * v[2], w * v[3]};
        Vec4<T>::store(c.C + (size_t)c.out_rows[r] * c.ldc + n, o);
        return 0.0f;
    } else if constexpr (EPI == EPI_STORE_F32) {
        *reinterpret_cast<float4*>(c.Cf + (size_t)r * c.ldc + n) = make_float4(v[0], v[1], v[2], v[3]);
        return 0.0f;
    } else {
        float* p = c.Cf + (size_t)r * c.ldc + n;
        float4 o = *reinterpret_cast<float4*>(p);
        o.x += v[0]; o.y += v[1]; o.z += v[2]; o.w += v[3];
        *reinterpret_cast<float4*>(p) = o;
        return 0.0f;
    }
}

}  // namespace moe
