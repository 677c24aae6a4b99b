// bf16 grouped GEMM on the CDNA4 matrix cores for the expert FFN: the two linear
// layers of every local expert (Section II-B2) and their four backward GEMMs
// (Table II counts 2 forward and 4 backward GEMM units per partition, 5 with
// recomputation).  Float accumulation in v_mfma_f32_32x32x16_bf16.
//
// One workgroup (4 wavefronts, 2x2) computes a BM x BN tile of one expert; each
// wavefront owns (BM/2) x (BN/2) as 32x32 MFMA tiles.  Both operands are staged
// in LDS with K contiguous (64 K-elements = one 128-byte row per tile row) and a
// 16-byte-chunk XOR swizzle, so fragment reads are conflict-free ds_read_b128.
// Operands whose K index is the slow one in memory (B of NN, both of TN) are
// transposed in registers (8x8 blocks, v_perm_b32) on their way into LDS, which
// keeps one MFMA loop for all three layouts.  LDS is double buffered and the
// global loads for tile k+2 are in flight while tile k is multiplied.
// Workgroup ids are remapped so that the workgroups resident on one XCD share
// A/B panels through that XCD's L2.
#include "common.h"
#include "epilogue.h"

namespace moe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int G_BK = 64;
constexpr int G_ROWB = G_BK * 2;          // bytes of one LDS tile row

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

// ---- tile shape ------------------------------------------------------------------
// BM x BN output tile, WAVES_M x WAVES_N wavefronts, STAGES LDS buffers (2: the
// next tile is written while this one is multiplied; 1: write after a barrier,
// with a second workgroup on the CU covering the gap), OCC wavefronts per SIMD.
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int STAGES_, int OCC_>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int STAGES = STAGES_, OCC = OCC_;
    static constexpr int THREADS = 64 * WAVES_M * WAVES_N;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int STAGE_BYTES = (BM + BN) * G_ROWB;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
};

// ---- global -> registers -> LDS -----------------------------------------------------
// Global reads go through buffer descriptors that cover exactly the valid rows
// of the operand, so out-of-range rows read as zero in hardware and the loop has
// no branches; a K tail or a column beyond the matrix is turned into an
// out-of-range offset by a select.
typedef int v4i __attribute__((ext_vector_type(4)));
constexpr unsigned OOB_OFFSET = 0x80000000u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t r, unsigned off) {
    return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0));
}

// Direct: operand rows are K-contiguous.  R rows x 64 K = R*8 chunks of 16 bytes.
// The descriptor starts at the tile's first row and ends after its last valid row.
template <int R, int THREADS>
struct DirectTile {
    static constexpr int N = R * 8 / THREADS;
    static_assert(R * 8 % THREADS == 0, "tile rows must divide over the threads");
    uint4 v[N];
    __amdgpu_buffer_rsrc_t rsrc;
    int ld;
    __device__ __forceinline__ void init(const bf16_t* P, int ld_, int row0, int row_limit, int /*col0*/, int /*col_limit*/, int K) {
        const int valid = min(R, row_limit - row0);
        ld = ld_;
        rsrc = make_rsrc(P + (size_t)row0 * ld_, (unsigned)(((size_t)(valid - 1) * ld_ + K) * 2));
    }
    __device__ __forceinline__ void load(int k0, int K, int tid) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int q = tid + i * THREADS;
            const int row = q >> 3, c = q & 7;
            const int gk = k0 + c * 8;
            const unsigned off = (unsigned)(row * ld + gk) * 2u;
            v[i] = buffer_load16(rsrc, gk < K ? off : OOB_OFFSET);
        }
    }
    __device__ __forceinline__ void store(char* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int q = tid + i * THREADS;
            const int row = q >> 3, c = q & 7;
            *reinterpret_cast<uint4*>(lds + row * G_ROWB + ((c ^ swz(row)) << 4)) = v[i];
        }
    }
};

// Transposed: operand is [k][n] with n contiguous.  A thread takes a KR(k) x 8(n)
// block (KR = 8 or 4), transposes it in registers and writes eight K-contiguous
// pieces of KR elements.  The descriptor starts at the tile's first column and
// ends after the last valid K row.
template <int R, int THREADS>
struct TransTile {
    static constexpr int NG = R / 8;                  // n-groups per tile
    static constexpr int KR = (THREADS >= 16 * NG) ? 4 : 8;
    static_assert(THREADS >= 64 * NG / KR, "not enough threads for the tile");
    static constexpr int UNITS = NG * (64 / KR);      // threads that carry a block
    uint4 v[KR];
    __amdgpu_buffer_rsrc_t rsrc;
    int ld, n_valid;
    __device__ __forceinline__ void init(const bf16_t* P, int ld_, int n0, int n_limit, int /*k0*/, int /*unused*/, int K) {
        ld = ld_;
        n_valid = n_limit - n0;
        rsrc = make_rsrc(P + n0, (unsigned)(((size_t)(K - 1) * ld_ + n_valid) * 2));
    }
    __device__ __forceinline__ void load(int k0, int /*K*/, int tid) {
        const int ng = tid % NG, kg = tid / NG;
        const bool on = tid < UNITS && ng * 8 < n_valid;
#pragma unroll
        for (int j = 0; j < KR; ++j) {
            const int gk = k0 + kg * KR + j;
            const unsigned off = (unsigned)(gk * ld + ng * 8) * 2u;
            v[j] = buffer_load16(rsrc, on ? off : OOB_OFFSET);
        }
    }
    __device__ __forceinline__ void store(char* lds, int tid) const {
        if (tid >= UNITS) return;
        const int ng = tid % NG, kg = tid / NG;
        const unsigned* w = reinterpret_cast<const unsigned*>(v);   // w[j*4 + q]
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int q = i >> 1;
            const unsigned sel = (i & 1) ? 0x07060302u : 0x05040100u;
            const int row = ng * 8 + i;
            if constexpr (KR == 8) {
                uint4 o;
                o.x = __builtin_amdgcn_perm(w[1 * 4 + q], w[0 * 4 + q], sel);
                o.y = __builtin_amdgcn_perm(w[3 * 4 + q], w[2 * 4 + q], sel);
                o.z = __builtin_amdgcn_perm(w[5 * 4 + q], w[4 * 4 + q], sel);
                o.w = __builtin_amdgcn_perm(w[7 * 4 + q], w[6 * 4 + q], sel);
                *reinterpret_cast<uint4*>(lds + row * G_ROWB + ((kg ^ swz(row)) << 4)) = o;
            } else {
                uint2 o;
                o.x = __builtin_amdgcn_perm(w[1 * 4 + q], w[0 * 4 + q], sel);
                o.y = __builtin_amdgcn_perm(w[3 * 4 + q], w[2 * 4 + q], sel);
                *reinterpret_cast<uint2*>(lds + row * G_ROWB + (((kg >> 1) ^ swz(row)) << 4) + ((kg & 1) << 3)) = o;
            }
        }
    }
};

template <int LAY, int R, int T> struct ATile { typedef DirectTile<R, T> type; };
template <int R, int T> struct ATile<GEMM_TN, R, T> { typedef TransTile<R, T> type; };
template <int LAY, int R, int T> struct BTile { typedef TransTile<R, T> type; };
template <int R, int T> struct BTile<GEMM_NT, R, T> { typedef DirectTile<R, T> type; };

template <int LAY, int EPI, typename C>
__global__ __launch_bounds__(C::THREADS) __attribute__((amdgpu_waves_per_eu(C::OCC, C::OCC)))
void gemm_bf16_kernel(GemmArgs g, int tiles_m, int tiles_n, int nblocks) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int BM = C::BM, BN = C::BN, WM = C::WM, WN = C::WN, TM = C::TM, TNN = C::TN;
    constexpr int STAGE = C::STAGE_BYTES;

    // ---- workgroup -> (expert, tile) with XCD-aware order ------------------------
    // Hardware deals consecutive workgroup ids round-robin to the 8 XCDs; give each
    // XCD a contiguous run of tiles, and walk tiles in groups of 4 tile-rows so the
    // workgroups running together on an XCD reuse A and B panels in its L2.
    int lin;
    {
        const int b = blockIdx.x;
        const int per = nblocks >> 3;                   // nblocks is a multiple of 8
        lin = (b & 7) * per + (b >> 3);
    }
    const int per_e = tiles_m * tiles_n;
    const int e = lin / per_e;
    if (e >= g.E) return;
    int tm, tn;
    {
        const int rem = lin - e * per_e;
        constexpr int GM = 4;
        const int grp = rem / (GM * tiles_n);
        const int first = grp * GM;
        const int gsz = min(GM, tiles_m - first);
        const int in = rem - grp * GM * tiles_n;
        tm = first + in % gsz;
        tn = in / gsz;
    }
    const int rows = g.counts[e];
    int Mdim, Kdim;
    if (LAY == GEMM_TN) { Mdim = g.Mo; Kdim = rows; } else { Mdim = rows; Kdim = g.K; }
    const int m0 = tm * BM, n0 = tn * BN;
    if (m0 >= Mdim || Kdim <= 0) return;

    const bf16_t* A = (const bf16_t*)g.A + (size_t)e * g.a_estride;
    const bf16_t* B = (const bf16_t*)g.B + (size_t)e * g.b_estride;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int wm = wid / C::WAVES_N, wn = wid % C::WAVES_N;

    typename ATile<LAY, BM, C::THREADS>::type ta;
    typename BTile<LAY, BN, C::THREADS>::type tb;
    const int KT = (Kdim + G_BK - 1) / G_BK;

    ta.init(A, g.lda, m0, Mdim, 0, 0, Kdim);
    tb.init(B, g.ldb, n0, g.N, 0, 0, Kdim);
    auto load_tiles = [&](int kt) {
        ta.load(kt * G_BK, Kdim, tid);
        tb.load(kt * G_BK, Kdim, tid);
    };
    auto store_tiles = [&](int stage) {
        ta.store(smem + stage * STAGE, tid);
        tb.store(smem + stage * STAGE + BM * G_ROWB, tid);
    };

    floatx16 acc[TM][TNN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TNN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // fragment addressing: lane reads tile row (lane & 31), logical chunk 2*kk + (lane >> 5)
    int a_off[TM], a_sw[TM], b_off[TNN], b_sw[TNN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = wm * WM + i * 32 + (lane & 31);
        a_off[i] = row * G_ROWB;
        a_sw[i] = swz(row);
    }
#pragma unroll
    for (int j = 0; j < TNN; ++j) {
        const int row = wn * WN + j * 32 + (lane & 31);
        b_off[j] = BM * G_ROWB + row * G_ROWB;
        b_sw[j] = swz(row);
    }
    const int khalf = lane >> 5;

    auto compute = [&](const char* base) {
#pragma unroll
        for (int kk = 0; kk < G_BK / 16; ++kk) {
            bf16x8 af[TM], bfr[TNN];
            const int c = kk * 2 + khalf;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(base + a_off[i] + ((c ^ a_sw[i]) << 4));
#pragma unroll
            for (int j = 0; j < TNN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8*>(base + b_off[j] + ((c ^ b_sw[j]) << 4));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TNN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
        }
    };

    if constexpr (C::STAGES == 2) {
        load_tiles(0);
        store_tiles(0);
        load_tiles(1);                       // tiles past the end read as zeros
        __syncthreads();
        for (int kt = 0; kt < KT; ++kt) {
            const int cur = kt & 1;
            // One straight-line block per iteration: write tile kt+1 into the other
            // LDS buffer, start the global reads of tile kt+2, multiply tile kt.
            store_tiles(cur ^ 1);
            load_tiles(kt + 2);
            compute(smem + cur * STAGE);
            // Issue order for the block: the first fragments, then the matrix
            // instructions with LDS reads, LDS writes and global reads between them,
            // so the matrix pipe stays busy while the memory pipes work.
            constexpr int NMFMA = TM * TNN * (G_BK / 16);
            constexpr int NDSR = (TM + TNN) * (G_BK / 16);
            constexpr int FIRST = TM + TNN;
            __builtin_amdgcn_sched_group_barrier(0x100, FIRST, 0);
#pragma unroll
            for (int i = 0; i < NMFMA; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (i < NDSR - FIRST) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if (i % 2 == 0) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                if (i % 2 == 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            __syncthreads();
        }
    } else {
        load_tiles(0);
        for (int kt = 0; kt < KT; ++kt) {
            store_tiles(0);
            __syncthreads();
            if (kt + 1 < KT) load_tiles(kt + 1);
            compute(smem);
            __syncthreads();
        }
    }

    // ---- epilogue: lane holds row m = (lane & 31), columns 8*g4 + 4*(lane>>5) + 0..3 ----
    // The lane id is passed through an empty asm so that none of the epilogue's
    // address arithmetic is hoisted above the main loop, where registers are scarce.
    int elane = lane;
    asm volatile("" : "+v"(elane));
    const int erow = elane & 31, ehalf = elane >> 5;
    EpiCtx<bf16_t> c;
    c.ldc = g.ldc; c.ldz = g.ldz;
    c.C = (bf16_t*)g.C + (size_t)e * g.c_estride;
    c.Cf = (float*)g.C + (size_t)e * g.c_estride;
    c.Z = g.Z ? (bf16_t*)g.Z + (size_t)e * g.Cp * g.ldz : nullptr;
    c.w = g.slot_w ? g.slot_w + (size_t)e * g.Cp : nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * WM + i * 32 + erow;
        float dot = 0.0f;
#pragma unroll
        for (int j = 0; j < TNN; ++j) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int n = n0 + wn * WN + j * 32 + g4 * 8 + ehalf * 4;
                float v[4] = {acc[i][j][g4 * 4 + 0], acc[i][j][g4 * 4 + 1], acc[i][j][g4 * 4 + 2], acc[i][j][g4 * 4 + 3]};
                if (m < Mdim && n < g.N) dot += epilogue4<bf16_t, EPI>(c, m, n, v);
            }
            __builtin_amdgcn_sched_barrier(0);   // keep one 32x32 tile's loads and stores together
        }
        if (EPI == EPI_DGELU && g.dw_part) {
            dot += __shfl_xor(dot, 32, 64);
            if (elane < 32 && m < Mdim)
                g.dw_part[((size_t)e * g.Cp + m) * g.dw_parts + tn * C::WAVES_N + wn] = dot;
        }
    }
}

// Tile shape in use.  MOE_GEMM_CFG selects it at build time for experiments.
#ifndef MOE_GEMM_CFG
#define MOE_GEMM_CFG 2
#endif
#if MOE_GEMM_CFG == 0
typedef TileCfg<256, 256, 2, 2, 2, 1> Cfg;     // 4 waves of 128x128, double-buffered LDS
#elif MOE_GEMM_CFG == 1
typedef TileCfg<128, 256, 2, 2, 1, 2> Cfg;     // 4 waves of 64x128, two workgroups per CU
#elif MOE_GEMM_CFG == 2
typedef TileCfg<256, 256, 2, 4, 2, 2> Cfg;     // 8 waves of 128x64, double-buffered LDS
#elif MOE_GEMM_CFG == 3
typedef TileCfg<256, 128, 2, 2, 1, 2> Cfg;     // 4 waves of 128x64, two workgroups per CU
#endif

int gemm_bf16_dw_parts(int H) { return ((H + Cfg::BN - 1) / Cfg::BN) * Cfg::WAVES_N; }

template <int LAY, int EPI, typename C>
static moe_status launch_one(const GemmArgs& a, hipStream_t s) {
    const int Mmax = (LAY == GEMM_TN) ? a.Mo : a.Cp;
    const int tiles_m = (Mmax + C::BM - 1) / C::BM, tiles_n = (a.N + C::BN - 1) / C::BN;
    int nblocks = a.E * tiles_m * tiles_n;
    nblocks = (nblocks + 7) / 8 * 8;
    constexpr int lds = C::LDS_BYTES;
    auto kern = gemm_bf16_kernel<LAY, EPI, C>;
    static bool attr_done = false;
    if (!attr_done) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_done = true;
    }
    {
        ProfScope ps(gemm_prof_kind(LAY, EPI), s);
        hipLaunchKernelGGL(kern, dim3(nblocks), dim3(C::THREADS), lds, s, a, tiles_m, tiles_n, nblocks);
    }
    count_launch(LC_GEMM);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

template <int LAY>
static moe_status launch_lay(GemmEpilogue epi, const GemmArgs& a, hipStream_t s) {
    switch (epi) {
        case EPI_STORE: return launch_one<LAY, EPI_STORE, Cfg>(a, s);
        case EPI_GELU: return launch_one<LAY, EPI_GELU, Cfg>(a, s);
        case EPI_DGELU: return launch_one<LAY, EPI_DGELU, Cfg>(a, s);
        case EPI_ACCUM_F32: return launch_one<LAY, EPI_ACCUM_F32, Cfg>(a, s);
    }
    return MOE_ERR_UNSUPPORTED;
}

moe_status gemm_bf16(GemmLayout lay, GemmEpilogue epi, const GemmArgs& a, hipStream_t s) {
    if (a.dw_part && a.dw_parts != gemm_bf16_dw_parts(a.N)) return MOE_ERR_SHAPE;
    if (lay == GEMM_NN) return launch_lay<GEMM_NN>(epi, a, s);
    if (lay == GEMM_NT) return launch_lay<GEMM_NT>(epi, a, s);
    return launch_lay<GEMM_TN>(epi, a, s);
}

}  // namespace moe
