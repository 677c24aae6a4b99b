// bf16 grouped GEMM on the CDNA4 matrix cores for the expert FFN: the two linear
// layers of every local expert (Section II-B2) and their four backward GEMMs
// (Table II counts 2 forward and 4 backward GEMM units per partition, 5 with
// recomputation).  Float accumulation in v_mfma_f32_32x32x16_bf16.
//
// One workgroup computes a BM x BN tile of one expert with WAVES_M x WAVES_N
// wavefronts, each owning (BM/WAVES_M) x (BN/WAVES_N) as 32x32 MFMA tiles.
//
// Operand tiles (64 K-elements deep) travel global -> LDS with
// buffer_load_dwordx4 ... lds: no staging registers, no LDS-write instructions,
// and rows beyond the valid range read as zeros in hardware (the buffer
// descriptor ends after the last valid row), so the main loop has no branches.
// Each lane of such a load lands at LDS base + 16*lane, so the LDS layout is
// chosen by choosing which 16 global bytes each lane fetches:
//   * an operand whose rows are K-contiguous in memory ("KC": A of NN/NT, B of
//     NT) is kept as [row][64 k] with a 16-byte-chunk XOR swizzle and read with
//     ds_read_b128 - conflict-free both ways;
//   * an operand stored [k][n] with n contiguous ("NC": B of NN, both of TN) is
//     kept as it is, rows rotated by 64 bytes per k mod 4, and read with
//     ds_read_b64_tr_b16, which hands each lane four consecutive k of one n.
// LDS is a ring of NS stages of BK K-elements each; the loads of the next NS-1
// tiles are in flight while one tile is multiplied (a CU draws about 64 KB per
// microsecond at speed and a miss in L2 takes longer than one tile's arithmetic,
// so the depth of the ring, not the hit rate, decides whether the matrix pipe
// waits).  One s_barrier per tile.
#include "common.h"
#include "epilogue.h"

namespace moe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4s lds_v4s;

constexpr unsigned OOB_OFFSET = 0x80000000u;

// Buffer descriptor (base, stride 0, size in bytes, raw 32-bit format) kept in SGPRs.
typedef int v4i __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v4i make_rsrc(const void* p, unsigned bytes) {
    // wave-uniform by construction; readfirstlane makes that visible to the compiler, which must
    // hand the descriptor to the assembly statements below in scalar registers
    const unsigned long long a = (unsigned long long)p;
    v4i d = {__builtin_amdgcn_readfirstlane((int)(unsigned)a), __builtin_amdgcn_readfirstlane((int)((a >> 32) & 0xffffu)),
             __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000};
    return d;
}
// 16 bytes per lane from the buffer straight into LDS at lds_off + 16*lane (lds_off is a
// wave-uniform LDS byte address).  Written as assembly so that the compiler's
// wait-count bookkeeping does not see an LDS store in flight: it would otherwise make
// every transposing LDS read wait for all of them (vmcnt(0)), which serialises the
// ring.  The kernel waits with explicit s_waitcnt vmcnt(N) before each barrier instead.
__device__ __forceinline__ void load_to_lds(v4i rsrc, unsigned lds_off, unsigned voff) {
    // m0 carries the LDS address of the load and nothing else in these kernels (no LDS-direct reads, no
    // relative register indexing, no message sends), so it is not saved and restored around the load
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "s_nop 0\n\t"
                 "buffer_load_dwordx4 %1, %2, 0 offen lds"
                 : : "s"(lds_off), "v"(voff), "s"(rsrc) : "memory");
}
__device__ __forceinline__ unsigned lds_address(const char* p) {
    return (unsigned)(unsigned long long)(__attribute__((address_space(3))) const char*)p;
}

// ---- tile shape ------------------------------------------------------------------
// Two main loops, both hand-scheduled:
//   LOOP_PIPE32 ring of five stages of 32 k;
//   LOOP_W64    64-k steps with one ring per operand: a K-contiguous operand travels as whole
//               128-byte lines (units of 64 k), the other one in tiles of 32 k.
enum { LOOP_PIPE32 = 1, LOOP_W64 = 2 };
template <int BM_, int BN_, int BK_, int NS_, int WAVES_M_, int WAVES_N_, int OCC_, int LOOP_>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, NS = NS_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int OCC = OCC_, LOOP = LOOP_;
    static constexpr int WAVES = WAVES_M * WAVES_N;
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    static constexpr int LDS_BYTES = LOOP == LOOP_W64 ? 160 * 1024 : NS * STAGE_BYTES;
    static constexpr bool PIPE = LOOP == LOOP_PIPE32;
    // columns of a wave's block that pass through the staging region at a time, and where that region starts
    static constexpr int CW = LOOP == LOOP_W64 ? 64 : WN;
    static constexpr int STAGING_OFF = LOOP == LOOP_W64 ? 64 * 1024 : 0;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS ring exceeds the CU's 160 KB");
    static_assert(BK == 32 || BK == 64, "tile depth");
    static_assert(LOOP != LOOP_PIPE32 || (BK == 32 && NS == 5), "the hand-scheduled ring is five stages of 32 k");
    static_assert(LOOP != LOOP_W64 || (BM == 256 && BN == 256 && BK == 64 && WAVES_M == 2 && WAVES_N == 2 && OCC == 1),
                  "the two-ring loop is written for four waves of 128 x 128");
};

// ---- K-contiguous operand tile: R rows x BK k ---------------------------------------
// A row is CPR = BK/8 chunks of 16 bytes.  LDS byte of (row, chunk c) =
// row*ROWB + ((c ^ sw(row)) << 4), with sw chosen so that the 16 rows one
// ds_read_b128 quarter-wave touches fall into 16 different 16-byte bank groups
// (64 banks of 4 bytes).  One wave instruction fills 1024 bytes = RPI rows:
// lane l -> row RPI*q + l/CPR, physical chunk l%CPR.
template <int R, int WAVES, int BK>
struct KCTile {
    static constexpr int ROWB = BK * 2;
    static constexpr int CPR = BK / 8;
    static constexpr int RPI = 1024 / ROWB;
    static constexpr int NI = R / RPI / WAVES;         // load instructions per wave per tile
    static constexpr int BYTES = R * ROWB;
    static_assert(R % (RPI * WAVES) == 0 && NI >= 1, "rows must divide over the wavefronts");
    static __device__ __forceinline__ int sw(int row) {
        return CPR == 8 ? ((row ^ (row >> 3)) & 7) : ((row >> 2) & 3);
    }
    v4i rsrc;
    unsigned voff[NI];       // byte offset of this lane's chunk at k0 = 0
    int kc[NI];              // first k of this lane's chunk
    int K;
    // P: operand base of this expert; rows [row0, row_limit) x [0, K) are valid
    __device__ __forceinline__ void init(const bf16_t* P, int ld, int row0, int row_limit, int K_, int lane, int wid) {
        const int valid = min(R, row_limit - row0);
        K = K_;
        rsrc = make_rsrc(P + (size_t)row0 * ld, K_ > 0 ? (unsigned)(((size_t)(valid - 1) * ld + K_) * 2) : 0u);
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int q = wid * NI + j;
            const int row = q * RPI + lane / CPR;
            const int c = (lane % CPR) ^ sw(row);
            kc[j] = c * 8;
            voff[j] = (unsigned)(row * ld + c * 8) * 2u;
        }
    }
    // The same tile with its rows gathered: row r of the tile is row rows[row0 + r] of the matrix P
    // (of n_rows rows); rows at or beyond row_limit read as zeros.  Only the lane offsets differ,
    // so the main loop is the same.
    __device__ __forceinline__ void init_gather(const bf16_t* P, int ld, const int* rows, int row0, int row_limit,
                                                int n_rows, int K_, int lane, int wid) {
        K = K_;
        rsrc = make_rsrc(P, K_ > 0 ? (unsigned)(((size_t)(n_rows - 1) * ld + K_) * 2) : 0u);
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int q = wid * NI + j;
            const int row = q * RPI + lane / CPR;
            const int c = (lane % CPR) ^ sw(row);
            kc[j] = c * 8;
            const int src = row0 + row < row_limit ? rows[row0 + row] : -1;
            voff[j] = src >= 0 ? (unsigned)(src * ld + c * 8) * 2u : OOB_OFFSET;
        }
    }
    __device__ __forceinline__ void load_one(char* tile, int k0, int wid, int j) const {
        const int q = wid * NI + j;
        unsigned off = voff[j] + (unsigned)k0 * 2u;
        // only a tile that reaches beyond K (a wave-uniform condition) has lanes to switch off
        if (k0 + BK > K) off = (k0 + kc[j] < K) ? off : OOB_OFFSET;
        load_to_lds(rsrc, lds_address(tile) + q * 1024, off);
    }
    __device__ __forceinline__ void load(char* tile, int k0, int wid) const {
#pragma unroll
        for (int j = 0; j < NI; ++j) load_one(tile, k0, wid, j);
    }
    // fragment of the 32 rows starting at rb: lane reads row rb + lane%32, k = 16*kk + 8*(lane/32) .. +7
    struct Frag {
        int addr;    // byte address inside the tile for kk = 0
        __device__ __forceinline__ void init(int rb, int lane) {
            const int row = rb + (lane & 31);
            addr = row * ROWB + (((lane >> 5) ^ sw(row)) << 4);
        }
        __device__ __forceinline__ bf16x8 read(const char* tile, int kk) const {
            return *reinterpret_cast<const bf16x8*>(tile + (addr ^ (kk << 5)));
        }
    };
};

// ---- N-contiguous operand tile: BK k rows x R n --------------------------------------
// LDS byte of (k, 16-byte unit u) = k*PITCH + (((u + 4*(k&3)) % UPR) << 4): the four k rows
// that one transposing read touches fall into different banks (64 banks of 4 bytes).
// One wave instruction fills 1024 bytes = RPI rows: lane l -> row RPI*q + l/UPR, unit l%UPR.
template <int R, int WAVES, int BK>
struct NCTile {
    static constexpr int PITCH = R * 2;                // bytes per k row
    static constexpr int UPR = R / 8;                  // 16-byte units per row
    static constexpr int RPI = 1024 / PITCH;           // rows per wave instruction
    static constexpr int NI = BK / RPI / WAVES;
    static constexpr int BYTES = BK * PITCH;
    static_assert(BK % (RPI * WAVES) == 0 && NI >= 1, "rows must divide over the wavefronts");
    v4i rsrc;
    unsigned voff[NI];
    unsigned kstep;          // bytes per k row in memory
    // descriptor of rows [0, K) x columns [0, n_valid) of the matrix at P
    static __device__ __forceinline__ v4i rsrc_of(const bf16_t* P, int ld, int n_valid, int K) {
        return make_rsrc(P, K > 0 ? (unsigned)(((size_t)(K - 1) * ld + n_valid) * 2) : 0u);
    }
    // P: operand base of this expert ([k][n], n contiguous); rows [0, K) x columns [n0, n_limit) valid
    __device__ __forceinline__ void init(const bf16_t* P, int ld, int n0, int n_limit, int K, int lane, int wid) {
        const int n_valid = n_limit - n0;
        kstep = (unsigned)ld * 2u;
        rsrc = rsrc_of(P + n0, ld, n_valid, K);
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int q = wid * NI + j;
            const int row = q * RPI + lane / UPR;
            const int u = ((lane % UPR) - 4 * (row & 3) + UPR) % UPR;
            voff[j] = (u * 8 < n_valid) ? (unsigned)(row * ld + u * 8) * 2u : OOB_OFFSET;
        }
    }
    __device__ __forceinline__ void load_one(char* tile, int k0, int wid, int j) const {
        const int q = wid * NI + j;
        load_to_lds(rsrc, lds_address(tile) + q * 1024, voff[j] + (unsigned)k0 * kstep);
    }
    __device__ __forceinline__ void load(char* tile, int k0, int wid) const {
#pragma unroll
        for (int j = 0; j < NI; ++j) load_one(tile, k0, wid, j);
    }
    // fragment of the 32 columns starting at nb: two transposing reads give the lane
    // n = nb + lane%32, k = 16*kk + 8*(lane/32) .. +7.  In a 16-lane group lane a points at
    // row a/4, columns 4*(a%4)..+3; the hardware returns to lane i four k of column i.
    struct Frag {
        int addr;
        __device__ __forceinline__ void init(int nb, int lane) {
            const int g = lane >> 4, a = lane & 15;
            const int k_in = 8 * (g >> 1) + (a >> 2);
            const int n = nb + 16 * (g & 1) + 4 * (a & 3);
            addr = k_in * PITCH + ((((n >> 3) + 4 * (k_in & 3)) % UPR) << 4) + ((n & 7) << 1);
        }
        __device__ __forceinline__ bf16x8 read(const char* tile, int kk) const {
            const char* p = tile + addr + kk * 16 * PITCH;
            v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)p);
            v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)(p + 4 * PITCH));
            typedef short v8s __attribute__((ext_vector_type(8)));
            v8s both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, both);
        }
    };
};

template <int LAY, int R, int W, int BK> struct ATile { typedef KCTile<R, W, BK> type; };
template <int R, int W, int BK> struct ATile<GEMM_TN, R, W, BK> { typedef NCTile<R, W, BK> type; };
template <int LAY, int R, int W, int BK> struct BTile { typedef NCTile<R, W, BK> type; };
template <int R, int W, int BK> struct BTile<GEMM_NT, R, W, BK> { typedef KCTile<R, W, BK> type; };

struct Unit8 {
    static __device__ __forceinline__ void to_float(const uint4& u, float* o) {
        const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = __uint_as_float(w[i] << 16);
            o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

// s_waitcnt vmcnt(N) only (N <= 63), with a compiler-level memory fence
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
    asm volatile("" ::: "memory");
}

// The matrix instruction as volatile assembly with a memory clobber: the compiler keeps
// such statements, the LDS reads and the loads into LDS in the order they are written,
// which is what the hand-scheduled loop below relies on (it still allocates registers
// and inserts the s_waitcnt lgkmcnt for LDS reads it issued itself).
template <bool ACC_IN_AGPR>
__device__ __forceinline__ void mfma_pinned(floatx16& acc, const bf16x8& a, const bf16x8& b) {
    // accumulators live in the AGPR half of the register file when a wave owns 512 registers,
    // in ordinary VGPRs when two waves share a SIMD
    if constexpr (ACC_IN_AGPR)
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b) : "memory");
    else
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b) : "memory");
}

// TN only: the reduction dimension may run over the rows of several partitions (up to MAX_KSEGS row
// ranges, one per partition buffer); tiles of 32 k never straddle two ranges.  KCursor says which range
// the tile that is being requested lies in and where.
constexpr int MAX_KSEGS = 8;
struct TileCoord { int e, tn, m0, n0, Mdim, Kdim, KT; };
struct KCursor { int seg, jl, tiles; };

// Persistent workgroups: the grid has one workgroup per CU, and workgroup b works through
// the tiles b, b + grid, b + 2 grid, ...  While a tile's epilogue runs (it needs only the
// staging part of LDS and no matrix instructions), the first operand tiles of the next
// tile are already on their way into the rest of the ring, so neither the launch of a new
// workgroup nor the first trip to memory stands between two main loops.
template <int LAY, int EPI, typename C>
__global__ __launch_bounds__(C::THREADS) __attribute__((amdgpu_waves_per_eu(C::OCC, C::OCC)))
void gemm_bf16_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int BM = C::BM, BN = C::BN, WM = C::WM, WN = C::WN, TM = C::TM, TNN = C::TN;
    constexpr int STAGE = C::STAGE_BYTES, BK = C::BK, NS = C::NS;
    constexpr bool W64 = C::LOOP == LOOP_W64;
    // Depth of one load unit of each operand.  In the two-ring loop a K-contiguous row operand (A of
    // NN) or the K-contiguous weights (B of NT) travel 64 k at a time, so that every request is a whole
    // 128-byte line; the other operand keeps tiles of 32 k.
    constexpr bool A_WIDE = W64 && LAY == GEMM_NN;
    constexpr int AK = W64 ? (A_WIDE ? 64 : 32) : BK, BKB = W64 ? (A_WIDE ? 32 : 64) : BK;
    static_assert(!W64 || LAY != GEMM_TN, "both operands of the weight-gradient GEMM are N-contiguous: five stages of 32 k serve them");
    constexpr int A_BYTES = BM * BK * 2;
    // The epilogue stages accumulators in the first SB stages of the ring; a tile's ring
    // starts at stage SB, so that its first operand tiles can arrive during the epilogue
    // of the tile before.  (Two-ring loop: in the third unit of the wide ring.)
    constexpr int SB = 2;
    constexpr int CW = C::CW;
    static_assert(W64 || C::WAVES * 32 * CW * 4 <= SB * STAGE, "staging does not fit below the ring's first stage");
    static_assert(!W64 || C::WAVES * 32 * CW * 4 <= 32 * 1024, "staging does not fit one unit of the wide ring");
    // two-ring LDS map: three units of 64 k x 256 rows, then four tiles of 32 k x 256 rows
    constexpr int WIDE_UNIT = 32 * 1024, NARROW_TILE = 16 * 1024, NARROW_OFF = 3 * WIDE_UNIT;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wid / C::WAVES_N, wn = wid % C::WAVES_N;
    typedef typename ATile<LAY, BM, C::WAVES, AK>::type AT;
    typedef typename BTile<LAY, BN, C::WAVES, BKB>::type BT;
    constexpr int LPW = AT::NI + BT::NI;         // loads per wave per tile
    typename AT::Frag fa[TM];
    typename BT::Frag fb[TNN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i].init(wm * WM + i * 32, lane);
#pragma unroll
    for (int j = 0; j < TNN; ++j) fb[j].init(wn * WN + j * 32, lane);

    // ---- tile number -> (expert, tile) -----------------------------------------------
    // Only tiles that exist are numbered: an expert with fewer rows than the capacity has fewer
    // tile rows (NN, NT), an expert without rows has no tiles at all (TN), so that the workgroups,
    // which take the numbers b, b + grid, ..., all get the same amount of work whatever the spread
    // of the counts.  Lane l of every wavefront holds the tiles of expert l (E <= 64); an inclusive
    // scan over the lanes gives the number at which each expert ends.
    int lane_tm = 0;                     // tile rows of expert `lane` (none: the expert has no tiles)
    if (lane < g.E) {
        int rows = 0;
        const int segs = (LAY == GEMM_TN && g.k_segs > 1) ? g.k_segs : 1;
        for (int sg = 0; sg < segs; ++sg) rows += g.counts[sg * g.E + lane];
        if (LAY == GEMM_TN) lane_tm = (rows > 0 || EPI == EPI_STORE_F32) ? tiles_m : 0;   // a plain store still writes zeros
        else lane_tm = min(tiles_m, (rows + BM - 1) / BM);
    }
    int lane_end = lane_tm * tiles_n;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(lane_end, off, 64);
        if (lane >= off) lane_end += o;
    }
    const int nblocks = __builtin_amdgcn_readlane(lane_end, 63);
    // Tiles are numbered expert by expert, in groups of 4 tile-rows walked column by
    // column, so 32 consecutive numbers form a 4 x 8 block that shares 4 A panels and 8
    // B panels.  Hardware deals consecutive workgroup ids round-robin to the 8 XCDs (each
    // with its own L2), and the grid is a multiple of 8, so tile number b always runs on
    // XCD b mod 8; within every run of 256 numbers, XCD x is given the x-th block of 32
    // consecutive tiles, so each L2 serves a compact block while all eight XCDs stay on
    // the same expert(s) and share its weights through the memory-side cache.  (Against
    // plain order this halves what the L2s fetch; against giving each XCD its own experts
    // it is 3-5 % faster.)  A last partial run keeps plain order.
    auto decode = [&](int b, TileCoord& t) -> bool {
        const int lin = (b < (nblocks & ~255)) ? (b & ~255) + (b & 7) * 32 + ((b >> 3) & 31) : b;
        // the expert: as many experts end at or before lin as lanes say so (the ends never decrease)
        const int e = __builtin_popcountll(__builtin_amdgcn_ballot_w64(lane_end <= lin));
        if (e >= g.E) return false;
        const int tm_e = __builtin_amdgcn_readlane(lane_tm, e);      // tile rows of this expert
        const int rem = lin - (__builtin_amdgcn_readlane(lane_end, e) - tm_e * tiles_n);
        constexpr int GM = 4;
        const int grp = rem / (GM * tiles_n);
        const int first = grp * GM;
        const int gsz = min(GM, tm_e - first);
        const int in = rem - grp * GM * tiles_n;
        const int tm = first + in % gsz;
        t.tn = in / gsz;
        const int rows = g.counts[e];
        if (LAY == GEMM_TN) { t.Mdim = g.Mo; t.Kdim = rows; } else { t.Mdim = rows; t.Kdim = g.K; }
        t.e = e;
        t.m0 = tm * BM;
        t.n0 = t.tn * BN;
        t.KT = (t.Kdim + BK - 1) / BK;
        if constexpr (LAY == GEMM_TN) {
            if (g.k_segs > 1) {
                t.Kdim = 0; t.KT = 0;
                for (int sg = 0; sg < g.k_segs; ++sg) {
                    const int r = g.counts[sg * g.E + e];
                    t.Kdim += r;
                    t.KT += (r + BK - 1) / BK;
                }
            }
        }
        if (t.m0 >= t.Mdim) return false;
        if (t.Kdim <= 0 && EPI != EPI_STORE_F32) return false;   // nothing to add; a plain store still writes zeros
        return true;
    };
    auto next_tile = [&](int b, TileCoord& t) -> int {          // first tile of this workgroup at or after b, or -1
        for (; b < nblocks; b += (int)gridDim.x)
            if (decode(b, t)) return b;
        return -1;
    };
    auto bind = [&](const TileCoord& t, AT& ta_, BT& tb_) {
        const bf16_t* A = (const bf16_t*)g.A + (size_t)t.e * g.a_estride;
        const bf16_t* B = (const bf16_t*)g.B + (size_t)t.e * g.b_estride;
        bool gathered = false;
        if constexpr (LAY != GEMM_TN) {
            if (g.a_rows) {
                ta_.init_gather((const bf16_t*)g.A, g.lda, g.a_rows + (size_t)t.e * g.Cp, t.m0, t.Mdim, g.a_row_limit,
                                t.Kdim, lane, wid);
                gathered = true;
            }
        }
        if (!gathered) ta_.init(A, g.lda, t.m0, t.Mdim, t.Kdim, lane, wid);
        tb_.init(B, g.ldb, t.n0, g.N, t.Kdim, lane, wid);
    };
    // load l of the tile that starts at k0.  Over several row ranges (TN) the tiles are requested in
    // ascending order, each starting with its load 0: that is where the cursor moves on, into the next
    // range with rows where the last one is used up (its operands then get new descriptors), and past
    // the last range, where everything reads as zeros.
    auto request = [&](const TileCoord& tc, KCursor& kc_, AT& ta_, BT& tb_, char* st, int k0, int l) {
        if constexpr (LAY == GEMM_TN) {
            if (g.k_segs > 1) {
                if (l == 0) {
                    if (k0 == 0) { kc_.seg = -1; kc_.jl = 0; kc_.tiles = 0; } else ++kc_.jl;
                    while (kc_.jl >= kc_.tiles) {
                        ++kc_.seg;
                        kc_.jl = 0;
                        const bool more = kc_.seg < g.k_segs;
                        const int rows = more ? g.counts[kc_.seg * g.E + tc.e] : 0;
                        kc_.tiles = more ? (rows + BK - 1) / BK : 0x7fffffff;
                        const bf16_t* A = (const bf16_t*)g.A + (size_t)tc.e * g.a_estride + kc_.seg * g.a_sstride + tc.m0;
                        const bf16_t* B = (const bf16_t*)g.B + (size_t)tc.e * g.b_estride + kc_.seg * g.b_sstride + tc.n0;
                        ta_.rsrc = AT::rsrc_of(A, g.lda, tc.Mdim - tc.m0, rows);
                        tb_.rsrc = BT::rsrc_of(B, g.ldb, g.N - tc.n0, rows);
                    }
                }
                k0 = kc_.jl * BK;
            }
        }
        if (l < AT::NI) ta_.load_one(st, k0, wid, l);
        else tb_.load_one(st + A_BYTES, k0, wid, l - AT::NI);
    };
    // two-ring loop: load l of wide unit u / of narrow tile j (k0 follows from the unit number)
    auto load_wide = [&](const AT& ta_, const BT& tb_, int slot3, int u, int l) {
        char* dst = smem + slot3 * WIDE_UNIT;
        if constexpr (A_WIDE) ta_.load_one(dst, u * 64, wid, l); else tb_.load_one(dst, u * 64, wid, l);
    };
    auto load_narrow = [&](const AT& ta_, const BT& tb_, int slot4, int j, int l) {
        char* dst = smem + NARROW_OFF + slot4 * NARROW_TILE;
        if constexpr (A_WIDE) tb_.load_one(dst, j * 32, wid, l); else ta_.load_one(dst, j * 32, wid, l);
    };
    constexpr int WL = W64 ? (A_WIDE ? AT::NI : BT::NI) : 0;       // loads per wave: one wide unit (8)
    constexpr int NL = W64 ? (A_WIDE ? BT::NI : AT::NI) : 0;       //                 one narrow tile (4)
    static_assert(!W64 || (WL == 8 && NL == 4), "the two-ring schedule issues two wide and two narrow loads per block");
    // the part of a tile's first loads that does not touch the staging region, and the rest
    auto issue_early = [&](const TileCoord& tc, KCursor& kc_, AT& ta_, BT& tb_) {
        if constexpr (W64) {
            // what the loop expects to be on its way when it starts: wide units 0 and 1 and the first
            // quarter of unit 2 (late: its slot is the staging region), narrow tiles 0..2 and half of tile 3
#pragma unroll
            for (int l = 0; l < WL; ++l) load_wide(ta_, tb_, 0, 0, l);
#pragma unroll
            for (int l = 0; l < NL; ++l) load_narrow(ta_, tb_, 0, 0, l);
#pragma unroll
            for (int l = 0; l < NL; ++l) load_narrow(ta_, tb_, 1, 1, l);
#pragma unroll
            for (int l = 0; l < WL; ++l) load_wide(ta_, tb_, 1, 1, l);
#pragma unroll
            for (int l = 0; l < NL; ++l) load_narrow(ta_, tb_, 2, 2, l);
#pragma unroll
            for (int l = 0; l < NL / 2; ++l) load_narrow(ta_, tb_, 3, 3, l);
        } else {
#pragma unroll
            for (int s = 0; s < 3; ++s)
#pragma unroll
                for (int l = 0; l < LPW; ++l) request(tc, kc_, ta_, tb_, smem + (SB + s) * STAGE, s * BK, l);
        }
    };
    auto issue_late = [&](const TileCoord& tc, KCursor& kc_, AT& ta_, BT& tb_) {
        if constexpr (W64) {
#pragma unroll
            for (int l = 0; l < WL / 4; ++l) load_wide(ta_, tb_, 2, 2, l);
        } else {
#pragma unroll
            for (int l = 0; l < LPW; ++l) request(tc, kc_, ta_, tb_, smem, 3 * BK, l);
#pragma unroll
            for (int l = 0; l < LPW / 2; ++l) request(tc, kc_, ta_, tb_, smem + STAGE, 4 * BK, l);
        }
    };

    TileCoord cur;
    int vb = next_tile(blockIdx.x, cur);
    if (vb < 0) return;
    AT ta;
    BT tb;
    bind(cur, ta, tb);
    KCursor kc = {0, 0, 0};
    issue_early(cur, kc, ta, tb);
    issue_late(cur, kc, ta, tb);
    bool first = true;

    for (;;) {
        const int m0 = cur.m0, n0 = cur.n0, e = cur.e, tn = cur.tn, Mdim = cur.Mdim, KT = cur.KT;
        floatx16 acc[TM][TNN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TNN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

        if constexpr (W64) {
            // Hand-scheduled loop over steps of 64 k = four blocks of TM x TN matrix instructions (16 k each).
            // While block b is multiplied, the fragments of block b+1 are read and four loads are issued, one
            // LDS read or load per matrix instruction.  Step t reads wide unit t (slot t mod 3) and narrow
            // tiles 2t, 2t+1 (slots mod 4).  Two barriers per step:
            //   after block 0: every wave has read narrow tile 2t for the last time (its slot then receives
            //           tile 2t+4), and tile 2t+1 has landed;
            //   after block 2: every wave has read wide unit t and narrow tile 2t+1 for the last time (their
            //           slots receive unit t+3 and tile 2t+5), and unit t+1 and tile 2t+2 have landed.
            // Each wave issues, per step, in this order: block 0 - wide unit t+2 loads 2,3, narrow tile 2t+3
            // loads 2,3; block 1 - unit t+2 loads 4,5, tile 2t+4 loads 0,1; block 2 - unit t+2 loads 6,7, tile
            // 2t+4 loads 2,3; block 3 - unit t+3 loads 0,1, tile 2t+5 loads 0,1.  At either barrier the sixteen
            // youngest loads of the wave may still be in flight; everything older is what the step needs next.
            constexpr int MB = TM * TNN, FR = TM + TNN;
            static_assert(FR + 7 <= MB, "one LDS read per matrix instruction, then a load after every other one");
            if (first) wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            bf16x8 F0[FR], F1[FR];
            // fragment f of 16-k block kk of a step: from the wide unit at wb or from the narrow tile pair at nb0, nb1
            auto frag = [&](int f, int kk, const char* wb, const char* nb0, const char* nb1) -> bf16x8 {
                const char* nb = kk < 2 ? nb0 : nb1;
                if constexpr (A_WIDE) return f < TM ? fa[f].read(wb, kk) : fb[f - TM].read(nb, kk & 1);
                else return f < TM ? fa[f].read(nb, kk & 1) : fb[f - TM].read(wb, kk);
            };
#pragma unroll
            for (int f = 0; f < FR; ++f) F0[f] = frag(f, 0, smem, smem + NARROW_OFF, smem + NARROW_OFF);
            int w3 = 0, n4 = 0;                       // slot of wide unit t, slot of narrow tile 2t
#pragma unroll 1
            for (int t = 0; t < KT; ++t) {
                const int w3a = w3 == 2 ? 0 : w3 + 1, w3b = w3a == 2 ? 0 : w3a + 1;   // slots of units t+1, t+2
                const int n4b = n4 ^ 2;                                               // slot of tile 2t+2
                const char* wb = smem + w3 * WIDE_UNIT;
                const char* nb0 = smem + NARROW_OFF + n4 * NARROW_TILE;
                const char* nb1 = nb0 + NARROW_TILE;
                const char* wb_next = smem + w3a * WIDE_UNIT;
                const char* nb_next = smem + NARROW_OFF + n4b * NARROW_TILE;
                // block 0
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    mfma_pinned<true>(acc[m / TNN][m % TNN], F0[TM + m % TNN], F0[m / TNN]);
                    if (m < FR) F1[m] = frag(m, 1, wb, nb0, nb1);
                    else if (m == FR || m == FR + 2) load_wide(ta, tb, w3b, t + 2, 2 + (m - FR) / 2);
                    else if (m == FR + 4 || m == FR + 6) load_narrow(ta, tb, n4b + 1, 2 * t + 3, 2 + (m - FR - 4) / 2);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                wait_vmcnt<16>();
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                // block 1
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    mfma_pinned<true>(acc[m / TNN][m % TNN], F1[TM + m % TNN], F1[m / TNN]);
                    if (m < FR) F0[m] = frag(m, 2, wb, nb0, nb1);
                    else if (m == FR || m == FR + 2) load_wide(ta, tb, w3b, t + 2, 4 + (m - FR) / 2);
                    else if (m == FR + 4 || m == FR + 6) load_narrow(ta, tb, n4, 2 * t + 4, (m - FR - 4) / 2);
                }
                // block 2
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    mfma_pinned<true>(acc[m / TNN][m % TNN], F0[TM + m % TNN], F0[m / TNN]);
                    if (m < FR) F1[m] = frag(m, 3, wb, nb0, nb1);
                    else if (m == FR || m == FR + 2) load_wide(ta, tb, w3b, t + 2, 6 + (m - FR) / 2);
                    else if (m == FR + 4 || m == FR + 6) load_narrow(ta, tb, n4, 2 * t + 4, 2 + (m - FR - 4) / 2);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                wait_vmcnt<16>();
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                // block 3
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    mfma_pinned<true>(acc[m / TNN][m % TNN], F1[TM + m % TNN], F1[m / TNN]);
                    if (m < FR) F0[m] = frag(m, 0, wb_next, nb_next, nb_next);
                    else if (m == FR || m == FR + 2) load_wide(ta, tb, w3, t + 3, (m - FR) / 2);
                    else if (m == FR + 4 || m == FR + 6) load_narrow(ta, tb, n4 + 1, 2 * t + 5, (m - FR - 4) / 2);
                }
                w3 = w3a;
                n4 = n4b;
            }
            asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        } else {
            // Hand-scheduled loop (with one wave per SIMD nothing else hides a stall): every
            // LDS read and every load into LDS sits between two matrix instructions, one per
            // instruction, and the data a block of TM x TN matrix instructions needs was
            // requested during the block before.
            // A tile is 32 k = two such blocks; the ring holds five tiles.  In iteration t
            //   block 0 multiplies k 0..15 of tile t, reads k 16..31 of it into the second
            //           fragment set and requests the second half of tile t+4;
            //   then the wave waits for its part of tile t+1 and meets the others (their
            //           parts have landed too, and nobody reads stage t any more);
            //   block 1 multiplies k 16..31, reads k 0..15 of tile t+1 into the first
            //           fragment set and requests the first half of tile t+5 into stage t.
            // Up to four tiles (128 KB) are in flight towards a CU.
            constexpr int MB = TM * TNN;                 // matrix instructions per block
            constexpr int FR = TM + TNN;                 // fragments per block: A rows first, then B columns
            static_assert(LPW % 2 == 0 && FR + LPW / 2 <= MB, "one LDS read or load per matrix instruction");
            // a load costs the wave more issue time than one matrix instruction hides: where there is room,
            // only every other matrix instruction is followed by one
            constexpr int LS = (FR + 2 * (LPW / 2) - 1 <= MB) ? 2 : 1;
            if (first) wait_vmcnt<3 * LPW + LPW / 2>();            // tile 0 is in (later tiles: waited for at the handover)
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            bf16x8 F0[FR], F1[FR];
#pragma unroll
            for (int f = 0; f < FR; ++f)
                F0[f] = f < TM ? fa[f].read(smem + SB * STAGE, 0) : fb[f - TM].read(smem + SB * STAGE + A_BYTES, 0);
            int st = SB;
#pragma unroll 1
            for (int kt = 0; kt < KT; ++kt) {
                char* cs = smem + st * STAGE;
                const int stn = (st + 1 == NS) ? 0 : st + 1;
                const int stp = (st == 0) ? NS - 1 : st - 1;
                char* nxt = smem + stn * STAGE;
                char* prv = smem + stp * STAGE;
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    mfma_pinned<C::OCC == 1>(acc[m / TNN][m % TNN], F0[TM + m % TNN], F0[m / TNN]);
                    if (m < TM) F1[m] = fa[m].read(cs, 1);
                    else if (m < FR) F1[m] = fb[m - TM].read(cs + A_BYTES, 1);
                    else if (m - FR < LS * (LPW / 2) && (m - FR) % LS == 0) request(cur, kc, ta, tb, prv, (kt + 4) * BK, LPW / 2 + (m - FR) / LS);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave no longer reads stage t
                wait_vmcnt<3 * LPW>();                               // its part of tile t+1 is in
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    mfma_pinned<C::OCC == 1>(acc[m / TNN][m % TNN], F1[TM + m % TNN], F1[m / TNN]);
                    if (m < TM) F0[m] = fa[m].read(nxt, 0);
                    else if (m < FR) F0[m] = fb[m - TM].read(nxt + A_BYTES, 0);
                    else if (m - FR < LS * (LPW / 2) && (m - FR) % LS == 0) request(cur, kc, ta, tb, cs, (kt + 5) * BK, (m - FR) / LS);
                }
                st = stn;
            }
            // the assembler-level matrix instructions are invisible to the compiler's hazard
            // checks: let the last of them retire before anything reads the accumulators
            asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        }
        wait_vmcnt<0>();                             // nothing of this workgroup is in flight into LDS any more
        __builtin_amdgcn_s_barrier();                // and every wave is done reading the ring
        asm volatile("" ::: "memory");

        // ---- the tile after this one ------------------------------------------------------
        TileCoord nx;
        AT ta2;
        BT tb2;
        KCursor kc2 = {0, 0, 0};
        const int vn = next_tile(vb + (int)gridDim.x, nx);
        if (vn >= 0) bind(nx, ta2, tb2);

        // ---- epilogue -----------------------------------------------------------------------
        // An MFMA accumulator holds one row per lane (row = lane & 31, four consecutive
        // columns per register group), which would make every global access a 8- or 16-byte
        // piece of 32 different rows.  Each wave therefore passes its 32 x WN blocks through a
        // private LDS region (float, 16-byte chunks XOR-swizzled by row) and picks them up
        // with eight consecutive columns per lane, so that eight lanes cover a whole line of
        // a row: all global reads and writes of the epilogue are 16 or 32 bytes per lane,
        // row-contiguous.  They go through buffer descriptors that end after the last valid
        // row, so there is no branch: out-of-range reads give zero, out-of-range writes are
        // dropped, and all reads of a 32-row pass are issued before the arithmetic starts.
        // A pass moves 32 rows x CW columns of the wave's block (CW = the block's width, or 64 where the
        // staging region is one ring unit).
        constexpr int CPRW = CW / 8;                 // 8-column pieces per row of a pass
        constexpr int NPIECE = 32 * CPRW / 64;       // pieces per lane
        constexpr int NCH = WN / CW, TJ = CW / 32;   // passes per 32 rows; 32-column accumulator blocks per pass
        constexpr int NPASS = TM * NCH;
        float* stage = reinterpret_cast<float*>(smem + C::STAGING_OFF + wid * (32 * CW * 4));
        constexpr int CES = (EPI == EPI_ACCUM_F32 || EPI == EPI_STORE_F32) ? 4 : 2;   // bytes per output element
        // (scattered rows: the whole output matrix, every row of which some tile may write)
        const char* Cbase = EPI == EPI_SCATTER ? (const char*)g.C : (const char*)g.C + (size_t)e * g.c_estride * CES;
        const __amdgpu_buffer_rsrc_t rC = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char*>(Cbase), 0,
            (unsigned)(((size_t)((EPI == EPI_SCATTER ? g.c_row_limit : Mdim) - 1) * g.ldc + g.N) * CES), 0x00020000);
        const int* crows = g.c_rows ? g.c_rows + (size_t)e * g.Cp : nullptr;
        const bf16_t* Zbase = g.Z ? (const bf16_t*)g.Z + (size_t)e * g.Cp * g.ldz : nullptr;
        const __amdgpu_buffer_rsrc_t rZ = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<bf16_t*>(Zbase), 0, Zbase ? (unsigned)(((size_t)(Mdim - 1) * g.ldz + g.N) * 2) : 0u, 0x00020000);
        const float* wbase = g.slot_w ? g.slot_w + (size_t)e * g.Cp : nullptr;
        const int erow = lane & 31, ehalf = lane >> 5;
        // What a pass reads from memory (the pre-activation and row weight for GeLU-backward, the old
        // sums for float accumulation) is requested one pass ahead.
        constexpr bool READS = (EPI == EPI_DGELU || EPI == EPI_ACCUM_F32 || EPI == EPI_SCATTER);
        struct PassIn { uint4 zin[NPIECE]; float4 cin0[NPIECE], cin1[NPIECE]; float wrow[NPIECE]; int crow[NPIECE]; };
        auto piece = [&](int ps, int t, int& m, int& c8, int& row, unsigned& oC, unsigned& oZ) {
            const int idx = lane + 64 * t;
            row = idx / CPRW; c8 = idx % CPRW;
            m = m0 + wm * WM + (ps / NCH) * 32 + row;
            const int n = n0 + wn * WN + (ps % NCH) * CW + c8 * 8;
            const bool in = n < g.N;                 // rows beyond Mdim fall outside the descriptors by themselves
            oC = in ? (unsigned)(m * g.ldc + n) * CES : OOB_OFFSET;
            oZ = in ? (unsigned)(m * g.ldz + n) * 2u : OOB_OFFSET;
        };
        // Float outputs: a lane's two 16-byte halves of "piece" t are units 2t and 2t+1 of a numbering in which the
        // 64 lanes of one store (or load) cover whole rows of the pass - 4 columns per lane, CW/4 lanes per row - so
        // that every such instruction moves whole 128-byte lines (8 columns per lane would leave each instruction
        // with every other 16 bytes).  Unit u of a lane is UROWS*u rows below its unit 0, in the same columns: one
        // vector offset per pass, the rest is a scalar offset.
        constexpr int ULANES = CW / 4, UROWS = 64 / ULANES;
        const int urow = lane / ULANES, uc4 = lane % ULANES;
        auto unit0 = [&](int ps) -> unsigned {
            const int m = m0 + wm * WM + (ps / NCH) * 32 + urow;
            const int n = n0 + wn * WN + (ps % NCH) * CW + uc4 * 4;
            return n < g.N ? (unsigned)(m * g.ldc + n) * 4u : OOB_OFFSET;
        };
        const unsigned ustep = (unsigned)(UROWS * g.ldc) * 4u;      // bytes from one unit of a lane to the next
        auto request_pass = [&](int ps, PassIn& in) {
#pragma unroll
            for (int t = 0; t < NPIECE; ++t) {
                int m, c8, row; unsigned oC, oZ;
                piece(ps, t, m, c8, row, oC, oZ);
                if constexpr (EPI == EPI_DGELU) {
                    in.zin[t] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rZ, oZ, 0, 0));
                    in.wrow[t] = m < Mdim ? wbase[m] : 0.0f;
                }
                if constexpr (EPI == EPI_SCATTER) {
                    in.crow[t] = m < Mdim ? crows[m] : -1;
                    in.wrow[t] = m < Mdim ? wbase[m] : 0.0f;
                }
                if constexpr (EPI == EPI_ACCUM_F32) {
                    const unsigned ob = unit0(ps);
                    in.cin0[t] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rC, ob, (2 * t) * ustep, 0));
                    in.cin1[t] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rC, ob, (2 * t + 1) * ustep, 0));
                }
            }
        };
        PassIn pin[2];
        if constexpr (READS) request_pass(0, pin[0]);
        float dotacc[NPIECE];                        // GeLU-backward: <gelu(Z), G> of a row over the passes of its 32 rows
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int i = ps / NCH, ch = ps % NCH;
#pragma unroll
            for (int jj = 0; jj < TJ; ++jj) {
                const int j = ch * TJ + jj;
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int cch = (jj * 32 + g4 * 8 + ehalf * 4) >> 2;
                    float4 v = make_float4(acc[i][j][g4 * 4 + 0], acc[i][j][g4 * 4 + 1], acc[i][j][g4 * 4 + 2], acc[i][j][g4 * 4 + 3]);
                    *reinterpret_cast<float4*>(stage + erow * CW + ((cch ^ (erow & 15)) << 2)) = v;
                }
            }
            if constexpr (READS) { if (ps + 1 < NPASS) request_pass(ps + 1, pin[(ps + 1) & 1]); }
            const PassIn& in = pin[ps & 1];
            // all LDS reads of the pass before its arithmetic: one round trip through LDS, not one per piece
            // (float accumulation keeps the old sums of two passes in registers and has none left for that)
            constexpr bool HOIST = EPI != EPI_ACCUM_F32;
            float4 lo[NPIECE], hi[NPIECE];
            auto read_piece = [&](int t) {
                if constexpr (CES == 4) {
                    const int r0 = urow + UROWS * (2 * t), r1 = r0 + UROWS;
                    lo[t] = *reinterpret_cast<const float4*>(stage + r0 * CW + ((uc4 ^ (r0 & 15)) << 2));
                    hi[t] = *reinterpret_cast<const float4*>(stage + r1 * CW + ((uc4 ^ (r1 & 15)) << 2));
                } else {
                    const int idx = lane + 64 * t;
                    const int row = idx / CPRW, c8 = idx % CPRW;
                    lo[t] = *reinterpret_cast<const float4*>(stage + row * CW + (((2 * c8) ^ (row & 15)) << 2));
                    hi[t] = *reinterpret_cast<const float4*>(stage + row * CW + (((2 * c8 + 1) ^ (row & 15)) << 2));
                }
            };
            if constexpr (HOIST) {
#pragma unroll
                for (int t = 0; t < NPIECE; ++t) read_piece(t);
            }
#pragma unroll
            for (int t = 0; t < NPIECE; ++t) {
                int m, c8, row; unsigned oC, oZ;
                piece(ps, t, m, c8, row, oC, oZ);
                if constexpr (!HOIST) read_piece(t);
                float v[8] = {lo[t].x, lo[t].y, lo[t].z, lo[t].w, hi[t].x, hi[t].y, hi[t].z, hi[t].w};
                if constexpr (EPI == EPI_STORE) {
                    uint4 o = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, o), rC, oC, 0, 0);
                } else if constexpr (EPI == EPI_SCATTER) {
                    // the row's place in the output and its weight; rows and columns out of range are dropped
                    const float w = in.wrow[t];
                    const int n = n0 + wn * WN + (ps % NCH) * CW + c8 * 8;
                    const unsigned oS = (in.crow[t] >= 0 && oC != OOB_OFFSET) ? (unsigned)(in.crow[t] * g.ldc + n) * 2u : OOB_OFFSET;
                    uint4 o = make_uint4(pack_bf16x2(w * v[0], w * v[1]), pack_bf16x2(w * v[2], w * v[3]),
                                         pack_bf16x2(w * v[4], w * v[5]), pack_bf16x2(w * v[6], w * v[7]));
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, o), rC, oS, 0, 0);
                } else if constexpr (EPI == EPI_GELU) {
                    float z[8], a[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) { z[q] = bf16_to_f32(f32_to_bf16(v[q])); a[q] = gelu_fast_f(z[q]); }
                    uint4 oz = make_uint4(pack_bf16x2(z[0], z[1]), pack_bf16x2(z[2], z[3]), pack_bf16x2(z[4], z[5]), pack_bf16x2(z[6], z[7]));
                    uint4 oa = make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(a[4], a[5]), pack_bf16x2(a[6], a[7]));
                    if (Zbase) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, oz), rZ, oZ, 0, 0);
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, oa), rC, oC, 0, 0);
                } else if constexpr (EPI == EPI_DGELU) {
                    float z[8], dz[8], a[8];
                    Unit8::to_float(in.zin[t], z);
                    const float w = in.wrow[t];
                    float dot = ch == 0 ? 0.0f : dotacc[t];
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        float gq, dg;
                        gelu_both_fast_f(z[q], &gq, &dg);
                        // columns out of range read z = 0 and an accumulator of 0: nothing to add; rows out of
                        // range are never written below
                        dot = fmaf(gq, v[q], dot);
                        a[q] = w * gq;
                        dz[q] = w * v[q] * dg;
                    }
                    dotacc[t] = dot;
                    uint4 od = make_uint4(pack_bf16x2(dz[0], dz[1]), pack_bf16x2(dz[2], dz[3]), pack_bf16x2(dz[4], dz[5]), pack_bf16x2(dz[6], dz[7]));
                    uint4 oa = make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(a[4], a[5]), pack_bf16x2(a[6], a[7]));
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, od), rC, oC, 0, 0);
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, oa), rZ, oZ, 0, 0);
                    if (g.dw_part && ch == NCH - 1) {
                        // the CPRW lanes of a row are neighbours
#pragma unroll
                        for (int off = CPRW / 2; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, 64);
                        if (c8 == 0 && m < Mdim)
                            g.dw_part[((size_t)e * g.Cp + m) * g.dw_parts + tn * C::WAVES_N + wn] = dot;
                    }
                } else if constexpr (EPI == EPI_STORE_F32) {
                    const unsigned ob = unit0(ps);
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, lo[t]), rC, ob, (2 * t) * ustep, 0);
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, hi[t]), rC, ob, (2 * t + 1) * ustep, 0);
                } else {
                    const unsigned ob = unit0(ps);
                    float4 o0 = in.cin0[t], o1 = in.cin1[t];
                    o0.x += v[0]; o0.y += v[1]; o0.z += v[2]; o0.w += v[3];
                    o1.x += v[4]; o1.y += v[5]; o1.z += v[6]; o1.w += v[7];
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, o0), rC, ob, (2 * t) * ustep, 0);
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, o1), rC, ob, (2 * t + 1) * ustep, 0);
                }
            }
            // the next tile's first operand tiles start their trip once the first pass is through
            // (earlier, and this pass's own reads would have to wait behind them)
            if (ps == 0 && vn >= 0) issue_early(nx, kc2, ta2, tb2);
        }
        if (vn < 0) break;
        // Everything this wave has in flight is through: the next tile's first operand tiles have
        // landed and the epilogue's stores are written.  (Counting on the stores being younger than
        // the loads would save waiting for the last of them, but the main loop's third wait would
        // wait for them anyway: vmcnt retires in order.)
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();                // every wave is done with the staging stages
        asm volatile("" ::: "memory");
        issue_late(nx, kc2, ta2, tb2);
        kc = kc2;
        ta = ta2;
        tb = tb2;
        cur = nx;
        vb = vn;
        first = false;
    }
}

// Tile shapes in use.  Both cover 256 x 256 per workgroup with four waves of 128 x 128, one per SIMD.
//   CfgW   two-ring loop: for every GEMM with a K-contiguous operand (NN, NT).  A request for half a
//          128-byte line costs the L1 as much as one for a whole line, and the loop's speed follows
//          the number of requests; here every request but those of NT's row operand is a whole line.
//   Cfg4   ring of 5 x 32 k: the weight-gradient GEMMs (TN), whose two operands are N-contiguous
//          and come in whole lines anyway.
// (Shapes with two waves of 128 x 64 per SIMD - TileCfg<256, 256, 32, 5, 2, 4, 2, LOOP_PIPE32> - ran the GeLU
// epilogues faster and the main loops slower, reading half as much again from LDS; with the cheaper GeLU
// arithmetic the four-wave shapes win everywhere.)
typedef TileCfg<256, 256, 32, 5, 2, 2, 1, LOOP_PIPE32> Cfg4;
typedef TileCfg<256, 256, 64, 3, 2, 2, 1, LOOP_W64> CfgW;
template <int LAY, int EPI> struct CfgFor { typedef CfgW type; };
template <int EPI> struct CfgFor<GEMM_TN, EPI> { typedef Cfg4 type; };
// every layout reports the row dot of the GeLU-backward epilogue in the same number of column blocks
typedef CfgFor<GEMM_NT, EPI_DGELU>::type CfgDgelu;
static_assert(CfgFor<GEMM_NN, EPI_DGELU>::type::WAVES_N * 256 / CfgFor<GEMM_NN, EPI_DGELU>::type::BN ==
              CfgDgelu::WAVES_N * 256 / CfgDgelu::BN &&
              CfgFor<GEMM_TN, EPI_DGELU>::type::WAVES_N * 256 / CfgFor<GEMM_TN, EPI_DGELU>::type::BN ==
              CfgDgelu::WAVES_N * 256 / CfgDgelu::BN, "column blocks per 256 columns");

int gemm_bf16_dw_parts(int H) { return ((H + CfgDgelu::BN - 1) / CfgDgelu::BN) * CfgDgelu::WAVES_N; }

// One workgroup per CU (a workgroup fills a CU's LDS), rounded down to a multiple of 8 so that
// tile numbers keep their XCD.
static int persistent_grid() {
    static int grid = 0;
    if (grid == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
            cus = 256;
        grid = cus / 8 * 8;
    }
    return grid;
}

template <int LAY, int EPI, typename C>
static moe_status launch_one(const GemmArgs& a, hipStream_t s) {
    const int Mmax = (LAY == GEMM_TN) ? a.Mo : a.Cp;
    const int tiles_m = (Mmax + C::BM - 1) / C::BM, tiles_n = (a.N + C::BN - 1) / C::BN;
    int nblocks = a.E * tiles_m * tiles_n;
    nblocks = (nblocks + 7) / 8 * 8;
    int full = persistent_grid() - (a.free_cus + 7) / 8 * 8;
    if (full < 8) full = 8;
    const int grid = nblocks < full ? nblocks : full;
    constexpr int lds = C::LDS_BYTES;
    auto kern = gemm_bf16_kernel<LAY, EPI, C>;
    static bool attr_done = false;
    if (!attr_done) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_done = true;
    }
    {
        ProfScope ps(gemm_prof_kind(LAY, EPI), s);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(C::THREADS), lds, s, a, tiles_m, tiles_n);
    }
    count_launch(LC_GEMM);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

// Only the combinations the expert FFN uses are instantiated: NN with plain, GeLU and scattered stores
// (both layers of forward, recomputation), NT with GeLU-backward and plain stores (the two input
// gradients), TN with float store and float accumulation (the weight gradients).
template <int LAY, int EPI>
static moe_status launch_cfg(const GemmArgs& a, hipStream_t s) {
    return launch_one<LAY, EPI, typename CfgFor<LAY, EPI>::type>(a, s);
}

}  // namespace moe
namespace moe {
moe_status gemm_bf16(GemmLayout lay, GemmEpilogue epi, const GemmArgs& a, hipStream_t s) {
    if (a.dw_part && a.dw_parts != gemm_bf16_dw_parts(a.N)) return MOE_ERR_SHAPE;
    // operand rows must be 16-byte aligned in memory
    if ((a.lda | a.ldb) & 7) return MOE_ERR_UNSUPPORTED;
    // buffer offsets are 32-bit: an expert's operand must stay below 2 GiB
    const long long ldmax = a.lda > a.ldb ? a.lda : a.ldb;
    const long long rmax = a.Cp > a.K ? a.Cp : a.K;
    if ((rmax + 8 * 64) * ldmax * 2 >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    if (a.k_segs > 1 && (lay != GEMM_TN || a.k_segs > MAX_KSEGS)) return MOE_ERR_UNSUPPORTED;
    if (epi == EPI_SCATTER) {
        if (lay == GEMM_TN || !a.c_rows || !a.slot_w || a.c_row_limit <= 0) return MOE_ERR_UNSUPPORTED;
        if (((long long)a.c_row_limit + 1) * a.ldc * 2 >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    }
    if (a.a_rows) {
        // gathered rows: only for the row operand of NN / NT, and the whole matrix must stay below 2 GiB
        if (lay == GEMM_TN || a.a_row_limit <= 0) return MOE_ERR_UNSUPPORTED;
        if (((long long)a.a_row_limit + 1) * a.lda * 2 >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    }
    if (lay == GEMM_NN && epi == EPI_STORE) return launch_cfg<GEMM_NN, EPI_STORE>(a, s);
    if (lay == GEMM_NN && epi == EPI_GELU) return launch_cfg<GEMM_NN, EPI_GELU>(a, s);
    if (lay == GEMM_NN && epi == EPI_SCATTER) return launch_cfg<GEMM_NN, EPI_SCATTER>(a, s);
    if (lay == GEMM_NT && epi == EPI_STORE) return launch_cfg<GEMM_NT, EPI_STORE>(a, s);
    if (lay == GEMM_NT && epi == EPI_DGELU) return launch_cfg<GEMM_NT, EPI_DGELU>(a, s);
    if (lay == GEMM_TN && epi == EPI_STORE_F32) return launch_cfg<GEMM_TN, EPI_STORE_F32>(a, s);
    if (lay == GEMM_TN && epi == EPI_ACCUM_F32) return launch_cfg<GEMM_TN, EPI_ACCUM_F32>(a, s);
    return MOE_ERR_UNSUPPORTED;
}

}  // namespace moe
