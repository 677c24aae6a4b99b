// Capacity-bounded slot assignment.  The paper has no capacity (its batch is
// "dynamic", Section III-C); here every micro-batch of Section III-B is an
// independent MoE call with C_p rows per expert, which is what makes partition
// buffers exactly 1/n of the whole (Section III-D).  Inside a partition,
// positions are granted choice-major then in token order, by a stable ranking:
// per-block histograms, a prefix over the blocks that come earlier in that
// order, and a stable in-block rank.  No result depends on atomic ordering.
#include "common.h"

namespace moe {

constexpr int SLOT_BLOCK = 1024;   // assignments ranked by one workgroup

// hist[((p*k + j)*nb + b)*E + e] = number of tokens of block b (partition p) whose
// j-th choice is expert e
__global__ __launch_bounds__(SLOT_BLOCK) void slot_hist_kernel(
    const int* __restrict__ topk_idx, int* __restrict__ hist, int Tp, int k, int E, int nb) {
    __shared__ int h[64];
    const int b = blockIdx.x, j = blockIdx.y, p = blockIdx.z;
    if (threadIdx.x < 64) h[threadIdx.x] = 0;
    __syncthreads();
    const int tl = b * SLOT_BLOCK + threadIdx.x;
    if (tl < Tp) {
        int e = topk_idx[(size_t)(p * Tp + tl) * k + j];
        atomicAdd(&h[e], 1);             // integer counts: order does not matter
    }
    __syncthreads();
    if (threadIdx.x < E) hist[((size_t)(p * k + j) * nb + b) * E + threadIdx.x] = h[threadIdx.x];
}

__global__ __launch_bounds__(SLOT_BLOCK) void slot_assign_kernel(
    const int* __restrict__ topk_idx, const float* __restrict__ topk_w, const int* __restrict__ hist,
    int* __restrict__ slot, int* __restrict__ counts, float* __restrict__ slot_w,
    int Tp, int k, int E, int nb, int Cp) {
    __shared__ int base[64];
    __shared__ int wcount[SLOT_BLOCK / 64][64];
    const int b = blockIdx.x, j = blockIdx.y, p = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    if (tid < 64) {
        int before = 0, total = 0;
        if (tid < E) {
            const int mine = j * nb + b;
            for (int q = 0; q < k * nb; ++q) {
                int v = hist[((size_t)p * k * nb + q) * E + tid];
                total += v;
                if (q < mine) before += v;
            }
            if (b == 0 && j == 0) counts[p * E + tid] = total < Cp ? total : Cp;
        }
        base[tid] = before;
    }
    const int tl = b * SLOT_BLOCK + tid;
    const bool valid = tl < Tp;
    const int t = p * Tp + tl;
    const int my_e = valid ? topk_idx[(size_t)t * k + j] : -1;
    int rank = 0;
    for (int e = 0; e < E; ++e) {
        unsigned long long m = __ballot(my_e == e);
        if (my_e == e) rank = __popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) wcount[wid][e] = __popcll(m);
    }
    __syncthreads();
    if (valid) {
        int pos = base[my_e] + rank;
        for (int w = 0; w < wid; ++w) pos += wcount[w][my_e];
        int s = pos < Cp ? my_e * Cp + pos : -1;
        slot[(size_t)t * k + j] = s;
        if (s >= 0 && slot_w) slot_w[(size_t)p * E * Cp + s] = topk_w[(size_t)t * k + j];
    }
}

// rows[p][slot[t,j]] = t for kept assignments: the map a gathering GEMM reads its rows through
__global__ __launch_bounds__(256) void slot_rows_kernel(const int* __restrict__ slot, int* __restrict__ rows,
                                                        int T, int Tp, int k, int Rp) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= T * k) return;
    const int t = i / k;
    const int s = slot[i];
    if (s >= 0) rows[(size_t)(t / Tp) * Rp + s] = t;
}

}  // namespace moe

extern "C" moe_status moe_slot_rows(const moe_config* cfg, const int32_t* slot, int32_t* rows, void* stream) {
    moe::Dims d;
    MOE_TRY(moe::make_dims(cfg, &d));
    if (!slot || !rows) return MOE_ERR_NULL;
    const int total = d.T * d.k;
    hipLaunchKernelGGL(moe::slot_rows_kernel, dim3((total + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                       slot, rows, d.T, d.Tp, d.k, d.Rp);
    moe::count_launch(moe::LC_OTHER);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

extern "C" moe_status moe_slot_scratch_bytes(const moe_config* cfg, size_t* bytes) {
    moe::Dims d;
    MOE_TRY(moe::make_dims(cfg, &d));
    if (!bytes) return MOE_ERR_NULL;
    int nb = (d.Tp + moe::SLOT_BLOCK - 1) / moe::SLOT_BLOCK;
    *bytes = (size_t)d.n * d.k * nb * d.E * sizeof(int);
    return MOE_OK;
}

namespace moe {

static moe_status assign_slots(const Dims& d, const int32_t* topk_idx, const float* topk_w, int32_t* slot,
                               int32_t* counts, float* slot_w, int* hist, hipStream_t s) {
    const int nb = (d.Tp + SLOT_BLOCK - 1) / SLOT_BLOCK;
    dim3 grid(nb, d.k, d.n);
    ProfScope ps(PK_SLOTS, s);
    hipLaunchKernelGGL(slot_hist_kernel, grid, dim3(SLOT_BLOCK), 0, s, topk_idx, hist, d.Tp, d.k, d.E, nb);
    MOE_CHECK_LAUNCH();
    hipLaunchKernelGGL(slot_assign_kernel, grid, dim3(SLOT_BLOCK), 0, s, topk_idx, topk_w, (const int*)hist, slot,
                       counts, slot_w, d.Tp, d.k, d.E, nb, d.Cp);
    count_launch(LC_OTHER, 2);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

// Histogram memory of moe_assign_slots_static: one array per GPU, resident for the life of the
// process.  In host code this name is only a handle for hipGetSymbolAddress; the device address
// it yields (one per device) is what kernels are given.
constexpr size_t STATIC_SCRATCH_BYTES = 256 * 1024;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_static_scratch[MAX_DEVICES];

static moe_status static_scratch(void** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return MOE_ERR_UNSUPPORTED;
    if (!g_static_scratch[dev]) {
        void* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return MOE_ERR_HIP;
        g_static_scratch[dev] = ptr;
    }
    *out = g_static_scratch[dev];
    return MOE_OK;
}

}  // namespace moe

extern "C" moe_status moe_assign_slots(const moe_config* cfg, const int32_t* topk_idx, const float* topk_w,
                                       int32_t* slot, int32_t* counts, float* slot_w,
                                       void* scratch, void* stream) {
    moe::Dims d;
    MOE_TRY(moe::make_dims(cfg, &d));
    if (!topk_idx || !slot || !counts || !scratch) return MOE_ERR_NULL;
    if (slot_w && !topk_w) return MOE_ERR_NULL;
    return moe::assign_slots(d, topk_idx, topk_w, slot, counts, slot_w, (int*)scratch, (hipStream_t)stream);
}

extern "C" moe_status moe_assign_slots_static(const moe_config* cfg, const int32_t* topk_idx, const float* topk_w,
                                              int32_t* slot, int32_t* counts, float* slot_w, void* stream) {
    moe::Dims d;
    MOE_TRY(moe::make_dims(cfg, &d));
    if (!topk_idx || !slot || !counts) return MOE_ERR_NULL;
    if (slot_w && !topk_w) return MOE_ERR_NULL;
    size_t need = 0;
    MOE_TRY(moe_slot_scratch_bytes(cfg, &need));
    if (need > moe::STATIC_SCRATCH_BYTES) return MOE_ERR_WORKSPACE;
    void* hist = nullptr;
    MOE_TRY(moe::static_scratch(&hist));
    // every histogram entry the ranking kernel reads is written by the histogram kernel of the same
    // call, so nothing of an earlier call's contents has to be cleared
    return moe::assign_slots(d, topk_idx, topk_w, slot, counts, slot_w, (int*)hist, (hipStream_t)stream);
}
