// Adaptive pipeline granularity (Algorithm 1, Section III-C): how many partitions
// n a batch of B tokens should be cut into, found with as few timed searches as
// possible.  State per handle: the ordered set S of pairs (range of B, n), one
// per n, kept in a balanced tree keyed by the lower bound as the section
// prescribes, and a hash table B -> n.  Host code only; the search by trials
// times moe_layer_step with HIP events.
#include "common.h"

#include <map>
#include <unordered_map>
#include <vector>

struct moe_gran {
    struct Range { long long upper; int n; };
    std::map<long long, Range> by_lower;                // S, ordered by lower bound
    std::unordered_map<long long, int> cache_table;     // B -> n
};

using namespace moe;

namespace {

// find(S, B): the pair whose range holds B.  Ranges are disjoint while the best n
// grows with B (the section's hypothesis); should they overlap, the one with the
// smallest lower bound wins.
int find_n(const moe_gran* g, long long B) {
    for (auto it = g->by_lower.begin(); it != g->by_lower.end() && it->first <= B; ++it)
        if (B <= it->second.upper) return it->second.n;
    return -1;
}

// Disjoint ranges (the normal case) need only the last pair that starts at or below B.
int find_n_disjoint(const moe_gran* g, long long B) {
    auto it = g->by_lower.upper_bound(B);
    if (it == g->by_lower.begin()) return -1;
    --it;
    return B <= it->second.upper ? it->second.n : -1;
}

bool disjoint(const moe_gran* g) {
    long long last_upper = 0;
    bool first = true;
    for (const auto& kv : g->by_lower) {
        if (!first && kv.first <= last_upper) return false;
        last_upper = kv.second.upper;
        first = false;
    }
    return true;
}

}  // namespace

extern "C" moe_status moe_gran_create(moe_gran** g) {
    if (!g) return MOE_ERR_NULL;
    *g = new moe_gran();
    return MOE_OK;
}

extern "C" moe_status moe_gran_destroy(moe_gran* g) {
    delete g;
    return MOE_OK;
}

extern "C" moe_status moe_gran_lookup(moe_gran* g, int64_t B, int32_t* n) {
    if (!g || !n) return MOE_ERR_NULL;
    if (B <= 0) return MOE_ERR_SHAPE;
    auto hit = g->cache_table.find(B);
    if (hit != g->cache_table.end()) { *n = hit->second; return MOE_OK; }
    const int found = disjoint(g) ? find_n_disjoint(g, B) : find_n(g, B);
    if (found != -1) g->cache_table[B] = found;
    *n = found;
    return MOE_OK;
}

extern "C" moe_status moe_gran_record(moe_gran* g, int64_t B, int32_t n) {
    if (!g) return MOE_ERR_NULL;
    if (B <= 0 || n <= 0) return MOE_ERR_SHAPE;
    // the pair of this n: absent -> range(B, B); present -> widened to hold B
    auto it = g->by_lower.begin();
    for (; it != g->by_lower.end(); ++it)
        if (it->second.n == n) break;
    if (it == g->by_lower.end()) {
        g->by_lower[B] = moe_gran::Range{B, n};
    } else {
        const long long lower = it->first < B ? it->first : B;
        const long long upper = it->second.upper > B ? it->second.upper : B;
        g->by_lower.erase(it);
        g->by_lower[lower] = moe_gran::Range{upper, n};
    }
    g->cache_table[B] = n;
    return MOE_OK;
}

extern "C" moe_status moe_gran_ranges(const moe_gran* g, int32_t capacity, int64_t* lower, int64_t* upper,
                                      int32_t* n, int32_t* count) {
    if (!g || !count) return MOE_ERR_NULL;
    *count = (int32_t)g->by_lower.size();
    if (capacity == 0 || *count == 0) return MOE_OK;
    if (capacity < *count) return MOE_ERR_SHAPE;
    if (!lower || !upper || !n) return MOE_ERR_NULL;
    int i = 0;
    for (const auto& kv : g->by_lower) {
        lower[i] = kv.first; upper[i] = kv.second.upper; n[i] = kv.second.n;
        ++i;
    }
    return MOE_OK;
}

extern "C" moe_status moe_search_best_gran(const moe_config* cfg, const void* x, const void* dy,
                                           const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                                           void* y, void* dx, float* dWg, float* dW1, float* dW2,
                                           float* logits, int32_t* topk_idx, float* topk_w, int32_t* slot,
                                           int32_t* counts, void* workspace, size_t workspace_bytes,
                                           void* const* streams, int32_t n_streams,
                                           const int32_t* candidates, int32_t n_candidates,
                                           int32_t warmup, int32_t iters, int32_t* best_n, float* ms) {
    if (!cfg || !candidates || !best_n || !streams) return MOE_ERR_NULL;
    if (n_candidates <= 0 || iters <= 0 || warmup < 0 || n_streams < 2) return MOE_ERR_SHAPE;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return MOE_ERR_HIP; }
    hipStream_t s0 = (hipStream_t)streams[0];
    moe_status result = MOE_OK;
    float best_ms = -1.0f;
    *best_n = -1;
    for (int c = 0; c < n_candidates && result == MOE_OK; ++c) {
        if (ms) ms[c] = -1.0f;
        moe_config trial = *cfg;
        trial.n_partitions = candidates[c];
        trial.grad_overwrite = 1;                 // trials must not pile up in the gradient buffers
        size_t need = 0;
        if (moe_workspace_bytes(&trial, &need, nullptr, nullptr, nullptr) != MOE_OK) continue;   // e.g. T % n != 0
        if (need > workspace_bytes) continue;
        float elapsed = 0.0f;
        for (int it = 0; it < warmup + iters && result == MOE_OK; ++it) {
            if (it == warmup && hipEventRecord(e0, s0) != hipSuccess) { result = MOE_ERR_HIP; break; }
            result = moe_layer_step(&trial, x, dy, Wg, gate_bias, W1, W2, y, dx, dWg, dW1, dW2, logits, topk_idx,
                                    topk_w, slot, counts, workspace, workspace_bytes, streams, n_streams);
        }
        if (result != MOE_OK) break;
        if (hipEventRecord(e1, s0) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&elapsed, e0, e1) != hipSuccess) { result = MOE_ERR_HIP; break; }
        const float per_step = elapsed / (float)iters;
        if (ms) ms[c] = per_step;
        if (best_ms < 0.0f || per_step < best_ms) { best_ms = per_step; *best_n = candidates[c]; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (result != MOE_OK) return result;
    return *best_n > 0 ? MOE_OK : MOE_ERR_SHAPE;
}

extern "C" moe_status moe_gran_get(moe_gran* g, const moe_config* cfg, const void* x, const void* dy,
                                   const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                                   void* y, void* dx, float* dWg, float* dW1, float* dW2,
                                   float* logits, int32_t* topk_idx, float* topk_w, int32_t* slot,
                                   int32_t* counts, void* workspace, size_t workspace_bytes,
                                   void* const* streams, int32_t n_streams,
                                   const int32_t* candidates, int32_t n_candidates,
                                   int32_t warmup, int32_t iters, int32_t* n, int32_t* searched) {
    if (!g || !cfg || !n) return MOE_ERR_NULL;
    if (searched) *searched = 0;
    MOE_TRY(moe_gran_lookup(g, cfg->T, n));
    if (*n != -1) return MOE_OK;
    MOE_TRY(moe_search_best_gran(cfg, x, dy, Wg, gate_bias, W1, W2, y, dx, dWg, dW1, dW2, logits, topk_idx, topk_w,
                                 slot, counts, workspace, workspace_bytes, streams, n_streams, candidates,
                                 n_candidates, warmup, iters, n, nullptr));
    if (searched) *searched = 1;
    return moe_gran_record(g, cfg->T, *n);
}

// ---- performance model of the memory-reuse strategies (Section III-E) ---------------
// Eq. 7-9: per micro-batch of b tokens one GEMM is b*H*M multiply-adds, one exchange and
// one copy of T_DI are b*M elements each.  Table II: units per stream in the forward and
// in the backward pass and the slowdown factors that apply.  Eq. 10: a pass costs what its
// slowest stream takes (eta in the copy term; the first printed line shows mu there).
namespace {

struct StrategyRow { int q_fw[3]; int q_bw[3]; bool all_streams; };
// none, S1, S2, S3, S4
const StrategyRow kTableII[5] = {
    {{2, 2, 0}, {4, 2, 0}, false},
    {{2, 2, 5}, {4, 2, 5}, true},
    {{2, 2, 4}, {4, 3, 4}, true},
    {{2, 2, 1}, {5, 2, 1}, true},
    {{2, 2, 0}, {5, 3, 0}, false},
};

double pass_cost(const int q[3], double v_comp, double v_io, const moe_speeds& s, double mu, double eta) {
    const double t_comp = q[0] * v_comp / (s.sigma * s.W_comp);
    const double t_comm = q[1] * v_io / (mu * s.W_comm);
    const double t_mem = q[2] ? q[2] * v_io / (eta * s.W_mem) : 0.0;
    double c = t_comp > t_comm ? t_comp : t_comm;
    return c > t_mem ? c : t_mem;
}

bool speeds_ok(const moe_speeds* s) {
    return s->W_comp > 0 && s->W_comm > 0 && s->W_mem > 0 && s->sigma > 0 && s->mu_comp > 0 && s->mu_all > 0 &&
           s->eta_all > 0;
}

}  // namespace

extern "C" moe_status moe_strategy_cost(int32_t strategy, int64_t b, int64_t M, int64_t H, const moe_speeds* speeds,
                                        double* cost_fw, double* cost_bw) {
    if (!speeds || !cost_fw || !cost_bw) return MOE_ERR_NULL;
    if (strategy < 0 || strategy > 4 || b <= 0 || M <= 0 || H <= 0 || !speeds_ok(speeds)) return MOE_ERR_SHAPE;
    const StrategyRow& r = kTableII[strategy];
    const double v_comp = (double)b * (double)H * (double)M, v_io = (double)b * (double)M;
    const double mu = r.all_streams ? speeds->mu_all : speeds->mu_comp;
    const double eta = r.all_streams ? speeds->eta_all : 1.0;
    *cost_fw = pass_cost(r.q_fw, v_comp, v_io, *speeds, mu, eta);
    *cost_bw = pass_cost(r.q_bw, v_comp, v_io, *speeds, mu, eta);
    return MOE_OK;
}

extern "C" moe_status moe_select_strategy(uint32_t allowed_mask, int64_t b, int64_t M, int64_t H,
                                          const moe_speeds* speeds, int32_t* best, double* cost) {
    if (!speeds || !best) return MOE_ERR_NULL;
    if ((allowed_mask & 31u) == 0) return MOE_ERR_SHAPE;
    int pick = -1;
    double pick_cost = 0.0;
    for (int s = 0; s < 5; ++s) {
        if (!((allowed_mask >> s) & 1u)) continue;
        double fw, bw;
        MOE_TRY(moe_strategy_cost(s, b, M, H, speeds, &fw, &bw));
        if (pick < 0 || fw + bw < pick_cost) { pick = s; pick_cost = fw + bw; }
    }
    *best = pick;
    if (cost) *cost = pick_cost;
    return MOE_OK;
}
