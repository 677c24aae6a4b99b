// Host-side helpers: configuration checks, capacity, launch counters.
#include "common.h"
#include <atomic>
#include <cmath>
#include <cstdio>
#include <vector>

namespace moe {

moe_status make_dims(const moe_config* cfg, Dims* d) {
    if (!cfg || !d) return MOE_ERR_NULL;
    if (cfg->T <= 0 || cfg->M <= 0 || cfg->H <= 0 || cfg->E <= 0 || cfg->k <= 0) return MOE_ERR_SHAPE;
    if (cfg->k > cfg->E) return MOE_ERR_SHAPE;
    if (!(cfg->capacity_factor > 0.0f) || !std::isfinite(cfg->capacity_factor)) return MOE_ERR_SHAPE;
    if (cfg->n_partitions <= 0 || cfg->T % cfg->n_partitions != 0) return MOE_ERR_SHAPE;
    if (cfg->dtype != MOE_F32 && cfg->dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
    if (cfg->reuse < MOE_REUSE_NONE || cfg->reuse > MOE_REUSE_S3) return MOE_ERR_UNSUPPORTED;
    if (cfg->E > 64 || cfg->k > 8 || cfg->n_partitions > 64) return MOE_ERR_UNSUPPORTED;
    if (cfg->M % 8 != 0 || cfg->H % 8 != 0) return MOE_ERR_UNSUPPORTED;
    d->T = cfg->T; d->M = cfg->M; d->H = cfg->H; d->E = cfg->E; d->k = cfg->k;
    d->n = cfg->n_partitions; d->Tp = cfg->T / cfg->n_partitions;
    double c = std::ceil((double)cfg->capacity_factor * (double)((long long)cfg->k * d->Tp) / (double)cfg->E);
    if (c < 1.0) c = 1.0;
    if (c * (double)cfg->E > 2.0e9) return MOE_ERR_SHAPE;
    d->Cp = (int)c;
    d->Rp = d->Cp * d->E;
    d->dtype = cfg->dtype; d->reuse = cfg->reuse;
    d->overwrite = cfg->grad_overwrite != 0;
    d->renorm = cfg->gate_renormalize != 0;
    if (cfg->fuse_gather != 0 && cfg->fuse_gather != 1) return MOE_ERR_UNSUPPORTED;
    if (cfg->fuse_gather && (cfg->reuse == MOE_REUSE_S1 || cfg->reuse == MOE_REUSE_S3)) return MOE_ERR_UNSUPPORTED;
    d->fuse = cfg->fuse_gather;
    if (cfg->wgrad_group < 0 || cfg->wgrad_group > 8) return MOE_ERR_UNSUPPORTED;
    d->G = cfg->wgrad_group < 1 ? 1 : (cfg->wgrad_group > d->n ? d->n : cfg->wgrad_group);
    if (d->G > 1 && cfg->reuse > MOE_REUSE_RECOMPUTE) return MOE_ERR_UNSUPPORTED;   // not with the offloading strategies
    if (cfg->fuse_combine != 0 && cfg->fuse_combine != 1) return MOE_ERR_UNSUPPORTED;
    if (cfg->fuse_combine && (cfg->k != 1 || cfg->reuse > MOE_REUSE_RECOMPUTE)) return MOE_ERR_UNSUPPORTED;
    d->fcomb = cfg->fuse_combine;
    if (cfg->gemm_free_cus < 0 || cfg->gemm_free_cus > 1024) return MOE_ERR_UNSUPPORTED;
    d->free_cus = cfg->gemm_free_cus;
    d->es = cfg->dtype == MOE_F32 ? 4 : 2;
    return MOE_OK;
}

moe_status check_part(const Dims& d, int part) {
    return (part < 0 || part >= d.n) ? MOE_ERR_SHAPE : MOE_OK;
}

static char g_last_error[512] = "";
void note_hip_error(hipError_t e, const char* file, int line) {
    snprintf(g_last_error, sizeof(g_last_error), "%s (%d) at %s:%d", hipGetErrorString(e), (int)e, file, line);
}

static std::atomic<long long> g_launches[3];
void count_launch(LaunchClass c, int n) { g_launches[c].fetch_add(n, std::memory_order_relaxed); }

// ---- optional kernel timing ---------------------------------------------------------
struct ProfRec { int kind; hipEvent_t a, b; };
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof_recs;      // records of the current session
static std::vector<hipEvent_t> g_prof_pool;   // timing events, reused across sessions
static size_t g_prof_pool_used = 0;
static const size_t PROF_MAX_RECS = 1u << 16;

static bool prof_event(hipEvent_t* e) {
    if (g_prof_pool_used == g_prof_pool.size()) {
        hipEvent_t n;
        if (hipEventCreate(&n) != hipSuccess) return false;
        g_prof_pool.push_back(n);
    }
    *e = g_prof_pool[g_prof_pool_used++];
    return true;
}

ProfScope::ProfScope(int kind, hipStream_t stream) : idx(-1), s(stream) {
    if (!g_prof_on || g_prof_recs.size() >= PROF_MAX_RECS) return;
    ProfRec r;
    r.kind = kind;
    if (!prof_event(&r.a) || !prof_event(&r.b)) return;
    if (hipEventRecord(r.a, s) != hipSuccess) return;
    idx = (int)g_prof_recs.size();
    g_prof_recs.push_back(r);
}
ProfScope::~ProfScope() {
    if (idx >= 0) (void)hipEventRecord(g_prof_recs[idx].b, s);
}

}  // namespace moe

extern "C" moe_status moe_profile_enable(int32_t on) {
    moe::g_prof_on = on != 0;
    if (on) { moe::g_prof_recs.clear(); moe::g_prof_pool_used = 0; }
    return MOE_OK;
}

extern "C" moe_status moe_profile_read(int32_t kinds, int64_t* launches, double* total_ms) {
    if (!launches || !total_ms) return MOE_ERR_NULL;
    for (int i = 0; i < kinds; ++i) { launches[i] = 0; total_ms[i] = 0.0; }
    for (const moe::ProfRec& r : moe::g_prof_recs) {
        if (r.kind >= kinds) continue;
        HIP_TRY(hipEventSynchronize(r.b));
        float ms = 0.0f;
        HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
        launches[r.kind] += 1;
        total_ms[r.kind] += ms;
    }
    return MOE_OK;
}

extern "C" moe_status moe_capacity(const moe_config* cfg, int32_t* C_p) {
    moe::Dims d;
    MOE_TRY(moe::make_dims(cfg, &d));
    if (!C_p) return MOE_ERR_NULL;
    *C_p = d.Cp;
    return MOE_OK;
}

extern "C" moe_status moe_launch_counts(int64_t out[3], int32_t reset) {
    if (!out) return MOE_ERR_NULL;
    for (int i = 0; i < 3; ++i) {
        out[i] = moe::g_launches[i].load();
        if (reset) moe::g_launches[i].store(0);
    }
    return MOE_OK;
}

extern "C" const char* moe_last_error(void) { return moe::g_last_error; }

extern "C" const char* moe_status_string(moe_status s) {
    switch (s) {
        case MOE_OK: return "ok";
        case MOE_ERR_NULL: return "required pointer is NULL";
        case MOE_ERR_SHAPE: return "invalid shape or partition";
        case MOE_ERR_UNSUPPORTED: return "unsupported configuration";
        case MOE_ERR_WORKSPACE: return "workspace too small";
        case MOE_ERR_HIP: return "HIP call failed";
    }
    return "unknown status";
}
