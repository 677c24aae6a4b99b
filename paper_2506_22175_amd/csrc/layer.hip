// The whole layer step as n micro-batch partitions on two HIP streams, with the
// paper's memory reuse.
//
// Section III-B: the token batch is split along its batch dimension into n
// partitions; for each one S (dispatch), C (expert computation) and R (combine)
// run in that order, partitions are independent, S and R alternate on their
// stream, and backward mirrors forward.  Section III-D: T_DI and T_DO of all
// partitions share two buffers each and T_M shares one; what is overwritten is
// restored in backward by sending T_I again (here: dispatching x again) and by
// recomputing T_M from T_DI (Table II, strategy S4: 5 GEMMs and 3 exchanges in
// backward instead of 4 and 2).
//
// Stream 0 carries the gate, S, R and their backward counterparts; stream 1
// carries the GEMMs.  Cross-stream order is kept with events; a buffer shared by
// partitions p and p+2 is rewritten only after its reader of partition p is done.
#include "common.h"
#include <vector>

namespace moe {

static inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

struct Workspace {
    // M-wide partition buffers
    size_t DI, DO, dDO, dDI;          // offsets; each region holds nDI / nDO / 2 / 2 buffers
    int nDI, nDO, ndDO;
    bool dDO_aliases_DO;
    // H-wide
    size_t Z, HT;                     // Z: nZ buffers; HT: G temporaries (forward A in the first, backward dZ)
    int nZ;
    // routing-class data
    size_t slot_w, dw, dw_part, dL, gate_scratch, slot_scratch, rows;
    size_t bufM, bufH, dw_part_bytes;
    size_t total, saved, temp, routing;
};

// What each mode does with the two tensors that backward needs again (Table II).
static bool mode_recomputes(int reuse) { return reuse == MOE_REUSE_RECOMPUTE || reuse == MOE_REUSE_S3; }
static bool mode_offloads_di(int reuse) { return reuse == MOE_REUSE_S1 || reuse == MOE_REUSE_S3; }
static bool mode_offloads_z(int reuse) { return reuse == MOE_REUSE_S1 || reuse == MOE_REUSE_S2; }
static bool mode_offloads(int reuse) { return mode_offloads_di(reuse) || mode_offloads_z(reuse); }

// Host side of the offloading strategies: where each partition's copy lives, and the copy stream.
struct Offload {
    char* host = nullptr;
    size_t DI = 0, Z = 0;        // offsets in host; n buffers each (when offloaded)
    hipStream_t s2 = nullptr;
};

static moe_status plan(const moe_config* cfg, const Dims& d, Workspace* w) {
    w->bufM = align_up((size_t)d.Rp * d.M * d.es);
    w->bufH = align_up((size_t)d.Rp * d.H * d.es);
    const bool reuse = d.reuse != MOE_REUSE_NONE;
    // Partition buffers of T_DI and dT_DO that backward keeps alive: two (one being filled while the other
    // is read), or the G partitions whose weight gradients are taken in one GEMM.
    const int alive = d.G > 2 ? d.G : 2;
    // with the gathered first GEMM forward keeps no T_DI at all; backward dispatches into `alive` buffers
    w->nDI = ((reuse || d.fuse) && d.n > alive) ? alive : d.n;
    w->nDO = d.fcomb ? 0 : (reuse && d.n > alive) ? alive : d.n;     // the fused combine keeps no T_DO
    w->nZ = mode_recomputes(d.reuse) ? d.G : mode_offloads_z(d.reuse) ? (d.n < 2 ? d.n : 2) : d.n;
    w->dDO_aliases_DO = reuse && !d.fcomb;
    w->ndDO = w->dDO_aliases_DO ? w->nDO : (d.n > alive ? alive : d.n);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    w->DI = take(w->bufM * w->nDI);
    w->DO = take(w->bufM * w->nDO);
    w->Z = take(w->bufH * w->nZ);
    w->saved = off;
    w->HT = take(w->bufH * d.G);
    w->dDO = w->dDO_aliases_DO ? w->DO : take(w->bufM * w->ndDO);
    w->dDI = take(w->bufM * 2);
    w->temp = off - w->saved;
    const size_t r0 = off;
    int parts = 0;
    MOE_TRY(moe_dw_parts(cfg, &parts));
    size_t gs = 0, ss = 0;
    MOE_TRY(moe_gate_scratch_bytes(cfg, &gs));
    MOE_TRY(moe_slot_scratch_bytes(cfg, &ss));
    w->slot_w = take((size_t)d.n * d.Rp * sizeof(float));
    w->dw = take((size_t)d.T * d.k * sizeof(float));
    w->dw_part_bytes = align_up((size_t)d.Rp * parts * sizeof(float));
    w->dw_part = take(w->dw_part_bytes * 2);
    w->dL = take((size_t)d.T * d.E * sizeof(float));
    w->gate_scratch = take(gs);
    w->slot_scratch = take(ss);
    w->rows = take((d.fuse || d.fcomb) ? (size_t)d.n * d.Rp * sizeof(int) : 0);
    w->routing = off - r0;
    w->total = off;
    return MOE_OK;
}

// Events are host objects; they are created once and reused by every call.
static std::vector<hipEvent_t> g_events;
static moe_status get_events(size_t n) {
    while (g_events.size() < n) {
        hipEvent_t e;
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return MOE_ERR_HIP;
        g_events.push_back(e);
    }
    return MOE_OK;
}

// R'_p: the rows of dy of partition p to the experts (and, where forward kept no T_DI buffer for it, the
// rows of x again); with T_DO kept, the combine-weight gradients <dy_t, T_DO row> on the way.
static moe_status dispatch_for_backward(const moe_config* cfg, const Dims& d, const Workspace& w, char* ws, int p,
                                        const void* x, const void* dy, const int* slot, bool redispatch,
                                        bool dw_in_gemm, hipStream_t s0) {
    char* DI = ws + w.DI + w.bufM * (p % w.nDI);
    char* DO = w.nDO ? ws + w.DO + w.bufM * (p % w.nDO) : nullptr;
    char* dDO = ws + w.dDO + w.bufM * (p % w.ndDO);
    if (dw_in_gemm) {
        MOE_TRY(moe_dispatch(cfg, p, dy, slot, dDO, nullptr, nullptr, s0));
        if (redispatch) MOE_TRY(moe_dispatch(cfg, p, x, slot, DI, nullptr, nullptr, s0));
    } else {
        // T_DO was kept: the combine-weight gradient is <dy_t, T_DO row>
        MOE_TRY(moe_dispatch(cfg, p, dy, slot, dDO, DO, (float*)(ws + w.dw), s0));
        if (d.fuse) MOE_TRY(moe_dispatch(cfg, p, x, slot, DI, nullptr, nullptr, s0));
    }
    return MOE_OK;
}

// In a whole step R'_0 need not wait for the end of forward: what it writes (the first dT_DO buffer, the first
// T_DI buffer when x is dispatched again) was last touched by partitions before the last one, unless the last
// partition shares those buffers.  It is then queued on stream 0 ahead of the last combine, so that the first
// backward GEMM follows the last forward GEMM without a gap.
static bool first_backward_dispatch_can_go_early(const Dims& d, const Workspace& w, bool offload) {
    if (d.n < 2 || offload) return false;
    const bool redispatch = w.nDI < d.n || d.fuse;
    if (w.dDO_aliases_DO && (d.n - 1) % w.nDO == 0) return false;
    if (redispatch && !d.fuse && (d.n - 1) % w.nDI == 0) return false;
    return true;
}

static moe_status forward(const moe_config* cfg, const Dims& d, const Workspace& w, char* ws,
                          const void* x, const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                          void* y, float* logits, int* topk_idx, float* topk_w, int* slot, int* counts,
                          hipStream_t s0, hipStream_t s1, const Offload* off = nullptr, const void* dy_early = nullptr) {
    const int n = d.n;
    MOE_TRY(get_events(7 * (size_t)n + 2));
    hipEvent_t* evS = g_events.data();
    hipEvent_t* evC = evS + n;
    hipEvent_t* evR = evC + n;
    hipEvent_t* evDIout = evR + n;            // T_DI of p is on the host
    hipEvent_t* evZout = evDIout + n;         // T_M of p is on the host
    hipEvent_t evFork = g_events[7 * (size_t)n];
    hipEvent_t evCopies = g_events[7 * (size_t)n + 1];
    const bool off_di = off && mode_offloads_di(d.reuse), off_z = off && mode_offloads_z(d.reuse);

    MOE_TRY(moe_route(cfg, x, Wg, gate_bias, logits, topk_idx, topk_w, s0));
    MOE_TRY(moe_assign_slots(cfg, topk_idx, topk_w, slot, counts, (float*)(ws + w.slot_w),
                             ws + w.slot_scratch, s0));
    const int* rows = (d.fuse || d.fcomb) ? (const int*)(ws + w.rows) : nullptr;
    if (rows) MOE_TRY(moe_slot_rows(cfg, slot, (int*)(ws + w.rows), s0));
    if (d.fcomb) MOE_TRY(zero_dropped(d, slot, y, s0));
    HIP_TRY(hipEventRecord(evFork, s0));
    HIP_TRY(hipStreamWaitEvent(s1, evFork, 0));

    auto DIbuf = [&](int p) { return ws + w.DI + w.bufM * (p % w.nDI); };
    auto DObuf = [&](int p) { return w.nDO ? ws + w.DO + w.bufM * (p % w.nDO) : nullptr; };
    auto Zbuf = [&](int p) { return ws + w.Z + w.bufH * (p % w.nZ); };
    const bool keepZ = !mode_recomputes(d.reuse);

    for (int p = 0; p <= n; ++p) {
        if (p < n) {
            // S_p.  A shared T_DI buffer was last read by C_{p-2}; R_{p-2}, already
            // queued on this stream, waited for C_{p-2}.  Its copy to the host must be through too.
            if (off_di && p >= w.nDI) HIP_TRY(hipStreamWaitEvent(s0, evDIout[p - w.nDI], 0));
            // (with the gathered first GEMM there is no S kernel: C_p reads T_I through the row map)
            if (!d.fuse) MOE_TRY(moe_dispatch(cfg, p, x, slot, DIbuf(p), nullptr, nullptr, s0));
            HIP_TRY(hipEventRecord(evS[p], s0));
            if (off_di) {
                HIP_TRY(hipStreamWaitEvent(off->s2, evS[p], 0));
                HIP_TRY(hipMemcpyAsync(off->host + off->DI + w.bufM * p, DIbuf(p), w.bufM, hipMemcpyDeviceToHost, off->s2));
                HIP_TRY(hipEventRecord(evDIout[p], off->s2));
            }
            // C_p
            HIP_TRY(hipStreamWaitEvent(s1, evS[p], 0));
            if (w.nDO && p >= w.nDO) HIP_TRY(hipStreamWaitEvent(s1, evR[p - w.nDO], 0));   // T_DO buffer free again
            if (off_z && p >= w.nZ) HIP_TRY(hipStreamWaitEvent(s1, evZout[p - w.nZ], 0));   // T_M buffer copied out
            // with recomputation T_M is not kept: the activated rows go to the one
            // shared H-wide buffer and the pre-activation is not written at all
            void* Aout = keepZ ? (void*)(ws + w.HT) : (void*)Zbuf(p);
            MOE_TRY(ffn_fwd(d, p, d.fuse ? x : (const void*)DIbuf(p), d.fuse ? rows : nullptr, counts, W1, W2,
                            keepZ ? Zbuf(p) : nullptr, Aout, DObuf(p), s1,
                            d.fcomb ? rows : nullptr, (const float*)(ws + w.slot_w), y));
            HIP_TRY(hipEventRecord(evC[p], s1));
            if (off_z) {
                HIP_TRY(hipStreamWaitEvent(off->s2, evC[p], 0));
                HIP_TRY(hipMemcpyAsync(off->host + off->Z + w.bufH * p, Zbuf(p), w.bufH, hipMemcpyDeviceToHost, off->s2));
                HIP_TRY(hipEventRecord(evZout[p], off->s2));
            }
        }
        if (p >= 1) {
            // R_{p-1}, issued after S_p so that S and R alternate on stream 0 (with the fused combine
            // C_{p-1} has written y itself and stream 0 only waits for it)
            if (p == n && dy_early) {
                // whole step: R'_0 of backward goes first (see first_backward_dispatch_can_go_early); backward
                // finds its event recorded
                const bool reuse = d.reuse != MOE_REUSE_NONE;
                MOE_TRY(dispatch_for_backward(cfg, d, w, ws, 0, x, dy_early, slot, w.nDI < n || d.fuse, reuse || d.fcomb, s0));
                HIP_TRY(hipEventRecord(evS[0], s0));
            }
            HIP_TRY(hipStreamWaitEvent(s0, evC[p - 1], 0));
            if (!d.fcomb) MOE_TRY(moe_combine(cfg, p - 1, DObuf(p - 1), slot, topk_w, y, s0));
            HIP_TRY(hipEventRecord(evR[p - 1], s0));
        }
    }
    if (off_di || off_z) {                       // the host copies belong to what stream 0 has finished
        HIP_TRY(hipEventRecord(evCopies, off->s2));
        HIP_TRY(hipStreamWaitEvent(s0, evCopies, 0));
    }
    return MOE_OK;
}

static moe_status backward(const moe_config* cfg, const Dims& d, const Workspace& w, char* ws,
                           const void* x, const void* dy, const void* Wg, const void* W1, const void* W2,
                           void* dx, float* dWg, float* dW1, float* dW2,
                           const float* logits, const int* topk_idx, const int* slot, const int* counts,
                           hipStream_t s0, hipStream_t s1, const Offload* off = nullptr, bool first_dispatch_done = false) {
    const int n = d.n, G = d.G;
    MOE_TRY(get_events(7 * (size_t)n + 2));
    hipEvent_t* evS = g_events.data();        // R'_p done (rows of dy, and of x again, are in place)
    hipEvent_t* evC = evS + n;                // backward GEMMs of p done, weight gradients apart
    hipEvent_t* evD = evC + n;                // S'_p done (dDI and dw_part of p consumed)
    hipEvent_t* evIn = evD + n;               // T_DI / T_M of p are back from the host
    hipEvent_t* evW = evIn + n;               // weight gradients of group g done
    hipEvent_t evFork = g_events[7 * (size_t)n];
    const bool reuse = d.reuse != MOE_REUSE_NONE;
    // the combine-weight gradient: from the kept T_DO, or (T_DO overwritten or never written) from the
    // GeLU-backward GEMM's row dots
    const bool dw_in_gemm = reuse || d.fcomb;
    const bool recompute = mode_recomputes(d.reuse);
    const bool off_di = off && mode_offloads_di(d.reuse), off_z = off && mode_offloads_z(d.reuse);

    auto DIbuf = [&](int p) { return ws + w.DI + w.bufM * (p % w.nDI); };
    auto DObuf = [&](int p) { return w.nDO ? ws + w.DO + w.bufM * (p % w.nDO) : nullptr; };
    auto Zbuf = [&](int p) { return ws + w.Z + w.bufH * (p % w.nZ); };
    auto dZbuf = [&](int p) { return ws + w.HT + w.bufH * (p % G); };
    auto dDObuf = [&](int p) { return ws + w.dDO + w.bufM * (p % w.ndDO); };
    auto dDIbuf = [&](int p) { return ws + w.dDI + w.bufM * (p % 2); };
    auto dwpart = [&](int p) { return (float*)(ws + w.dw_part + w.dw_part_bytes * (p % 2)); };
    float* dw = (float*)(ws + w.dw);
    float* dL = (float*)(ws + w.dL);
    const float* slot_w = (const float*)(ws + w.slot_w);
    // forward left T_DI of every partition in place unless buffers are shared or it never wrote any
    const bool redispatch = !off_di && (w.nDI < n || d.fuse);

    HIP_TRY(hipEventRecord(evFork, s0));
    // (whole step with R'_0 already queued: the GEMM stream goes straight on from forward's last GEMM; what its
    // first backward GEMMs touch is ordered by R'_0's event and by the stream itself)
    if (!first_dispatch_done) HIP_TRY(hipStreamWaitEvent(s1, evFork, 0));
    // copies back into the shared buffers must not overtake the forward GEMMs that still read them
    if (off_di || off_z) HIP_TRY(hipStreamWaitEvent(off->s2, evFork, 0));

    for (int p = 0; p <= n; ++p) {
        if (p < n && !(p == 0 && first_dispatch_done)) {
            // R'_p: rows of dy to the experts.  Their buffer (and the re-dispatched T_DI buffer) was last
            // read by partition p - (number of buffers): by its GEMMs and by the weight-gradient GEMMs of
            // its group, which come last.
            if (p >= w.ndDO) HIP_TRY(hipStreamWaitEvent(s0, evW[(p - w.ndDO) / G], 0));
            if (redispatch && p >= w.nDI && w.nDI != w.ndDO) HIP_TRY(hipStreamWaitEvent(s0, evW[(p - w.nDI) / G], 0));
            MOE_TRY(dispatch_for_backward(cfg, d, w, ws, p, x, dy, slot, redispatch, dw_in_gemm, s0));
            HIP_TRY(hipEventRecord(evS[p], s0));
        }
        if (p < n) {
            if (off_di || off_z) {
                // what was offloaded comes back into the shared buffers, last read by the GEMMs of p-2
                // (the copy stream runs in order, so the forward copies are through)
                if (p >= 2) HIP_TRY(hipStreamWaitEvent(off->s2, evW[p - 2], 0));
                if (off_di)
                    HIP_TRY(hipMemcpyAsync(DIbuf(p), off->host + off->DI + w.bufM * p, w.bufM, hipMemcpyHostToDevice, off->s2));
                if (off_z)
                    HIP_TRY(hipMemcpyAsync(Zbuf(p), off->host + off->Z + w.bufH * p, w.bufH, hipMemcpyHostToDevice, off->s2));
                HIP_TRY(hipEventRecord(evIn[p], off->s2));
                HIP_TRY(hipStreamWaitEvent(s1, evIn[p], 0));
            }
            // C'_p: everything but the weight gradients
            HIP_TRY(hipStreamWaitEvent(s1, evS[p], 0));
            if (p >= 2) HIP_TRY(hipStreamWaitEvent(s1, evD[p - 2], 0));
            MOE_TRY(ffn_bwd_main(d, p, recompute ? 1 : 0, DIbuf(p), Zbuf(p), dDObuf(p), counts, slot_w, W1, W2,
                                 dZbuf(p), dDIbuf(p), dw_in_gemm ? dwpart(p) : nullptr, s1));
            HIP_TRY(hipEventRecord(evC[p], s1));
            // the weight gradients of a whole group after its last partition (Section III-B's per-partition
            // schedule when G = 1)
            if (p % G == G - 1 || p == n - 1) {
                const int p0 = p / G * G;
                MOE_TRY(ffn_wgrad(d, p0, p - p0 + 1, d.overwrite && p0 == 0, DIbuf(p0), Zbuf(p0), dDObuf(p0), dZbuf(p0),
                                  (long long)(w.bufM / d.es), (long long)(w.bufH / d.es), counts, dW1, dW2, s1));
                HIP_TRY(hipEventRecord(evW[p / G], s1));
            }
        }
        if (p >= 1) {
            // S'_{p-1}: gate backward and rows of dDI back to token order
            const int q = p - 1;
            HIP_TRY(hipStreamWaitEvent(s0, evC[q], 0));
            MOE_TRY(moe_gate_bwd(cfg, q, x, logits, topk_idx, slot, dw_in_gemm ? nullptr : dw,
                                 dw_in_gemm ? dwpart(q) : nullptr, dL, dWg, ws + w.gate_scratch, s0));
            MOE_TRY(moe_dispatch_bwd(cfg, q, dDIbuf(q), slot, dL, Wg, dx, s0));
            HIP_TRY(hipEventRecord(evD[q], s0));
        }
    }
    HIP_TRY(hipStreamWaitEvent(s0, evW[(n - 1) / G], 0));      // the last weight gradients belong to the step
    return MOE_OK;
}

static moe_status setup(const moe_config* cfg, Dims* d, Workspace* w, void* workspace, size_t workspace_bytes,
                        void* const* streams, int n_streams, hipStream_t* s0, hipStream_t* s1,
                        bool with_host = false) {
    MOE_TRY(make_dims(cfg, d));
    if (!workspace || !streams) return MOE_ERR_NULL;
    if (n_streams < 2) return MOE_ERR_SHAPE;
    if (mode_offloads(d->reuse) != with_host) return MOE_ERR_UNSUPPORTED;
    MOE_TRY(plan(cfg, *d, w));
    if (workspace_bytes < w->total) return MOE_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 255) != 0) return MOE_ERR_WORKSPACE;
    *s0 = (hipStream_t)streams[0];
    *s1 = (hipStream_t)streams[1];
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" moe_status moe_workspace_bytes(const moe_config* cfg, size_t* total, size_t* saved,
                                          size_t* temp, size_t* routing) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    Workspace w;
    MOE_TRY(plan(cfg, d, &w));
    if (total) *total = w.total;
    if (saved) *saved = w.saved;
    if (temp) *temp = w.temp;
    if (routing) *routing = w.routing;
    return MOE_OK;
}

extern "C" moe_status moe_layer_forward(const moe_config* cfg, const void* x,
                                        const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                                        void* y, float* logits, int32_t* topk_idx, float* topk_w,
                                        int32_t* slot, int32_t* counts,
                                        void* workspace, size_t workspace_bytes,
                                        void* const* streams, int32_t n_streams) {
    Dims d; Workspace w; hipStream_t s0, s1;
    MOE_TRY(setup(cfg, &d, &w, workspace, workspace_bytes, streams, n_streams, &s0, &s1));
    if (!x || !Wg || !W1 || !W2 || !y || !logits || !topk_idx || !topk_w || !slot || !counts) return MOE_ERR_NULL;
    return forward(cfg, d, w, (char*)workspace, x, Wg, gate_bias, W1, W2, y, logits, topk_idx, topk_w, slot,
                   counts, s0, s1);
}

extern "C" moe_status moe_layer_backward(const moe_config* cfg, const void* x, const void* dy,
                                         const void* Wg, const void* W1, const void* W2,
                                         void* dx, float* dWg, float* dW1, float* dW2,
                                         const float* logits, const int32_t* topk_idx, const float* topk_w,
                                         const int32_t* slot, const int32_t* counts,
                                         void* workspace, size_t workspace_bytes,
                                         void* const* streams, int32_t n_streams) {
    Dims d; Workspace w; hipStream_t s0, s1;
    MOE_TRY(setup(cfg, &d, &w, workspace, workspace_bytes, streams, n_streams, &s0, &s1));
    if (!x || !dy || !Wg || !W1 || !W2 || !dx || !dWg || !dW1 || !dW2 || !logits || !topk_idx || !topk_w ||
        !slot || !counts) return MOE_ERR_NULL;
    return backward(cfg, d, w, (char*)workspace, x, dy, Wg, W1, W2, dx, dWg, dW1, dW2, logits, topk_idx, slot,
                    counts, s0, s1);
}

extern "C" moe_status moe_layer_step(const moe_config* cfg, const void* x, const void* dy,
                                     const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                                     void* y, void* dx, float* dWg, float* dW1, float* dW2,
                                     float* logits, int32_t* topk_idx, float* topk_w, int32_t* slot, int32_t* counts,
                                     void* workspace, size_t workspace_bytes,
                                     void* const* streams, int32_t n_streams) {
    Dims d; Workspace w; hipStream_t s0, s1;
    MOE_TRY(setup(cfg, &d, &w, workspace, workspace_bytes, streams, n_streams, &s0, &s1));
    if (!x || !dy || !Wg || !W1 || !W2 || !y || !dx || !dWg || !dW1 || !dW2 || !logits || !topk_idx ||
        !topk_w || !slot || !counts) return MOE_ERR_NULL;
    const bool early = first_backward_dispatch_can_go_early(d, w, false);
    MOE_TRY(forward(cfg, d, w, (char*)workspace, x, Wg, gate_bias, W1, W2, y, logits, topk_idx, topk_w, slot,
                    counts, s0, s1, nullptr, early ? dy : nullptr));
    return backward(cfg, d, w, (char*)workspace, x, dy, Wg, W1, W2, dx, dWg, dW1, dW2, logits, topk_idx, slot,
                    counts, s0, s1, nullptr, early);
}

static void offload_layout(const Dims& d, const Workspace& w, Offload* o, size_t* total) {
    size_t off = 0;
    o->DI = off;
    if (mode_offloads_di(d.reuse)) off += w.bufM * (size_t)d.n;
    o->Z = off;
    if (mode_offloads_z(d.reuse)) off += w.bufH * (size_t)d.n;
    *total = off;
}

extern "C" moe_status moe_offload_bytes(const moe_config* cfg, size_t* host_bytes) {
    Dims d;
    MOE_TRY(make_dims(cfg, &d));
    if (!host_bytes) return MOE_ERR_NULL;
    if (!mode_offloads(d.reuse)) return MOE_ERR_UNSUPPORTED;
    Workspace w;
    MOE_TRY(plan(cfg, d, &w));
    Offload o;
    offload_layout(d, w, &o, host_bytes);
    return MOE_OK;
}

extern "C" moe_status moe_layer_step_offload(const moe_config* cfg, const void* x, const void* dy,
                                             const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                                             void* y, void* dx, float* dWg, float* dW1, float* dW2,
                                             float* logits, int32_t* topk_idx, float* topk_w, int32_t* slot,
                                             int32_t* counts, void* workspace, size_t workspace_bytes,
                                             void* host_buffer, size_t host_bytes,
                                             void* const* streams, int32_t n_streams) {
    Dims d; Workspace w; hipStream_t s0, s1;
    if (n_streams < 3) return streams ? MOE_ERR_SHAPE : MOE_ERR_NULL;
    MOE_TRY(setup(cfg, &d, &w, workspace, workspace_bytes, streams, n_streams, &s0, &s1, true));
    if (!x || !dy || !Wg || !W1 || !W2 || !y || !dx || !dWg || !dW1 || !dW2 || !logits || !topk_idx ||
        !topk_w || !slot || !counts || !host_buffer) return MOE_ERR_NULL;
    Offload o;
    size_t need = 0;
    offload_layout(d, w, &o, &need);
    if (host_bytes < need) return MOE_ERR_WORKSPACE;
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, host_buffer) != hipSuccess || attr.type != hipMemoryTypeHost) {
        (void)hipGetLastError();
        return MOE_ERR_UNSUPPORTED;               // pageable memory would make the copies synchronous
    }
    o.host = (char*)host_buffer;
    o.s2 = (hipStream_t)streams[2];
    MOE_TRY(forward(cfg, d, w, (char*)workspace, x, Wg, gate_bias, W1, W2, y, logits, topk_idx, topk_w, slot,
                    counts, s0, s1, &o));
    return backward(cfg, d, w, (char*)workspace, x, dy, Wg, W1, W2, dx, dWg, dW1, dW2, logits, topk_idx, slot,
                    counts, s0, s1, &o);
}
