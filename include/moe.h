/*
 * C ABI of the MI355X (gfx950) MoE-layer hot path.
 *
 * One GPU's share of a Mixture-of-Experts layer's training step: gate ->
 * capacity-bounded dispatch -> per-expert FFN (linear, GeLU, linear) ->
 * weighted combine, forward and backward, run as n micro-batch partitions on
 * HIP streams with optional sharing of partition buffers and recomputation of
 * the middle activation (MPipeMoE, Sections II-A, II-B2, III-B, III-D).
 *
 * Conventions for every call unless stated otherwise
 *   - every pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates, frees or keeps device memory (the config and the size queries
 *     are host memory);
 *   - tensors are dense, row-major, 16-byte aligned; element type `dtype` is
 *     MOE_F32 (float) or MOE_BF16 (bfloat16 bit patterns) for x, dy, y, dx, Wg,
 *     W1, W2 and all activation buffers; logits, combine weights and weight
 *     gradients are always float; indices are int32;
 *   - `stream` is a hipStream_t passed as void*; calls are asynchronous and
 *     stream-ordered;
 *   - the return value is a moe_status; nothing throws or aborts.
 *       MOE_ERR_NULL        a required pointer is NULL
 *       MOE_ERR_SHAPE       non-positive dimension, k > E, T % n != 0, cf <= 0,
 *                           partition index out of range
 *       MOE_ERR_UNSUPPORTED E > 64, k > 8, n > 64, M % 8 != 0, H % 8 != 0, unknown dtype or
 *                           reuse mode, a reuse mode the entry point does not serve
 *       MOE_ERR_WORKSPACE   workspace smaller than moe_workspace_bytes(), or not
 *                           256-byte aligned
 *       MOE_ERR_HIP         a HIP call or kernel launch failed
 *   - notation: T tokens, M model dim, H expert hidden dim, E local experts,
 *     k experts per token, n partitions, T_p = T/n, C_p = rows per expert per
 *     partition, R_p = E*C_p rows of one partition's expert-contiguous buffers.
 *   - rows of a partition buffer at or beyond counts[p][e] inside expert e's
 *     C_p-row segment are padding: never read as data, contents unspecified.
 *   - host-side state (a pool of events, the launch counters, the timing
 *     records) is process-wide and unsynchronised: call the library from one
 *     host thread at a time.  Calls on different streams may overlap on the GPU;
 *     the bf16 GEMMs launch one persistent workgroup per CU, so two GEMMs that
 *     overlap share the CUs by whole workgroups.
 */
#ifndef MOE_H
#define MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0, MOE_ERR_NULL = 1, MOE_ERR_SHAPE = 2, MOE_ERR_UNSUPPORTED = 3,
    MOE_ERR_WORKSPACE = 4, MOE_ERR_HIP = 5
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

/* Memory-reuse modes (Section III-D, Table II).
 *   NONE      every partition's T_DI, T_M, T_DO is kept for backward (row "none").
 *   BUFFERS   T_DI and T_DO live in two partition-sized buffers each; T_DI is
 *             re-dispatched from T_I in backward; T_M is kept whole.
 *   RECOMPUTE as BUFFERS, and T_M lives in one partition-sized buffer and is
 *             recomputed from T_DI in backward (strategy S4 with the
 *             re-communication read as a local re-dispatch).
 *   S1, S2, S3  the offloading strategies of Table II, for moe_layer_step_offload
 *             only: shared T_DI/T_DO buffers as in BUFFERS, and in forward T_DI (S1,
 *             S3) and/or T_M (S1, S2) of every partition are copied to pinned host
 *             memory on a third stream and copied back before the partition's
 *             backward GEMMs; S2 re-dispatches T_DI, S3 recomputes T_M.  T_M then
 *             lives in two partition-sized buffers (one being copied while the next
 *             is written), one for S3. */
typedef enum { MOE_REUSE_NONE = 0, MOE_REUSE_BUFFERS = 1, MOE_REUSE_RECOMPUTE = 2,
               MOE_REUSE_S1 = 3, MOE_REUSE_S2 = 4, MOE_REUSE_S3 = 5 } moe_reuse;

typedef struct {
    int32_t T, M, H, E, k;
    float capacity_factor;
    int32_t n_partitions;
    int32_t dtype;   /* moe_dtype */
    int32_t reuse;   /* moe_reuse */
    int32_t grad_overwrite; /* 0: dWg, dW1, dW2 are accumulated into (caller zeroes them);
                               1: calls for partition 0 store, calls for later partitions
                               accumulate, so one pass over partitions 0..n-1 leaves the
                               gradients of this step whatever the buffers held before */
    int32_t gate_renormalize; /* 0: combine weights are the chosen softmax probabilities
                               (what the paper's k = 1 gate implies); 1: they are divided
                               by their sum over the token's k choices, drops included
                               (a softmax over the chosen logits only) */
    int32_t fuse_gather;    /* 0: forward dispatches T_I into T_DI and the first expert GEMM
                               reads T_DI; 1: in forward the first expert GEMM reads its rows
                               straight from T_I through the slot-to-token map, so forward runs
                               no S kernel and writes no T_DI (one permutation unit per
                               micro-batch instead of Table II's two); backward dispatches T_I
                               into two partition-sized T_DI buffers for the weight-gradient
                               GEMM, as the shared-buffer modes do.  Not with S1 and S3, which
                               copy forward's T_DI to the host. */
    int32_t wgrad_group;    /* 0 or 1: backward runs the two weight-gradient GEMMs once per partition
                               (Table II's schedule).  G in 2..8: once per G consecutive partitions,
                               reducing over all their rows in one GEMM, so the float gradients are
                               read and written n/G times per step instead of n times; the price is
                               G partition-sized buffers each of T_DI, dT_DO, T_M and dT_M alive in
                               backward instead of two (one for T_M, dT_M).  Values above n count as
                               n.  Not with S1..S3. */
    int32_t gemm_free_cus;  /* The bfloat16 expert GEMMs launch one persistent workgroup per compute unit,
                               which leaves no room for a kernel of another stream until a GEMM ends.
                               r > 0 launches them on r compute units fewer (rounded up to a multiple of 8,
                               at least 8 stay), so that the permutation kernels of Section III-B's other
                               stream run beside them on the units left free.  0: every unit. */
    int32_t fuse_combine;   /* 1 (only with k = 1, the paper's own gate, Section IV-A): the second expert
                               GEMM writes each kept row, times its combine weight, straight into its
                               token's row of y, and the rows of dropped tokens are zeroed beforehand.
                               Forward then runs no R kernel and keeps no T_DO (with fuse_gather: two
                               GEMMs and no permutation per micro-batch); backward takes the
                               combine-weight gradient in the GeLU-backward GEMM in every mode.  Not with
                               S1..S3. */
} moe_config;

/* Host only.  C_p = ceil(capacity_factor * k * (T / n) / E), evaluated in double
 * from the float capacity_factor.  (The paper has no capacity; each micro-batch
 * of Section III-B is treated as an independent MoE call, so the bound is per
 * partition and buffers are exactly 1/n of the whole.) */
moe_status moe_capacity(const moe_config* cfg, int32_t* C_p);

/* Host only.  Bytes of the workspace moe_layer_step needs for cfg, and how they
 * split: `saved` = activations kept from forward for backward (T_DI, T_M, T_DO
 * in the sense of Eq. 2 / Eq. 4), `temp` = forward/backward temporaries (Eq. 3),
 * `routing` = slot weights, gate gradients, partial sums.  Any output pointer
 * may be NULL. */
moe_status moe_workspace_bytes(const moe_config* cfg, size_t* total, size_t* saved,
                               size_t* temp, size_t* routing);

/* Gate (Sections II-B2, IV-A): logits = x Wg (+ gate_bias) in float with a fixed
 * summation order (element d goes to accumulator (d/8) mod 64, fused
 * multiply-adds in ascending d, then pairwise folding with offsets 32..1, bias
 * added last); softmax over all E; the k largest logits, ties to the lower
 * index, NaN ordered as -inf; topk_w are the chosen probabilities.
 *   x [T,M], Wg [M,E] in dtype; gate_bias [E] float, may be NULL;
 *   logits [T,E] float out; topk_idx [T,k] int32 out; topk_w [T,k] float out. */
moe_status moe_route(const moe_config* cfg, const void* x, const void* Wg, const float* gate_bias,
                     float* logits, int32_t* topk_idx, float* topk_w, void* stream);

/* Capacity-bounded slot assignment for all n partitions.  Inside a partition,
 * positions are granted choice-major (all first choices in token order, then
 * second choices, ...); an assignment whose position reaches C_p is dropped.
 *   slot [T,k] int32 out: partition-local row e*C_p + pos, or -1 if dropped;
 *   counts [n,E] int32 out: kept rows per expert;
 *   slot_w [n*R_p] float out, may be NULL: combine weight of the assignment that
 *   owns each kept row (padding rows are not written);
 *   scratch: at least moe_slot_scratch_bytes(cfg) bytes. */
moe_status moe_assign_slots(const moe_config* cfg, const int32_t* topk_idx, const float* topk_w,
                            int32_t* slot, int32_t* counts, float* slot_w,
                            void* scratch, void* stream);
moe_status moe_slot_scratch_bytes(const moe_config* cfg, size_t* bytes);

/* moe_assign_slots for callers that cannot allocate device memory or size a scratch
 * buffer themselves (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): same arguments without `scratch`, same results bit for bit.  The
 * histograms live in a 256 KiB array that the library holds on every GPU it runs on
 * until the process ends; the call allocates and frees nothing.
 *   moe_slot_scratch_bytes(cfg) > 256 KiB (that is n*k*ceil(T_p/1024)*E > 65536):
 *   MOE_ERR_WORKSPACE, nothing is launched.
 *   The first call on a device looks up the array's address on that device (make it
 *   outside stream capture).  Every call on a GPU uses that GPU's one array: calls
 *   that overlap in time on one GPU (different streams, or graphs replayed side by
 *   side) race; serialise them.  Nothing needs clearing between calls. */
moe_status moe_assign_slots_static(const moe_config* cfg, const int32_t* topk_idx, const float* topk_w,
                                   int32_t* slot, int32_t* counts, float* slot_w, void* stream);

/* Dispatch S of partition `part` (Fig. 1: T_I -> T_DI; on one GPU the All-to-All
 * is a local permutation): DI[slot[t,j]] = src[t] for every kept (t, j) of the
 * partition's tokens.  src [T,M] (x, or dy in backward); DI [R_p,M] out.
 * If dO_saved and dw are non-NULL also dw[t,j] = <src[t], dO_saved[slot[t,j]]>
 * (0 if dropped): the combine-weight gradient when T_DO was kept. */
moe_status moe_dispatch(const moe_config* cfg, int32_t part, const void* src, const int32_t* slot,
                        void* DI, const void* dO_saved, float* dw, void* stream);

/* Expert FFN forward of one partition (Section II-B2: T_DI -> T_M -> T_DO).
 * For each expert e and its counts[part][e] rows: Z = DI W1[e]; A = gelu(Z)
 * (erf form); DO = A W2[e].  bf16 runs on MFMA with float accumulation.
 *   DI [R_p,M]; counts [n,E]; W1 [E,M,H]; W2 [E,H,M];
 *   Z [R_p,H] out, may be NULL when the pre-activation is not kept;
 *   A [R_p,H] scratch (activated rows, dead after the call); DO [R_p,M] out. */
moe_status moe_expert_ffn_fwd(const moe_config* cfg, int32_t part, const void* DI, const int32_t* counts,
                              const void* W1, const void* W2, void* Z, void* A, void* DO, void* stream);

/* Expert FFN backward of one partition ("symmetric", Section III-B; Table II's
 * 4 GEMMs, 5 with recomputation).  dDO holds the UNWEIGHTED upstream rows
 * (dispatch of dy); the combine weight of each row is applied here:
 *   [recompute != 0: Z = DI W1[e] first]
 *   G = dDO W2[e]^T;  dw_part[row, c] = partial sums over column block c of
 *   <gelu(Z_row), G_row> (their sum over c is d loss / d weight of the row);
 *   dZ = slot_w * G * gelu'(Z);  Z is overwritten with slot_w * gelu(Z);
 *   dW2[e] += (slot_w gelu(Z))^T dDO;  dDI = dZ W1[e]^T;  dW1[e] += DI^T dZ.
 *   Z [R_p,H] in/out (input ignored when recompute); dZ [R_p,H] scratch;
 *   dDI [R_p,M] out; dW1 [E,M,H], dW2 [E,H,M] float, accumulated into (stored
 *   when cfg->grad_overwrite and part == 0; an expert without rows then gets zeros);
 *   dw_part [R_p, moe_dw_parts(cfg)] float out, may be NULL. */
moe_status moe_expert_ffn_bwd(const moe_config* cfg, int32_t part, int32_t recompute,
                              const void* DI, void* Z, const void* dDO, const int32_t* counts,
                              const float* slot_w, const void* W1, const void* W2,
                              void* dZ, void* dDI, float* dW1, float* dW2, float* dw_part, void* stream);
moe_status moe_dw_parts(const moe_config* cfg, int32_t* parts);

/* Combine R of partition `part` (Fig. 1: T_DO -> T_O): for the partition's tokens
 * y[t] = sum over kept j of topk_w[t,j] * DO[slot[t,j]], float accumulation in
 * ascending j; exactly zero when every choice was dropped.  y [T,M] out. */
moe_status moe_combine(const moe_config* cfg, int32_t part, const void* DO, const int32_t* slot,
                       const float* topk_w, void* y, void* stream);

/* Gate backward of partition `part`: dL = softmax Jacobian applied to the
 * combine-weight gradients, dWg += x^T dL (two-stage, fixed order; dWg = x^T dL
 * when cfg->grad_overwrite and part == 0).  float32 storage multiplies in float;
 * bfloat16 storage multiplies on the matrix cores with dL split into two bfloat16
 * terms (16 bits of mantissa) and float accumulation.
 *   dw [T,k] float (used when dw_part is NULL) or dw_part [R_p, parts] summed in
 *   ascending c; dL [T,E] float out; scratch: moe_gate_scratch_bytes(cfg). */
moe_status moe_gate_bwd(const moe_config* cfg, int32_t part, const void* x, const float* logits,
                        const int32_t* topk_idx, const int32_t* slot, const float* dw,
                        const float* dw_part, float* dL, float* dWg, void* scratch, void* stream);
moe_status moe_gate_scratch_bytes(const moe_config* cfg, size_t* bytes);

/* Inverse of the slot map: rows[p][slot[t,j]] = t for every kept assignment of
 * partition p (t counted over the whole batch).  Entries at or beyond
 * counts[p][e] inside expert e's C_p-entry segment are not written.
 *   slot [T,k] in; rows [n, E*C_p] int32 out. */
moe_status moe_slot_rows(const moe_config* cfg, const int32_t* slot, int32_t* rows, void* stream);

/* moe_expert_ffn_fwd with the first GEMM's operand gathered: row r of expert e is
 * x[rows[part][e*C_p + r]] (Section II-B2's T_DI never exists; the result is the same
 * as dispatching first, bit for bit).  x [T,M]; rows from moe_slot_rows. */
moe_status moe_expert_ffn_fwd_gather(const moe_config* cfg, int32_t part, const void* x, const int32_t* rows,
                                     const int32_t* counts, const void* W1, const void* W2,
                                     void* Z, void* A, void* DO, void* stream);

/* Dispatch backward S' of partition `part`:
 * dx[t] = sum over kept j of dDI[slot[t,j]] + dL[t,:] Wg^T.   dx [T,M] out.
 * Float accumulation; for bfloat16 storage and E <= 16 the gate term runs on the
 * matrix cores with dL carried as the sum of two bfloat16 numbers (16 bits of its
 * mantissa), otherwise as float multiply-adds. */
moe_status moe_dispatch_bwd(const moe_config* cfg, int32_t part, const void* dDI, const int32_t* slot,
                            const float* dL, const void* Wg, void* dx, void* stream);

/* One whole training step of the layer: route, then for each partition
 * S -> C -> R pipelined over two streams (permutations on streams[0], GEMMs on
 * streams[1]; Section III-B), then the backward pass in the same fashion, under
 * cfg->reuse (Section III-D).  Forks from streams[0] and joins back to it: the
 * caller synchronises streams[0] only.  n_streams must be >= 2 (both may be the
 * same stream, which serialises the schedule).
 *   x, dy [T,M]; y, dx [T,M] out; dWg [M,E], dW1 [E,M,H], dW2 [E,H,M] float,
 *   accumulated into (caller zeroes) or, with cfg->grad_overwrite, overwritten;
 *   logits [T,E], topk_idx, topk_w, slot
 *   [T,k], counts [n,E] out; workspace of moe_workspace_bytes(cfg). */
moe_status moe_layer_step(const moe_config* cfg, const void* x, const void* dy,
                          const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                          void* y, void* dx, float* dWg, float* dW1, float* dW2,
                          float* logits, int32_t* topk_idx, float* topk_w, int32_t* slot, int32_t* counts,
                          void* workspace, size_t workspace_bytes,
                          void* const* streams, int32_t n_streams);

/* moe_layer_step for the offloading strategies (cfg->reuse = MOE_REUSE_S1..S3; Section
 * III-D, Table II).  host_buffer: pinned host memory (hipHostMalloc) of at least
 * moe_offload_bytes(cfg) bytes, owned by the caller, overwritten by every call.
 * streams: at least 3 (permutations, GEMMs, copies); joins back to streams[0].
 * The copies are hipMemcpyAsync calls: not for use under stream capture.
 * The other entry points reject these modes with MOE_ERR_UNSUPPORTED. */
moe_status moe_offload_bytes(const moe_config* cfg, size_t* host_bytes);
moe_status moe_layer_step_offload(const moe_config* cfg, const void* x, const void* dy,
                                  const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                                  void* y, void* dx, float* dWg, float* dW1, float* dW2,
                                  float* logits, int32_t* topk_idx, float* topk_w, int32_t* slot, int32_t* counts,
                                  void* workspace, size_t workspace_bytes,
                                  void* host_buffer, size_t host_bytes,
                                  void* const* streams, int32_t n_streams);

/* Forward half / backward half of moe_layer_step, for callers that run other
 * work between them.  Same arguments and workspace; backward reads what forward
 * left in the workspace and in the routing outputs, and consumes it: the kept T_M is
 * overwritten with the weighted activations and, in the shared-buffer modes, T_DO with
 * rows of dy.  One backward per forward; a second backward without a new forward gives
 * wrong gradients. */
moe_status moe_layer_forward(const moe_config* cfg, const void* x,
                             const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                             void* y, float* logits, int32_t* topk_idx, float* topk_w,
                             int32_t* slot, int32_t* counts,
                             void* workspace, size_t workspace_bytes,
                             void* const* streams, int32_t n_streams);
moe_status moe_layer_backward(const moe_config* cfg, const void* x, const void* dy,
                              const void* Wg, const void* W1, const void* W2,
                              void* dx, float* dWg, float* dW1, float* dW2,
                              const float* logits, const int32_t* topk_idx, const float* topk_w,
                              const int32_t* slot, const int32_t* counts,
                              void* workspace, size_t workspace_bytes,
                              void* const* streams, int32_t n_streams);

/* Counters of kernels launched by this process since the last reset, by class:
 * out[0] GEMM launches, out[1] permutation launches (dispatch, combine,
 * dispatch-backward), out[2] everything else.  Host only. */
moe_status moe_launch_counts(int64_t out[3], int32_t reset);

/* Optional timing of the library's kernels with HIP events recorded on the
 * stream each kernel is launched on.  moe_profile_enable(1) clears earlier
 * records and starts recording; moe_profile_enable(0) stops.  moe_profile_read
 * waits for the recorded events and returns, per kernel kind, the number of
 * launches and the summed duration in milliseconds.  Kinds: 0 first FFN GEMM
 * (GeLU epilogue), 1 second FFN GEMM and recomputation, 2 GEMM with the
 * GeLU-backward epilogue, 3 input-gradient GEMM, 4 weight-gradient GEMMs,
 * 5 dispatch, 6 combine, 7 dispatch backward, 8 gate, 9 slot assignment,
 * 10 gate backward.  Arrays of `kinds` entries (at most 11).  Host only; not
 * for use under stream capture. */
moe_status moe_profile_enable(int32_t on);
moe_status moe_profile_read(int32_t kinds, int64_t* launches, double* total_ms);

const char* moe_status_string(moe_status s);

/* Text of the most recent HIP failure behind a MOE_ERR_HIP (HIP's message and the
 * source line of the failing call); empty if there was none.  Host only. */
const char* moe_last_error(void);

/* ---- adaptive pipeline granularity (Algorithm 1, Section III-C) ------------------
 * Which n a batch of B tokens should be cut into, with as few timed searches as
 * possible: a table B -> n of answers given before, and the set S of pairs
 * (range of B, n), one per n, which answers every B inside a known range on the
 * hypothesis that the best n grows with B.  A handle owns both (host memory,
 * created and destroyed by the caller; not thread-safe).
 *
 * moe_gran_lookup: the listing's first half.  *n = the cached n, else the n of the
 *   range that holds B (then cached), else -1: a search is needed.  Should ranges
 *   overlap (hypothesis violated), the one with the smallest lower bound wins.
 * moe_gran_record: the listing's second half, after a search found n for B: the
 *   pair of that n is inserted as range(B, B) or widened to hold B; B is cached.
 * moe_gran_ranges: S ordered by lower bound; *count pairs (capacity 0: count only;
 *   a smaller non-zero capacity is MOE_ERR_SHAPE).
 * B <= 0 or n <= 0: MOE_ERR_SHAPE. */
typedef struct moe_gran moe_gran;
moe_status moe_gran_create(moe_gran** g);
moe_status moe_gran_destroy(moe_gran* g);
moe_status moe_gran_lookup(moe_gran* g, int64_t B, int32_t* n);
moe_status moe_gran_record(moe_gran* g, int64_t B, int32_t n);
moe_status moe_gran_ranges(const moe_gran* g, int32_t capacity, int64_t* lower, int64_t* upper,
                           int32_t* n, int32_t* count);

/* searchBestGran of Algorithm 1, by trials: for every candidate n (host array) runs
 * `warmup` untimed and `iters` timed moe_layer_step calls on the given buffers with
 * cfg->n_partitions replaced by the candidate (HIP events on streams[0]; blocks the
 * host) and returns the candidate with the least time per step.  Candidates that
 * do not divide T or whose workspace exceeds workspace_bytes are skipped.  counts
 * must hold [max candidate, E].  Trials run with grad_overwrite forced on; outputs
 * and gradients hold the last trial's results afterwards.
 *   ms: time per step of each candidate in milliseconds, -1 for skipped; may be NULL.
 *   No usable candidate: MOE_ERR_SHAPE. */
moe_status moe_search_best_gran(const moe_config* cfg, const void* x, const void* dy,
                                const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                                void* y, void* dx, float* dWg, float* dW1, float* dW2,
                                float* logits, int32_t* topk_idx, float* topk_w, int32_t* slot, int32_t* counts,
                                void* workspace, size_t workspace_bytes,
                                void* const* streams, int32_t n_streams,
                                const int32_t* candidates, int32_t n_candidates,
                                int32_t warmup, int32_t iters, int32_t* best_n, float* ms);

/* Algorithm 1 as a whole for B = cfg->T: lookup; if that fails, the search by
 * trials above and the record.  *n is the answer, *searched (may be NULL) tells
 * whether trials ran. */
moe_status moe_gran_get(moe_gran* g, const moe_config* cfg, const void* x, const void* dy,
                        const void* Wg, const float* gate_bias, const void* W1, const void* W2,
                        void* y, void* dx, float* dWg, float* dW1, float* dW2,
                        float* logits, int32_t* topk_idx, float* topk_w, int32_t* slot, int32_t* counts,
                        void* workspace, size_t workspace_bytes,
                        void* const* streams, int32_t n_streams,
                        const int32_t* candidates, int32_t n_candidates,
                        int32_t warmup, int32_t iters, int32_t* n, int32_t* searched);

/* ---- performance model of the memory-reuse strategies (Section III-E) ---------------
 * Strategies: 0 none, 1..4 = S1..S4 of Table II.  Per micro-batch of b tokens a GEMM is
 * b*H*M multiply-adds, an exchange (here: a local dispatch or combine) and a copy of T_DI
 * are b*M elements (Eq. 7-9); Table II gives the number of such units per stream and
 * pass; a pass costs the time of its slowest stream (Eq. 10; the copy term uses eta).
 *   W_comp multiply-adds/s, W_comm and W_mem elements/s when running alone;
 *   sigma, mu_*, eta_all: relative speed of computation, exchange and copy when the
 *   other streams run beside them (mu_comp: beside computation only; *_all: all three).
 * moe_strategy_cost: seconds per micro-batch, forward and backward.
 * moe_select_strategy: among the strategies whose bit is set in allowed_mask (bit s =
 *   strategy s), the one with the least forward + backward cost; ties to the lower
 *   number.  Non-positive sizes or speeds, unknown strategy, empty mask: MOE_ERR_SHAPE.
 * Host only.  (All five rows can be run and timed: "none" and S4 through moe_layer_step,
 * S1-S3 through moe_layer_step_offload.) */
typedef struct {
    double W_comp, W_comm, W_mem;
    double sigma, mu_comp, mu_all, eta_all;
} moe_speeds;
moe_status moe_strategy_cost(int32_t strategy, int64_t b, int64_t M, int64_t H, const moe_speeds* speeds,
                             double* cost_fw, double* cost_bw);
moe_status moe_select_strategy(uint32_t allowed_mask, int64_t b, int64_t M, int64_t H, const moe_speeds* speeds,
                               int32_t* best, double* cost);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H */
