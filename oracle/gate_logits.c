/*
 * TEST INFRASTRUCTURE ONLY -- part of the CPU oracle, never of the product path.
 *
 * Gate logits of the MoE layer's gating network (a linear map of E*M
 * parameters, Section II-B2; top-k gate, Section IV-A) in float32 with ONE
 * written-down summation order, so that routing decisions can be compared bit
 * for bit with any other implementation of the same order.
 *
 * The paper fixes no order; this is the reading used here:
 *
 *   - element d of a token row belongs to accumulator  l = (d / 8) mod 64;
 *   - each of the 64 accumulators starts at +0.0f and takes its elements in
 *     ascending d with one fused multiply-add per element,
 *         acc[l] = fmaf(x[t][d], Wg[d][e], acc[l]);
 *   - the 64 accumulators are then folded pairwise with offsets
 *     32, 16, 8, 4, 2, 1:  acc[l] = acc[l] + acc[l + off]  for l < off;
 *   - the logit is acc[0], plus bias[e] (one float32 add) when a bias is given.
 *
 * Inputs are float32; bf16 data is widened to float32 by the caller.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

void oracle_gate_logits_f32(const float *x, const float *wg, const float *bias,
                            int64_t T, int64_t M, int64_t E, float *logits)
{
    for (int64_t t = 0; t < T; ++t) {
        const float *xt = x + (size_t)t * (size_t)M;
        for (int64_t e = 0; e < E; ++e) {
            float acc[64];
            for (int l = 0; l < 64; ++l) acc[l] = 0.0f;
            for (int64_t d = 0; d < M; ++d) {
                int l = (int)((d / 8) % 64);
                acc[l] = fmaf(xt[d], wg[(size_t)d * (size_t)E + (size_t)e], acc[l]);
            }
            for (int off = 32; off >= 1; off >>= 1)
                for (int l = 0; l < off; ++l) acc[l] = acc[l] + acc[l + off];
            float v = acc[0];
            if (bias) v = v + bias[e];
            logits[(size_t)t * (size_t)E + (size_t)e] = v;
        }
    }
}
