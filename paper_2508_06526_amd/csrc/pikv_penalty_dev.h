// The additive per-expert term of PiKV's penalised routers (Section 3.2, Table 1, column
// "Penalty Term"), as one wavefront's work: shared by the stand-alone kernel and by the fused
// decode step, whose last launch runs it so that closing the loop costs no launch of its own.
#pragma once

#include "pikv_common.h"

#include <math.h>

namespace pikv {

struct PenaltyParams {
    int mode;               // pikv_penalty
    const int32_t *topk;    // [n_sel] this step's selections
    int n_sel, E;
    int32_t *load;          // [E] running selection counts
    const int32_t *miss;    // [E], cache-aware mode
    float coef;
    float *bias;            // [E] out
};

// Lane e owns expert e: absorbs this step's selections into the load counter (integer,
// order-free) and writes the term the next routing call adds to the logits:
//   load balance   -alpha (mu_e - mean mu), mu_e = how often expert e has been selected
//   cache aware    -lambda log(1 + miss_e)
//   entropy        -beta (h_e - mean h), h_e = -p_e ln p_e, p_e = mu_e / sum mu (0 ln 0 = 0)
__device__ __forceinline__ void penalty_wave(const PenaltyParams &p, int e) {
    // lane e counts the selections equal to e: 64 ids per load, each then passed to every lane
    // through the scalar unit (one round trip per 64 selections instead of one per selection)
    int cnt = 0;
    for (int base = 0; base < p.n_sel; base += kWave) {
        const int mine_sel = base + e < p.n_sel ? p.topk[base + e] : -1;
#pragma unroll
        for (int s = 0; s < kWave; ++s) cnt += (__builtin_amdgcn_readlane(mine_sel, s) == e);
    }
    int mine = 0;
    if (e < p.E) {
        mine = p.load[e] + cnt;
        p.load[e] = mine;
    }
    if (p.mode == PIKV_PENALTY_CACHE_AWARE) {
        if (e < p.E) p.bias[e] = -p.coef * log1pf((float)p.miss[e]);
        return;
    }
    // exact integer total: neither the mean load nor the shares depend on lane order
    int total = mine;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) total += __shfl_xor(total, off, kWave);
    if (p.mode == PIKV_PENALTY_LOAD_BALANCE) {
        const float mean = (float)total / (float)p.E;
        if (e < p.E) p.bias[e] = -p.coef * ((float)mine - mean);
    } else {
        const float pe = total > 0 ? (float)mine / (float)total : 0.0f;
        const float he = pe > 0.0f ? -pe * logf(pe) : 0.0f;
        float sum = he;                      // lanes >= E hold 0; fixed butterfly order
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, kWave);
        if (e < p.E) p.bias[e] = -p.coef * (he - sum / (float)p.E);
    }
}

// Host-side checks shared by both callers.
inline int check_penalty(int mode, const int32_t *load, const int32_t *miss, float coef, const float *bias,
                         int E) {
    if (mode != PIKV_PENALTY_LOAD_BALANCE && mode != PIKV_PENALTY_CACHE_AWARE && mode != PIKV_PENALTY_ENTROPY)
        return PIKV_ERR_INVALID;
    if (!load || !bias || E < 1 || E > 64) return PIKV_ERR_INVALID;
    if (mode == PIKV_PENALTY_CACHE_AWARE && !miss) return PIKV_ERR_INVALID;
    if (!(coef == coef)) return PIKV_ERR_INVALID;
    return PIKV_OK;
}

}  // namespace pikv
