// Scheduling policies of PiKV Section 3.4 / Table 3 (rows H2O, SL, LRU, LRU+) as one device
// function, shared by the stand-alone policy kernel and the fused decode step, so that the
// float that decides an eviction is the same float on every path.
#pragma once

#include "pikv_common.h"

#include <math.h>

namespace pikv {

struct PolicyView {
    int policy;                  // pikv_policy
    int now, window, protect;
    float lambda, threshold;
    int32_t *birth;              // [B,E,S] each; which ones are needed depends on the policy
    int32_t *last_access;
    int32_t *freq;
};

// Utility of the entry at flat index `at` (= (b * E + e) * S + slot).
__device__ __forceinline__ float policy_value(const PolicyView &v, int64_t at, const float *h2o) {
    float u;
    if (v.policy == PIKV_POLICY_H2O) {
        u = h2o[at];
    } else if (v.policy == PIKV_POLICY_SL) {
        u = (v.now - v.birth[at] < v.window) ? 1.0f : 0.0f;
    } else {
        const float r = (float)(v.now - v.last_access[at]);
        u = (v.policy == PIKV_POLICY_LRU) ? -r : fmaf(v.lambda, (float)v.freq[at], -r);
    }
    if (v.protect > 0 && v.now - v.birth[at] < v.protect) u = INFINITY;
    return u;
}

// The same for four consecutive entries starting at `at` (a multiple of 4; the arrays are
// 16-byte aligned): 16-byte loads of only the arrays the policy reads.
__device__ __forceinline__ void policy_value4(const PolicyView &v, int64_t at, const float *h2o, float (&u)[4]) {
    int4 birth = make_int4(0, 0, 0, 0);
    const bool need_birth = v.policy == PIKV_POLICY_SL || v.protect > 0;
    if (need_birth) birth = *reinterpret_cast<const int4 *>(v.birth + at);
    const int b4[4] = {birth.x, birth.y, birth.z, birth.w};
    if (v.policy == PIKV_POLICY_H2O) {
        const float4 h = *reinterpret_cast<const float4 *>(h2o + at);
        u[0] = h.x, u[1] = h.y, u[2] = h.z, u[3] = h.w;
    } else if (v.policy == PIKV_POLICY_SL) {
#pragma unroll
        for (int t = 0; t < 4; ++t) u[t] = (v.now - b4[t] < v.window) ? 1.0f : 0.0f;
    } else {
        const int4 last = *reinterpret_cast<const int4 *>(v.last_access + at);
        const int l4[4] = {last.x, last.y, last.z, last.w};
        int4 freq = make_int4(0, 0, 0, 0);
        if (v.policy == PIKV_POLICY_LRU_PLUS) freq = *reinterpret_cast<const int4 *>(v.freq + at);
        const int f4[4] = {freq.x, freq.y, freq.z, freq.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float r = (float)(v.now - l4[t]);
            u[t] = (v.policy == PIKV_POLICY_LRU) ? -r : fmaf(v.lambda, (float)f4[t], -r);
        }
    }
    if (v.protect > 0) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (v.now - b4[t] < v.protect) u[t] = INFINITY;
    }
}

// True when policy_value4 may be used on rows of S entries of these arrays.
__device__ __forceinline__ bool policy_vec_ok(const PolicyView &v, const float *h2o, int S) {
    const uintptr_t all = reinterpret_cast<uintptr_t>(v.birth) | reinterpret_cast<uintptr_t>(v.last_access) |
                          reinterpret_cast<uintptr_t>(v.freq) | reinterpret_cast<uintptr_t>(h2o);
    return (S & 3) == 0 && (all & 15) == 0;
}

// Host-side argument check shared by the entry points that take a policy.
inline int check_policy(int policy, int window, int protect, float lambda, const int32_t *birth,
                        const int32_t *last_access, const int32_t *freq, const float *h2o) {
    if (policy < PIKV_POLICY_H2O || policy > PIKV_POLICY_LRU_PLUS) return PIKV_ERR_INVALID;
    if (policy == PIKV_POLICY_H2O && !h2o) return PIKV_ERR_INVALID;
    if ((policy == PIKV_POLICY_SL || protect > 0) && !birth) return PIKV_ERR_INVALID;
    if (policy >= PIKV_POLICY_LRU && !last_access) return PIKV_ERR_INVALID;
    if (policy == PIKV_POLICY_LRU_PLUS && (!freq || !(lambda == lambda))) return PIKV_ERR_INVALID;
    if (window < 0 || protect < 0) return PIKV_ERR_INVALID;
    return PIKV_OK;
}

}  // namespace pikv
