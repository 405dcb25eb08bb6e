// Device-side pieces of the router shared by the stand-alone routing kernel and the fused
// step kernel (PiKV Section 3.2, Table 1 "TopK softmax").
#pragma once

#include <type_traits>

#include "pikv_common.h"

#include <math.h>

namespace pikv {

constexpr int kRouteThreads = 1024;

// Softmax over the E logits, rank-count selection and gate renormalisation by one wavefront,
// from registers: lane e holds expert e's logit (-inf in lanes >= E).  Returns the lane's rank
// under (logit descending, index ascending); lanes with rank < k are the selection.  Every
// wavefront that calls it with the same logits gets the same result, so a block may let all
// its waves call it instead of broadcasting one wave's result through a barrier.
// Lane i receives the value of lane (i - R) & 15 of its row of 16 lanes (DPP row rotate right).
template <int R>
__device__ __forceinline__ float row_rotate(float x) {
    static_assert(R >= 1 && R <= 15, "rotation inside a row of 16 lanes");
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x120 + R, 0xf, 0xf, true));
}

// rank += [expert (lane - R) & 15 beats this lane's expert], R = 1 .. 15: with E <= 16 all experts
// sit in the first row of 16 lanes, and every pair meets in one rotation without the scalar unit.
template <int R>
__device__ __forceinline__ void rank_by_rotation(float mine, int lane, int &rank) {
    if constexpr (R <= 15) {
        const float other = row_rotate<R>(mine);
        const int o = (lane - R) & 15;
        rank += (other > mine) || (other == mine && o < lane);
        rank_by_rotation<R + 1>(mine, lane, rank);
    }
}

// The selection in two parts, so that a caller can start what depends on the selected experts
// alone (their ranks) before the gates exist: the rank needs the logits only, the gates need the
// softmax as well.
//   route_rank : the lane's rank under (logit descending, index ascending), 64 in lanes >= E.
//   route_gates: softmax over the E logits, the gates of the k selected experts renormalised
//                over the selection; writes topk_idx / gates (and probs) when given.
__device__ __forceinline__ int route_rank(float mine, int lane, int E) {
    int rank = 0;
    if (E <= 16) {
        rank_by_rotation<1>(mine, lane, rank);
    } else {
        for (int o = 0; o < E; ++o) {      // every lane's logit passes through the scalar unit
            const float other = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mine), o));
            rank += (other > mine) || (other == mine && o < lane);
        }
    }
    return lane < E ? rank : 64;
}
__device__ __forceinline__ void route_gates(float mine, int rank, int lane, int row, int E, int k,
                                            int32_t *topk_idx, float *gates, float *probs) {
    // Lanes >= E hold the identities (-inf, 0), and only lanes < E use the results: with E <= 16
    // the butterflies stay inside the first row of 16 lanes (same operands, same bits).
    const bool one_row = E <= 16;
    const float mx = one_row ? bits_max<0, 4>(mine) : bits_max<0, 6>(mine);
    const float pe = lane < E ? __expf(mine - mx) : 0.0f;
    const float den = one_row ? bits_sum<0, 4>(pe) : bits_sum<0, 6>(pe);
    if (probs && lane < E) probs[(int64_t)row * E + lane] = pe / den;
    const bool chosen = lane < E && rank < k;
    const float picked = chosen ? pe : 0.0f;
    const float sel = one_row ? bits_sum<0, 4>(picked) : bits_sum<0, 6>(picked);
    if (chosen && topk_idx) {
        topk_idx[(int64_t)row * k + rank] = lane;
        gates[(int64_t)row * k + rank] = pe / sel;
    }
}
__device__ __forceinline__ int select_topk(float mine, int lane, int row, int E, int k,
                                           int32_t *topk_idx, float *gates, float *probs) {
    const int rank = route_rank(mine, lane, E);
    route_gates(mine, rank, lane, row, E, k, topk_idx, gates, probs);
    return rank;
}

// Logits of one routed row with the whole 1024-thread block, for a row-major W_r whose rows
// are `cpr` (a power of two <= 16) 16-byte chunks.  Thread t streams chunks t, t+1024, ...
// (a wave reads 1 KiB of consecutive bytes per load; all loads of a thread are independent);
// its chunk-in-row index never changes, so it accumulates the same EPL experts throughout.
// Lanes with equal chunk index are summed by xor-shuffles, the 16 waves through LDS in fixed
// order, so the logits do not depend on scheduling.  Ends, after one block barrier, with the
// per-wave sums in `red`; route_logit_of_lane then gives any wavefront its lanes' logits.
template <typename T>
__device__ __forceinline__ void route_logits_vec(const T *xr, const T *W_r, const float *bias,
                                                 int d_r, int E, int cpr, float (*red)[64]) {
    constexpr int EPL = Pack16<T>::N;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int cir = tid & (cpr - 1);
    (void)bias;
    (void)E;
    const int cshift = ilog2(cpr);
    const int total = d_r * cpr;

    float acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.0f;
    // batches of 8, then 4, then single chunks: all loads of a batch are in flight together,
    // the multiply-adds stay in ascending chunk order whatever the batching
    auto batch = [&](int c, auto nload) {
        constexpr int NB = decltype(nload)::value;
        uint4 w[NB];
        float xj[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            w[u] = load16(W_r + (int64_t)(c + u * kRouteThreads) * EPL);
            xj[u] = load_scalar<T>(xr, (c + u * kRouteThreads) >> cshift);
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            float wf[EPL];
            Pack16<T>::widen(w[u], wf);
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] = fmaf(xj[u], wf[i], acc[i]);
        }
    };
    int c = tid;
    for (; c + 7 * kRouteThreads < total; c += 8 * kRouteThreads) batch(c, std::integral_constant<int, 8>{});
    for (; c + 3 * kRouteThreads < total; c += 4 * kRouteThreads) batch(c, std::integral_constant<int, 4>{});
    for (; c < total; c += kRouteThreads) batch(c, std::integral_constant<int, 1>{});
    // lanes with the same chunk-in-row index: xor butterfly over the lane bits from log2(cpr) up
    auto join = [&](auto bit) {
        constexpr int BIT = decltype(bit)::value;
        if ((1 << BIT) >= cpr) {
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] += lane_xor<BIT>(acc[i]);
        }
    };
    join(std::integral_constant<int, 0>{});
    join(std::integral_constant<int, 1>{});
    join(std::integral_constant<int, 2>{});
    join(std::integral_constant<int, 3>{});
    join(std::integral_constant<int, 4>{});
    join(std::integral_constant<int, 5>{});
    if (lane < cpr) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) red[wave][cir * EPL + i] = acc[i];
    }
    __syncthreads();
}

// Logits of one routed row for any E <= 64 and any alignment (scalar element loads): thread =
// (expert e = tid % EP, row slice tid / EP) with EP = E rounded up to a power of two, the slices
// joined by a fixed-order LDS tree.  Ends, after a block barrier, with expert e's sum in red[e];
// `red` holds kRouteThreads floats.
template <typename T>
__device__ __forceinline__ void route_logits_generic(const T *xr, const T *W_r, int d_r, int E, int EP,
                                                     float *red) {
    const int tid = threadIdx.x;
    const int e = tid % EP;
    const int js = tid / EP;
    const int JS = kRouteThreads / EP;
    float acc = 0.0f;
    if (e < E) {
        for (int j = js; j < d_r; j += JS)
            acc = fmaf(load_scalar<T>(xr, j), load_scalar<T>(W_r, (int64_t)j * E + e), acc);
    }
    red[tid] = acc;
    __syncthreads();
    for (int half = JS >> 1; half >= 1; half >>= 1) {
        if (js < half) red[tid] += red[tid + half * EP];
        __syncthreads();
    }
}
// Expert `lane`'s logit after route_logits_generic (experts >= E hold -inf; a NaN logit ranks last).
__device__ __forceinline__ float route_logit_generic_of_lane(const float *red, float bias_of_lane, int E,
                                                             int lane) {
    float v = -INFINITY;
    if (lane < E) {
        v = red[lane] + bias_of_lane;
        if (v != v) v = -INFINITY;
    }
    return v;
}

// The additive term of expert `lane` (0 without a bias or past the last expert).  Callers read
// it before the weights: it depends on nothing, and a load issued after the block barrier
// would put a whole trip to memory between the logits and the selection.
__device__ __forceinline__ float route_bias_of_lane(const float *bias, int E, int lane) {
    return (bias != nullptr && lane < E) ? bias[lane] : 0.0f;
}

// Expert `lane`'s logit from the per-wave sums (waves joined in ascending order; experts >= E
// hold -inf; a NaN logit is replaced by -inf).  Any wavefront may call it after the barrier.
__device__ __forceinline__ float route_logit_of_lane(const float (*red)[64], float bias_of_lane, int E,
                                                     int lane) {
    constexpr int kWaves = kRouteThreads / kWave;
    float v = -INFINITY;
    if (lane < E) {
        v = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) v += red[w][lane];
        v += bias_of_lane;
        if (v != v) v = -INFINITY;
    }
    return v;
}

// True when route_logits_vec applies: W_r rows are a power-of-two number of aligned 16-byte
// chunks.
inline bool route_vec_ok(const void *W_r, int E, int dtype, int *cpr) {
    const int row_bytes = E * elem_bytes(dtype);
    *cpr = row_bytes / 16;
    return row_bytes % 16 == 0 && (*cpr & (*cpr - 1)) == 0 &&
           reinterpret_cast<uintptr_t>(W_r) % 16 == 0;
}

}  // namespace pikv
