// Merging the split partials of the attention pass (PiKV Algorithm 1, f_attn over C[g_t], with
// the router gates): device code shared by the stand-alone combine kernel and the fused
// post-attention kernel of the decode step.
#pragma once

#include "pikv_common.h"

#include <math.h>

namespace pikv {

struct CombineParams {
    const float *part_acc;
    const float *part_ml;
    const float *gates;
    const void *U_V;
    float *y;
    float *row_max;
    float *row_norm;
    float *slot_coef;
    int Hq, G, D, W, k, rr, rank, nsplit, combine;
    int value_bias;   // U_V holds rank + 1 rows per kv head, the last one the decoder's additive term
    int tq;           // draft queries per sequence: y and the row statistics are [B, tq, Hq / tq, ...]
};

constexpr int kCombinePrefetch = 4;         // partial rows each thread loads before the weights exist
constexpr int kMaxPartialsPerHead = 2048;   // k * nsplit

// (max, normaliser) of one selected shard from its nsplit partial (max, sum) pairs, computed by
// a group of 8 adjacent lanes: lane `sub` takes splits sub, sub+8, ... in ascending order, the
// 8 lane results are joined by an xor butterfly.  Every caller uses this one arrangement, so the
// stand-alone and the fused kernels produce identical bits.  `get(s)` returns split s's pair;
// all 8 lanes of a group must call together (pass nsplit = 0 for a padding group).
// The first kShardPairsHeld pairs of a lane are fetched once and kept (shard_pairs_load), so a
// caller can issue these loads ahead of other, slower ones; later pairs are fetched again in
// each of the two passes.
constexpr int kShardPairsHeld = 4;
struct ShardPairs {
    float2 v[kShardPairsHeld];
};
template <class F>
__device__ __forceinline__ ShardPairs shard_pairs_load(int nsplit, int sub, F get) {
    ShardPairs sp;
#pragma unroll
    for (int u = 0; u < kShardPairsHeld; ++u) {
        const int s = sub + 8 * u;
        sp.v[u] = s < nsplit ? get(s) : make_float2(-INFINITY, 0.0f);
    }
    return sp;
}
template <class F>
__device__ __forceinline__ void shard_stats8(const ShardPairs &sp, int nsplit, int sub, F get, float *M_out,
                                             float *Z_out) {
    float M = -INFINITY;
#pragma unroll
    for (int u = 0; u < kShardPairsHeld; ++u) M = sp.v[u].y > 0.0f ? fmaxf(M, sp.v[u].x) : M;
    for (int s = sub + 8 * kShardPairsHeld; s < nsplit; s += 8) {
        const float2 v = get(s);
        M = v.y > 0.0f ? fmaxf(M, v.x) : M;
    }
    M = bits_max<0, 3>(M);      // xor butterfly over the 8 lanes, inside a DPP row
    float Z = 0.0f;
#pragma unroll
    for (int u = 0; u < kShardPairsHeld; ++u) Z += sp.v[u].y > 0.0f ? sp.v[u].y * __expf(sp.v[u].x - M) : 0.0f;
    for (int s = sub + 8 * kShardPairsHeld; s < nsplit; s += 8) {
        const float2 v = get(s);
        Z += v.y > 0.0f ? v.y * __expf(v.x - M) : 0.0f;
    }
    Z = bits_sum<0, 3>(Z);
    *M_out = M;
    *Z_out = Z;
}
template <class F>
__device__ __forceinline__ void shard_stats8(int nsplit, int sub, F get, float *M_out, float *Z_out) {
    shard_stats8(shard_pairs_load(nsplit, sub, get), nsplit, sub, get, M_out, Z_out);
}

// The k shard weights of one query head in either combine mode, from the per-shard
// (max, normaliser), computed by an aligned group of `kp` lanes (kp = the power of two >= k, at
// most 64): lane j of the group holds shard j's values (Zj = 0 in lanes j >= k), the row max and
// the normaliser are joined by xor butterflies inside the group (fixed order).  Every lane of
// the group must call.  Outputs for the lane's own shard: weight w of its un-normalised
// accumulator and the (shift, coef) pair with p_i = coef * exp(s_i - shift); M and norm are the
// row max / normaliser (the same in every lane of the group).
struct HeadWeights {
    float w, shift, coef, M, norm;
};
__device__ __forceinline__ HeadWeights head_weights(int kp, float Mj, float Zj, float gj, int combine) {
    const bool live = Zj > 0.0f;
    float M = live ? Mj : -INFINITY;
    for (int off = 1; off < kp; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, kWave));
    HeadWeights out;
    out.M = M;
    if (combine == PIKV_COMBINE_LSE) {
        float norm = live ? gj * Zj * __expf(Mj - M) : 0.0f;
        for (int off = 1; off < kp; off <<= 1) norm += __shfl_xor(norm, off, kWave);
        out.norm = norm;
        out.w = live ? gj * __expf(Mj - M) / norm : 0.0f;
        out.shift = live ? M : 0.0f;
        out.coef = live ? gj / norm : 0.0f;
    } else {
        float norm = live ? gj : 0.0f;
        for (int off = 1; off < kp; off <<= 1) norm += __shfl_xor(norm, off, kWave);
        out.norm = norm;
        out.w = live ? gj / (norm * Zj) : 0.0f;
        out.shift = live ? Mj : 0.0f;
        out.coef = out.w;
    }
    return out;
}
inline __host__ __device__ int pow2_at_least(int v) {
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

// One block (THREADS threads) merges the k * nsplit partials of head `bh`.  The partial
// accumulators do not depend on the weights, so their loads are issued first and overlap the
// whole weight computation:
//   phase 0: every thread = (slice of partials, float4 column group) issues its first
//            accumulator loads; (max, sum) of every partial goes to LDS.
//   phase 1: 8 lanes per selected shard reduce its splits to (max, normaliser).
//   phase 2: k lanes form the k gate-weighted shard weights in either combine mode.
//   phase 3: weighted sum of the accumulators, slices reduced through LDS in fixed order,
//            then (rank > 0) the value decoder y = ycode U_V[h'].
// Bytes of LDS combine_head<., threads> carves from the buffer it is given (np = k * nsplit
// partials per head).  Sized by the real np, not by its maximum: the blocks are short and
// many, and the LDS they reserve decides how many of them a CU holds at once.
inline __host__ __device__ int combine_np_pad(int np) { return (np + 3) & ~3; }
inline size_t combine_smem_bytes(int threads, int np) {
    return (size_t)(2 * combine_np_pad(np) + 6 * 64 + 128 + 4) * 4 + (size_t)threads * 16;
}

// Block size of the merge: one query head rarely has more than a few dozen partials; a small
// block then has the same latency and leaves the rest of the GPU to other work.  The fused
// and the stand-alone kernels use the same rule, which keeps their results bit-identical.
inline int combine_threads(int np) { return np <= 32 ? 256 : 1024; }

// Internal row bh = b * Hq + h (rows ordered kv head, draft query, head of the group) -> the row
// of the caller's [B, tq, Hq / tq] arrays (y, row_max, row_norm).
__device__ __forceinline__ int64_t caller_row(const CombineParams &p, int b, int h) {
    if (p.tq <= 1) return (int64_t)b * p.Hq + h;
    const int heads = p.Hq / p.tq, g = p.G / p.tq;
    const int hk = h / p.G, rem = h - hk * p.G;
    const int t = rem / g, gg = rem - t * g;
    return ((int64_t)b * p.tq + t) * heads + hk * g + gg;
}

template <typename T, int THREADS>
__device__ __forceinline__ void combine_head(const CombineParams &p, int bh, unsigned char *smem) {
    const int b = bh / p.Hq, h = bh - b * p.Hq;
    const int hk = h / p.G;
    const int64_t out = caller_row(p, b, h);
    const int tid = threadIdx.x;
    const int np = p.k * p.nsplit;

    float4 *red = reinterpret_cast<float4 *>(smem);                  // [THREADS]
    float *wt = reinterpret_cast<float *>(smem + THREADS * 16);     // max of every partial, later its weight
    float *ls = wt + combine_np_pad(np);
    float *Mj = ls + combine_np_pad(np), *Zj = Mj + 64, *shard_w = Zj + 64;
    float *g_s = shard_w + 3 * 64;
    float *ycode = g_s + 64;                                         // [128]
    float *live_s = ycode + 128;                                     // [1] 1 if any selected shard holds entries

    const int cgroups = p.W / 4;                 // float4 column groups: 4..32
    const int slices = THREADS / cgroups;        // partial slices
    const int cg = tid % cgroups, sl = tid / cgroups;
    const float *acc = p.part_acc + (int64_t)bh * np * p.W + cg * 4;
    float4 pre[kCombinePrefetch];
#pragma unroll
    for (int u = 0; u < kCombinePrefetch; ++u) {
        const int i = sl + u * slices;
        pre[u] = i < np ? *reinterpret_cast<const float4 *>(acc + (int64_t)i * p.W)
                        : make_float4(0.f, 0.f, 0.f, 0.f);
    }

    // the gates are read once into LDS: head_weights walks them several times
    if (p.gates != nullptr && tid < p.k)
        g_s[tid] = p.gates[(int64_t)(b * p.rr + (p.rr == 1 ? 0 : h)) * p.k + tid];
    const float *ml = p.part_ml + (int64_t)bh * np * 2;
    for (int i = tid; i < np; i += THREADS) {
        const float2 v = *reinterpret_cast<const float2 *>(ml + 2 * i);
        wt[i] = v.x;
        ls[i] = v.y;
    }
    __syncthreads();
    for (int j0 = 0; j0 < p.k; j0 += THREADS / 8) {   // 8 lanes per selected shard
        const int j = j0 + tid / 8;
        float M, Z;
        shard_stats8(j < p.k ? p.nsplit : 0, tid & 7,
                     [&](int sp) { return make_float2(wt[j * p.nsplit + sp], ls[j * p.nsplit + sp]); }, &M, &Z);
        if (j < p.k && (tid & 7) == 0) {
            Mj[j] = M;
            Zj[j] = Z;
        }
    }
    __syncthreads();
    if (tid < kWave) {   // lane j of the first wave owns selected shard j
        const bool mine = tid < p.k;
        const HeadWeights hw = head_weights(pow2_at_least(p.k), mine ? Mj[tid] : 0.0f, mine ? Zj[tid] : 0.0f,
                                            (mine && p.gates) ? g_s[tid] : 1.0f, p.combine);
        if (mine) {
            shard_w[tid] = hw.w;
            if (p.slot_coef)
                *reinterpret_cast<float2 *>(p.slot_coef + ((int64_t)bh * p.k + tid) * 2) =
                    make_float2(hw.shift, hw.coef);
        }
        if (tid == 0) {
            if (p.row_max) p.row_max[out] = hw.M;
            if (p.row_norm) p.row_norm[out] = hw.norm;
            *live_s = hw.M > -INFINITY ? 1.0f : 0.0f;
        }
    }
    __syncthreads();
    // weight of every partial: shard weight * exp(m_split - M_shard)
    for (int i = tid; i < np; i += THREADS) {
        const int j = i / p.nsplit;
        wt[i] = ls[i] > 0.0f ? shard_w[j] * __expf(wt[i] - Mj[j]) : 0.0f;
    }
    __syncthreads();

    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int u = 0; u < kCombinePrefetch; ++u) {
        const int i = sl + u * slices;
        const float w = i < np ? wt[i] : 0.0f;
        a.x = fmaf(w, pre[u].x, a.x);
        a.y = fmaf(w, pre[u].y, a.y);
        a.z = fmaf(w, pre[u].z, a.z);
        a.w = fmaf(w, pre[u].w, a.w);
    }
    for (int i = sl + kCombinePrefetch * slices; i < np; i += slices) {
        const float w = wt[i];
        const float4 v = *reinterpret_cast<const float4 *>(acc + (int64_t)i * p.W);
        a.x = fmaf(w, v.x, a.x);
        a.y = fmaf(w, v.y, a.y);
        a.z = fmaf(w, v.z, a.z);
        a.w = fmaf(w, v.w, a.w);
    }
    red[tid] = a;
    __syncthreads();
    // fixed-order tree over the slices (slices is a power of two)
    for (int half = slices >> 1; half >= 1; half >>= 1) {
        if (sl < half) {
            const float4 v = red[tid + half * cgroups];
            float4 t = red[tid];
            t.x += v.x;
            t.y += v.y;
            t.z += v.z;
            t.w += v.w;
            red[tid] = t;
        }
        __syncthreads();
    }
    if (tid < cgroups) {
        const float4 t = red[tid];
        if (p.rank == 0) {
            *reinterpret_cast<float4 *>(p.y + out * p.D + tid * 4) = t;
        } else {
            ycode[tid * 4 + 0] = t.x;
            ycode[tid * 4 + 1] = t.y;
            ycode[tid * 4 + 2] = t.z;
            ycode[tid * 4 + 3] = t.w;
        }
    }
    if (p.rank != 0) {  // value decoder: y = ycode U_V[h'] (+ b[h'], the weights of a row sum to one)
        __syncthreads();
        const T *U = static_cast<const T *>(p.U_V) + (int64_t)hk * (p.rank + p.value_bias) * p.D;
        for (int d = tid; d < p.D; d += THREADS) {
            float a2 = 0.0f;
            for (int cidx = 0; cidx < p.rank; ++cidx)
                a2 = fmaf(ycode[cidx], load_scalar<T>(U, (int64_t)cidx * p.D + d), a2);
            if (p.value_bias && *live_s != 0.0f) a2 += load_scalar<T>(U, (int64_t)p.rank * p.D + d);
            p.y[out * p.D + d] = a2;
        }
    }
}

// Host side (pikv_attn.hip).  check_attn_args: every host-side check of the attention call and
// its split plan, nothing launched - a caller with earlier launches of its own (the step's
// routing / insert kernel) rejects bad arguments before anything is enqueued.
int check_attn_args(const pikv_desc *desc, const void *q, const void *const *K_shards,
                    const void *const *V_shards, const void *U_K, const void *U_V,
                    const int32_t *n_valid, const int32_t *topk_idx, int32_t k, int32_t combine,
                    float scale, const float *y, const void *workspace, size_t workspace_bytes,
                    AttnPlan *plan_out);
// True while a profiling event pair is installed (pikv_set_profile_events).
bool profile_events_set();

// launch_attn_partial: validate, plan and launch the split pass only, and fill the parameters
// of the merge pass.
int launch_attn_partial(const pikv_desc *desc, const void *q, const void *const *K_shards,
                        const void *const *V_shards, const void *U_K, const void *U_V,
                        const int32_t *n_valid, const int32_t *topk_idx, const float *gates,
                        int32_t k, int32_t combine, float scale, float *y, float *row_max,
                        float *row_norm, float *scores, float *slot_coef, void *workspace,
                        size_t workspace_bytes, void *stream, AttnPlan *plan_out,
                        CombineParams *c_out);

int pikv_sharded_attn_merge(const pikv_desc *desc, const CombineParams *c, void *stream);

}  // namespace pikv
