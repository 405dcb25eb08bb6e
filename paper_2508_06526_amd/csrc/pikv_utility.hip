// PiKV scheduling score (Section 3.4, Table 3 row H2O: u_i = a_i, the attention an entry
// received), kept as a running value u_i <- decay * u_i + a_i.
//
// The attention pass left the raw scores s_{h,i} of every visited entry and, per (query
// head, selected shard), a pair (shift, coef) with p_{h,i} = coef * exp(s_{h,i} - shift).
// This pass turns them into probabilities and sums them over the heads that read the
// entry, in fixed head order (no atomics, bit-reproducible).  Grid: (sequence, expert,
// slot tile); blocks of shards nobody selected exit at once and leave u untouched.
//
// The tracked form also keeps the per-entry bookkeeping of Table 3's LRU / LRU+ rows in the
// same pass: an entry whose attention mass of this step exceeds a threshold has its
// last-access stamp set to the step counter and its access count raised by one.
#include "pikv_common.h"

#include <math.h>

namespace pikv {
namespace {

constexpr int kUtilThreads = 256;
// Two block shapes.  One slot per thread (256 slots per block, a wave reads 256 contiguous
// bytes, every thread walks through all the heads): few heads per entry.  Or one (slot, quarter
// of the heads) per thread (64 slots per block, one wave per quarter): with hundreds of query
// rows per entry - a multi-query step - the walk through the heads is four times shorter, four
// times as many blocks share the score bytes, and each thread keeps 8 loads in flight.  The
// heads are summed in the same four ascending groups joined as (g0 + g1) + (g2 + g3) either way.
constexpr int kUtilManyHeads = 128;     // from this many query rows per sequence on: the second shape
constexpr int kUtilBatch = 8;           // loads in flight per thread in the second shape

struct UtilParams {
    const float *scores;
    const float *slot_coef;
    const int32_t *n_valid;
    const int32_t *topk;
    float *utility;      // may be null in the tracked form
    int Hq, E, S, k, rr, tiles;
    float decay;
    // access bookkeeping (Table 3 rows LRU / LRU+): an entry whose attention mass of this
    // step exceeds `threshold` is accessed at step `now`
    int32_t *last_access;
    int32_t *freq;
    float threshold;
    int now;
};

template <bool TRACK, bool SPREAD>
__global__ __launch_bounds__(kUtilThreads) void utility_kernel(UtilParams p) {
    constexpr int kUtilTile = SPREAD ? kUtilThreads / 4 : kUtilThreads;
    int bid = blockIdx.x;
    const int tile = bid % p.tiles;
    bid /= p.tiles;
    const int e = bid % p.E;
    const int b = bid / p.E;
    const int n = p.n_valid[(int64_t)b * p.E + e];
    const int i0 = tile * kUtilTile;
    if (i0 >= n) return;

    // heads that selected expert e, compacted in ascending head order (fixed summation order)
    __shared__ int head_off[256];       // offset of the head's score row for this shard
    __shared__ float head_shift[256];
    __shared__ float head_coef[256];
    __shared__ int wave_cnt[kUtilThreads / kWave];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;

    int jj = -1;
    if (tid < p.Hq) {
        const int row = b * p.rr + (p.rr == 1 ? 0 : tid);
        for (int j = 0; j < p.k; ++j)
            if (p.topk[(int64_t)row * p.k + j] == e) jj = j;
    }
    const uint64_t mask = __ballot(jj >= 0);
    if (lane == 0) wave_cnt[wave] = __popcll(mask);
    __syncthreads();
    int before = 0, nact = 0;
#pragma unroll
    for (int w = 0; w < kUtilThreads / kWave; ++w) {
        if (w < wave) before += wave_cnt[w];
        nact += wave_cnt[w];
    }
    if (nact == 0) return;
    if (jj >= 0) {
        const int pos = before + __popcll(mask & ((1ull << lane) - 1ull));
        const int hrow = (b * p.Hq + tid) * p.k + jj;
        head_off[pos] = hrow;
        head_shift[pos] = p.slot_coef[(int64_t)hrow * 2 + 0];
        head_coef[pos] = p.slot_coef[(int64_t)hrow * 2 + 1];
    }
    __syncthreads();

    const int gsize = (nact + 3) / 4;
    if constexpr (SPREAD) {
        // thread = (slot, group): wave g walks through group g's heads, kUtilBatch loads at a time
        // from clamped addresses (no load under a lane-dependent condition), the sums meet in LDS
        __shared__ float part_s[4][kUtilTile];
        const int slot = tid & (kUtilTile - 1), g = tid / kUtilTile;
        const int i = i0 + slot, ic = min(i, n - 1);
        const int lo = g * gsize, hi = min(nact, lo + gsize);
        float a = 0.0f;
        for (int t0 = lo; t0 < hi; t0 += kUtilBatch) {
            float sc[kUtilBatch];
#pragma unroll
            for (int u = 0; u < kUtilBatch; ++u)
                sc[u] = p.scores[(int64_t)head_off[min(t0 + u, hi - 1)] * p.S + ic];
            const int left = __builtin_amdgcn_readfirstlane(hi - t0);   // the group is the wave's
#pragma unroll
            for (int u = 0; u < kUtilBatch; ++u) {
                const int t = min(t0 + u, hi - 1);
                const float with = fmaf(head_coef[t], __expf(sc[u] - head_shift[t]), a);
                a = u < left ? with : a;
            }
        }
        part_s[g][slot] = a;
        __syncthreads();
        if (g != 0 || i >= n) return;
        const float mass = (part_s[0][slot] + part_s[1][slot]) + (part_s[2][slot] + part_s[3][slot]);
        const int64_t at = ((int64_t)b * p.E + e) * p.S + i;
        if (!TRACK || p.utility) p.utility[at] = fmaf(p.decay, p.utility[at], mass);
        if (TRACK && mass > p.threshold) {
            p.last_access[at] = p.now;
            p.freq[at] += 1;
        }
        return;
    }
    const int i = i0 + tid;
    if (i >= n) return;
    // the active heads are cut into 4 consecutive groups, each summed in ascending order, the
    // groups joined as (g0 + g1) + (g2 + g3): the fused step kernel spreads the groups over
    // threads and must reproduce these bits
    float part[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int lo = g * gsize, hi = min(nact, lo + gsize);
        float a = 0.0f;
        int t = lo;
        for (; t + 4 <= hi; t += 4) {   // four independent loads in flight per thread
            const float s0 = p.scores[(int64_t)head_off[t + 0] * p.S + i];
            const float s1 = p.scores[(int64_t)head_off[t + 1] * p.S + i];
            const float s2 = p.scores[(int64_t)head_off[t + 2] * p.S + i];
            const float s3 = p.scores[(int64_t)head_off[t + 3] * p.S + i];
            a = fmaf(head_coef[t + 0], __expf(s0 - head_shift[t + 0]), a);
            a = fmaf(head_coef[t + 1], __expf(s1 - head_shift[t + 1]), a);
            a = fmaf(head_coef[t + 2], __expf(s2 - head_shift[t + 2]), a);
            a = fmaf(head_coef[t + 3], __expf(s3 - head_shift[t + 3]), a);
        }
        for (; t < hi; ++t)
            a = fmaf(head_coef[t], __expf(p.scores[(int64_t)head_off[t] * p.S + i] - head_shift[t]), a);
        part[g] = a;
    }
    const float mass = (part[0] + part[1]) + (part[2] + part[3]);
    const int64_t at = ((int64_t)b * p.E + e) * p.S + i;
    if (!TRACK || p.utility) p.utility[at] = fmaf(p.decay, p.utility[at], mass);
    if (TRACK && mass > p.threshold) {
        p.last_access[at] = p.now;
        p.freq[at] += 1;
    }
}

int launch_utility(const pikv_desc *desc, const float *scores, const float *slot_coef,
                   const int32_t *n_valid, const int32_t *topk_idx, int32_t k, float decay,
                   float *utility, bool track, float threshold, int32_t now,
                   int32_t *last_access, int32_t *freq, void *stream) {
    UtilParams p;
    p.scores = scores;
    p.slot_coef = slot_coef;
    p.n_valid = n_valid;
    p.topk = topk_idx;
    p.utility = utility;
    p.Hq = desc->Hq;
    p.E = desc->E;
    p.S = desc->S;
    p.k = k;
    p.rr = desc->route_rows_per_seq;
    const bool spread = desc->Hq >= kUtilManyHeads;
    const int tile_slots = spread ? kUtilThreads / 4 : kUtilThreads;
    p.tiles = (desc->S + tile_slots - 1) / tile_slots;
    p.decay = decay;
    p.last_access = last_access;
    p.freq = freq;
    p.threshold = threshold;
    p.now = now;
    const int64_t blocks = (int64_t)desc->B * desc->E * p.tiles;
    if (blocks > 0x7fffffff) return PIKV_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)blocks), block(kUtilThreads);
    hipStream_t st = as_stream(stream);
    if (track && spread) hipLaunchKernelGGL((utility_kernel<true, true>), grid, block, 0, st, p);
    else if (track) hipLaunchKernelGGL((utility_kernel<true, false>), grid, block, 0, st, p);
    else if (spread) hipLaunchKernelGGL((utility_kernel<false, true>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((utility_kernel<false, false>), grid, block, 0, st, p);
    return launch_status();
}

}  // namespace
}  // namespace pikv

using namespace pikv;

extern "C" int pikv_update_utility(const pikv_desc *desc, const float *scores,
                                   const float *slot_coef, const int32_t *n_valid,
                                   const int32_t *topk_idx, int32_t k, float decay,
                                   float *utility, void *stream) {
    const int rc = check_desc(desc);
    if (rc != PIKV_OK) return rc;
    if (!scores || !slot_coef || !n_valid || !topk_idx || !utility) return PIKV_ERR_INVALID;
    if (k < 1 || k > desc->E) return PIKV_ERR_INVALID;
    if (!(decay >= 0.0f) || decay > 3.0e38f) return PIKV_ERR_INVALID;
    if (desc->B == 0) return PIKV_OK;
    return launch_utility(desc, scores, slot_coef, n_valid, topk_idx, k, decay, utility, false, 0.0f,
                          0, nullptr, nullptr, stream);
}

extern "C" int pikv_update_utility_tracked(const pikv_desc *desc, const float *scores,
                                           const float *slot_coef, const int32_t *n_valid,
                                           const int32_t *topk_idx, int32_t k, float decay,
                                           float *utility, float threshold, int32_t now,
                                           int32_t *last_access, int32_t *freq, void *stream) {
    const int rc = check_desc(desc);
    if (rc != PIKV_OK) return rc;
    if (!scores || !slot_coef || !n_valid || !topk_idx || !last_access || !freq)
        return PIKV_ERR_INVALID;
    if (k < 1 || k > desc->E) return PIKV_ERR_INVALID;
    if (utility && (!(decay >= 0.0f) || decay > 3.0e38f)) return PIKV_ERR_INVALID;
    if (!(threshold >= 0.0f)) return PIKV_ERR_INVALID;
    if (desc->B == 0) return PIKV_OK;
    return launch_utility(desc, scores, slot_coef, n_valid, topk_idx, k, decay, utility, true,
                          threshold, now, last_access, freq, stream);
}
