// PiKV scheduling score (Section 3.4, Table 3 row H2O: u_i = a_i, the attention an entry
// received), kept as a running value u_i <- decay * u_i + a_i.
//
// The attention pass left the raw scores s_{h,i} of every visited entry and, per (query
// head, selected shard), a pair (shift, coef) with p_{h,i} = coef * exp(s_{h,i} - shift).
// This pass turns them into probabilities and sums them over the heads that read the
// entry, in fixed head order (no atomics, bit-reproducible).  Grid: (sequence, expert,
// slot tile); blocks of shards nobody selected exit at once and leave u untouched.
#include "pikv_common.h"

#include <math.h>

namespace pikv {
namespace {

constexpr int kUtilThreads = 256;
constexpr int kUtilSlotsPerThread = 4;
constexpr int kUtilTile = kUtilThreads * kUtilSlotsPerThread;

struct UtilParams {
    const float *scores;
    const float *slot_coef;
    const int32_t *n_valid;
    const int32_t *topk;
    float *utility;
    int Hq, E, S, k, rr, tiles;
    float decay;
};

__global__ __launch_bounds__(kUtilThreads) void utility_kernel(UtilParams p) {
    int bid = blockIdx.x;
    const int tile = bid % p.tiles;
    bid /= p.tiles;
    const int e = bid % p.E;
    const int b = bid / p.E;
    const int n = p.n_valid[(int64_t)b * p.E + e];
    const int i0 = tile * kUtilTile;
    if (i0 >= n) return;

    __shared__ int head_j[256];       // position of expert e in head h's selection, or -1
    __shared__ float head_shift[256];
    __shared__ float head_coef[256];
    __shared__ int any_head;
    const int tid = threadIdx.x;
    if (tid == 0) any_head = 0;
    __syncthreads();
    for (int h = tid; h < p.Hq; h += blockDim.x) {
        const int row = b * p.rr + (p.rr == 1 ? 0 : h);
        int jj = -1;
        for (int j = 0; j < p.k; ++j)
            if (p.topk[(int64_t)row * p.k + j] == e) jj = j;
        head_j[h] = jj;
        if (jj >= 0) {
            const float *sc = p.slot_coef + (((int64_t)b * p.Hq + h) * p.k + jj) * 2;
            head_shift[h] = sc[0];
            head_coef[h] = sc[1];
            any_head = 1;
        }
    }
    __syncthreads();
    if (!any_head) return;

    const int i = i0 + tid * kUtilSlotsPerThread;
    if (i >= n) return;
    float a[kUtilSlotsPerThread] = {0.0f, 0.0f, 0.0f, 0.0f};
    const bool full = (i + kUtilSlotsPerThread <= n) && (p.S % kUtilSlotsPerThread == 0);
    for (int h = 0; h < p.Hq; ++h) {
        const int jj = head_j[h];
        if (jj < 0) continue;
        const float shift = head_shift[h], coef = head_coef[h];
        const float *s = p.scores + (((int64_t)b * p.Hq + h) * p.k + jj) * p.S + i;
        if (full) {
            const float4 v = *reinterpret_cast<const float4 *>(s);
            a[0] += coef * __expf(v.x - shift);
            a[1] += coef * __expf(v.y - shift);
            a[2] += coef * __expf(v.z - shift);
            a[3] += coef * __expf(v.w - shift);
        } else {
#pragma unroll
            for (int t = 0; t < kUtilSlotsPerThread; ++t)
                if (i + t < n) a[t] += coef * __expf(s[t] - shift);
        }
    }
    float *u = p.utility + ((int64_t)b * p.E + e) * p.S + i;
#pragma unroll
    for (int t = 0; t < kUtilSlotsPerThread; ++t)
        if (i + t < n) u[t] = fmaf(p.decay, u[t], a[t]);
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
    p.tiles = (desc->S + kUtilTile - 1) / kUtilTile;
    p.decay = decay;
    const int64_t blocks = (int64_t)desc->B * desc->E * p.tiles;
    if (blocks > 0x7fffffff) return PIKV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(utility_kernel, dim3((unsigned)blocks), dim3(kUtilThreads), 0,
                       as_stream(stream), p);
    return launch_status();
}
