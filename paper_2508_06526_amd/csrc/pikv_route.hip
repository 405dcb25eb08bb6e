// PiKV routing (Section 3.2, Table 1 "TopK softmax" with the optional additive penalty):
// one block per routed row computes the E logits of x W_r (+ bias), the softmax over all
// experts and the k-hot mask, in a single launch.
//
// Threads are laid out as (row slice js, expert e): consecutive lanes read consecutive
// elements of W_r, so a wave's load is one contiguous run of the row-major matrix.  The
// slices are summed by a fixed-order LDS tree, which makes the logits (and therefore the
// selection) independent of scheduling.  Selection is by rank counting: expert e's rank is
// the number of experts that beat it under (logit descending, index ascending), so the
// output order and the tie-break need no sorting network.
#include "pikv_common.h"

#include <math.h>

namespace pikv {
namespace {

constexpr int kRouteThreads = 1024;

template <typename T>
__global__ __launch_bounds__(kRouteThreads) void route_kernel(const T *x, const T *W_r,
                                                              const float *bias, int d_r, int E,
                                                              int EP, int k, int32_t *topk_idx,
                                                              float *gates, float *probs) {
    const int row = blockIdx.x;
    const int tid = threadIdx.x;
    const int e = tid % EP;           // EP = E rounded up to a power of two
    const int js = tid / EP;
    const int JS = kRouteThreads / EP;

    __shared__ float red[kRouteThreads];
    __shared__ float logit[64];

    float acc = 0.0f;
    if (e < E) {
        const T *xr = x + (int64_t)row * d_r;
        for (int j = js; j < d_r; j += JS)
            acc = fmaf(load_scalar<T>(xr, j), load_scalar<T>(W_r, (int64_t)j * E + e), acc);
    }
    red[tid] = acc;
    __syncthreads();
    for (int half = JS >> 1; half >= 1; half >>= 1) {
        if (js < half) red[tid] += red[tid + half * EP];
        __syncthreads();
    }
    if (tid < 64) {
        float v = -INFINITY;
        if (tid < E) {
            v = red[tid] + (bias ? bias[tid] : 0.0f);
            if (v != v) v = -INFINITY;          // a NaN logit ranks last
        }
        logit[tid] = v;
    }
    __syncthreads();
    if (tid >= 64) return;

    // wave 0: lane e owns expert e
    const float mine = logit[tid];
    float mx = mine;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
    const float pe = tid < E ? __expf(mine - mx) : 0.0f;
    float den = pe;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) den += __shfl_xor(den, off, kWave);
    if (probs && tid < E) probs[(int64_t)row * E + tid] = pe / den;

    int rank = 0;
    for (int o = 0; o < E; ++o) {
        const float other = logit[o];
        rank += (other > mine) || (other == mine && o < tid);
    }
    const bool chosen = tid < E && rank < k;
    float sel = chosen ? pe : 0.0f;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sel += __shfl_xor(sel, off, kWave);
    if (chosen) {
        topk_idx[(int64_t)row * k + rank] = tid;
        gates[(int64_t)row * k + rank] = pe / sel;
    }
}

}  // namespace
}  // namespace pikv

using namespace pikv;

extern "C" int pikv_route(const void *x, const void *W_r, const float *bias, int32_t rows,
                          int32_t d_r, int32_t E, int32_t k, int32_t dtype, int32_t *topk_idx,
                          float *gates, float *probs, void *stream) {
    if (!x || !W_r || !topk_idx || !gates) return PIKV_ERR_INVALID;
    if (rows < 0 || d_r < 1 || E < 1 || E > 64 || k < 1 || k > E) return PIKV_ERR_INVALID;
    if (dtype != PIKV_F32 && dtype != PIKV_BF16) return PIKV_ERR_INVALID;
    if (rows == 0) return PIKV_OK;
    int EP = 1;
    while (EP < E) EP <<= 1;
    hipStream_t st = as_stream(stream);
    const dim3 grid(rows), block(kRouteThreads);
    if (dtype == PIKV_F32)
        hipLaunchKernelGGL(route_kernel<float>, grid, block, 0, st, static_cast<const float *>(x),
                           static_cast<const float *>(W_r), bias, d_r, E, EP, k, topk_idx, gates,
                           probs);
    else
        hipLaunchKernelGGL(route_kernel<bf16>, grid, block, 0, st, static_cast<const bf16 *>(x),
                           static_cast<const bf16 *>(W_r), bias, d_r, E, EP, k, topk_idx, gates,
                           probs);
    return launch_status();
}
