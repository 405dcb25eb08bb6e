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

// Softmax over the E logits, rank-count selection and gate renormalisation, by the first
// wavefront of the block (lane e owns expert e).  `logit` is in LDS.
__device__ __forceinline__ void select_topk(const float *logit, int lane, int row, int E, int k,
                                            int32_t *topk_idx, float *gates, float *probs) {
    const float mine = logit[lane];
    float mx = mine;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
    const float pe = lane < E ? __expf(mine - mx) : 0.0f;
    float den = pe;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) den += __shfl_xor(den, off, kWave);
    if (probs && lane < E) probs[(int64_t)row * E + lane] = pe / den;

    int rank = 0;
    for (int o = 0; o < E; ++o) {
        const float other = logit[o];
        rank += (other > mine) || (other == mine && o < lane);
    }
    const bool chosen = lane < E && rank < k;
    float sel = chosen ? pe : 0.0f;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sel += __shfl_xor(sel, off, kWave);
    if (chosen) {
        topk_idx[(int64_t)row * k + rank] = lane;
        gates[(int64_t)row * k + rank] = pe / sel;
    }
}

// Generic path (any E <= 64): scalar element loads, LDS tree over the row slices.
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
    if (tid < 64) select_topk(logit, tid, row, E, k, topk_idx, gates, probs);
}

// Fast path: a row of W_r is a whole number (1, 2, 4, 8 or 16) of 16-byte chunks.  Every
// thread streams 16-byte chunks of the row-major matrix (thread t takes chunks t, t+1024,
// ... so a wave reads 1 KiB of consecutive bytes per load and all loads of a thread are
// independent); its chunk-in-row index never changes, so it accumulates EPL experts.
// Lanes with the same chunk index are summed by xor-shuffles, the 16 waves through LDS in
// fixed order.
template <typename T>
__global__ __launch_bounds__(kRouteThreads) void route_vec_kernel(const T *x, const T *W_r,
                                                                  const float *bias, int d_r,
                                                                  int E, int cpr, int k,
                                                                  int32_t *topk_idx, float *gates,
                                                                  float *probs) {
    constexpr int EPL = Pack16<T>::N;
    constexpr int kWaves = kRouteThreads / kWave;
    const int row = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int cir = tid & (cpr - 1);
    const int cshift = ilog2(cpr);
    const int total = d_r * cpr;

    __shared__ float red[kWaves][64];
    __shared__ float logit[64];

    const T *xr = x + (int64_t)row * d_r;
    float acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.0f;
#pragma unroll 4
    for (int c = tid; c < total; c += kRouteThreads) {
        const uint4 w = load16(W_r + (int64_t)c * EPL);
        const float xj = load_scalar<T>(xr, c >> cshift);
        float wf[EPL];
        Pack16<T>::widen(w, wf);
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] = fmaf(xj, wf[i], acc[i]);
    }
    for (int off = cpr; off < kWave; off <<= 1) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] += __shfl_xor(acc[i], off, kWave);
    }
    if (lane < cpr) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) red[wave][cir * EPL + i] = acc[i];
    }
    __syncthreads();
    if (tid < 64) {
        float v = -INFINITY;
        if (tid < E) {
            v = 0.0f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) v += red[w][tid];
            v += bias ? bias[tid] : 0.0f;
            if (v != v) v = -INFINITY;
        }
        logit[tid] = v;
    }
    __syncthreads();
    if (tid < 64) select_topk(logit, tid, row, E, k, topk_idx, gates, probs);
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
    hipStream_t st = as_stream(stream);
    const dim3 grid(rows), block(kRouteThreads);
    const int row_bytes = E * elem_bytes(dtype);
    const int cpr = row_bytes / 16;
    const bool vec = row_bytes % 16 == 0 && (cpr & (cpr - 1)) == 0 &&
                     reinterpret_cast<uintptr_t>(W_r) % 16 == 0;
    if (vec) {
        if (dtype == PIKV_F32)
            hipLaunchKernelGGL(route_vec_kernel<float>, grid, block, 0, st,
                               static_cast<const float *>(x), static_cast<const float *>(W_r), bias,
                               d_r, E, cpr, k, topk_idx, gates, probs);
        else
            hipLaunchKernelGGL(route_vec_kernel<bf16>, grid, block, 0, st,
                               static_cast<const bf16 *>(x), static_cast<const bf16 *>(W_r), bias,
                               d_r, E, cpr, k, topk_idx, gates, probs);
        return launch_status();
    }
    int EP = 1;
    while (EP < E) EP <<= 1;
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
