// PiKV routing (Section 3.2, Table 1 "TopK softmax" with the optional additive penalty):
// one 1024-thread block per routed row computes the E logits of x W_r (+ bias), the softmax
// over all experts and the k-hot mask, in a single launch.
//
//   route_vec_kernel : W_r rows that are a power-of-two number of 16-byte chunks (E = 8..64
//                      in bf16, 4..64 in fp32): 16-byte loads, see pikv_route_dev.h.
//   route_kernel     : any E <= 64: threads laid out as (row slice, expert) with scalar
//                      element loads (consecutive lanes read consecutive elements of W_r),
//                      slices summed by a fixed-order LDS tree.
// Both make the logits (and therefore the selection) independent of scheduling.  Selection
// is by rank counting: expert e's rank is the number of experts that beat it under (logit
// descending, index ascending), so the output order and the tie-break need no sorting network.
#include "pikv_common.h"
#include "pikv_route_dev.h"

#include <math.h>

namespace pikv {
namespace {

// Generic path (any E <= 64): scalar element loads, LDS tree over the row slices.
template <typename T>
__global__ __launch_bounds__(kRouteThreads) void route_kernel(const T *x, const T *W_r,
                                                              const float *bias, int d_r, int E,
                                                              int EP, int k, int32_t *topk_idx,
                                                              float *gates, float *probs) {
    const int row = blockIdx.x;
    const int tid = threadIdx.x;
    __shared__ float red[kRouteThreads];
    const float bias_e = route_bias_of_lane(bias, E, tid & (kWave - 1));
    route_logits_generic<T>(x + (int64_t)row * d_r, W_r, d_r, E, EP, red);   // EP = E rounded up to a power of two
    if (tid < 64) select_topk(route_logit_generic_of_lane(red, bias_e, E, tid), tid, row, E, k, topk_idx, gates, probs);
}

// Fast path: a row of W_r is a whole number (1, 2, 4, 8 or 16) of 16-byte chunks; see
// route_logits_vec for the thread layout.
template <typename T>
__global__ __launch_bounds__(kRouteThreads) void route_vec_kernel(const T *x, const T *W_r,
                                                                  const float *bias, int d_r,
                                                                  int E, int cpr, int k,
                                                                  int32_t *topk_idx, float *gates,
                                                                  float *probs) {
    __shared__ float red[kRouteThreads / kWave][64];
    const int row = blockIdx.x;
    const float bias_e = route_bias_of_lane(bias, E, threadIdx.x & (kWave - 1));
    route_logits_vec<T>(x + (int64_t)row * d_r, W_r, bias, d_r, E, cpr, red);
    if (threadIdx.x < 64)
        select_topk(route_logit_of_lane(red, bias_e, E, threadIdx.x), threadIdx.x, row, E, k, topk_idx, gates,
                    probs);
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
    int cpr = 0;
    if (route_vec_ok(W_r, E, dtype, &cpr)) {
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
