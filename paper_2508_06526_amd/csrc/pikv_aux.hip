// Two small stages around the hot path:
//
//   router_penalty : the additive per-expert term of PiKV's penalised routers (Section 3.2,
//                    Table 1, column "Penalty Term", rows LB, P and E), one wavefront
//                    (pikv_penalty_dev.h): absorbs this step's selections into the load counter
//                    and writes the bias that the next pikv_route / pikv_decode_step call adds
//                    to the logits.
//   compress_rows  : Algorithm 1, (K^, V^) <- C_cmp(K_t, V_t) for the rank-r linear compressor of
//                    Section 3.3 (Table 2, LoRA rows): code = W_enc x, rounded once to the storage
//                    type.  One block per (sequence, kv head, K or V); 8 lanes per code element read the
//                    encoder row and the vector with 16-byte loads and join by an xor butterfly.
#include "pikv_common.h"
#include "pikv_penalty_dev.h"

#include <math.h>

namespace pikv {
namespace {

__global__ __launch_bounds__(kWave) void router_penalty(PenaltyParams p) { penalty_wave(p, threadIdx.x); }

// Table 1 row B: the score-free round-robin router.  One thread per (routed row, position).
__global__ __launch_bounds__(256) void route_round_robin(int n, int E, int k, long long step, int32_t *topk,
                                                         float *gates) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int r = i / k, j = i - r * k;
    topk[i] = (int32_t)(((step + r) * k + j) % E);
    gates[i] = 1.0f / (float)k;
}

// Measurement kernel: reads `parts` spans of each of n buffers once, the way the attention pass
// reads K/V rows (4 waves per block, a wave load = 1 KiB of consecutive bytes, non-temporal,
// 16 loads of a wave in flight), folds the words (xor) and writes one per block.  No arithmetic
// besides the fold: what it reaches is the most any pass that has to read these bytes can.
__global__ __launch_bounds__(256) void stream_read_probe(const char *const *bufs, size_t bytes_each, size_t span,
                                                         int parts, uint32_t *out) {
    const int buf = blockIdx.x / parts, part = blockIdx.x - buf * parts;
    const char *base = bufs[buf];
    const size_t lo = (size_t)part * span, hi = lo + span < bytes_each ? lo + span : bytes_each;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint4 acc = make_uint4(0, 0, 0, 0);
    constexpr size_t kWaveBytes = 16 * 1024;           // per wave and iteration: 16 loads of 1 KiB
    for (size_t at = lo + (size_t)wave * kWaveBytes; at < hi; at += 4 * kWaveBytes) {
        uint4 v[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const size_t a = at + (size_t)t * 1024 + (size_t)lane * 16;
            const bool in = a + 16 <= hi;
            v[t] = load16_stream(base + (in ? a : hi - 16));   // clamped onto the span's last 16 bytes,
            if (!in) v[t] = make_uint4(0, 0, 0, 0);            // which then do not count
        }
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            acc.x ^= v[t].x;
            acc.y ^= v[t].y;
            acc.z ^= v[t].z;
            acc.w ^= v[t].w;
        }
    }
    uint32_t w = acc.x ^ acc.y ^ acc.z ^ acc.w;
    for (int off = 1; off < 64; off <<= 1) w ^= __shfl_xor(w, off, 64);
    __shared__ uint32_t ws[4];
    if (lane == 0) ws[wave] = w;
    __syncthreads();
    if (threadIdx.x == 0) out[blockIdx.x] = ws[0] ^ ws[1] ^ ws[2] ^ ws[3];
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

template <typename T>
__device__ __forceinline__ void store_elem(T *p, int64_t i, float v);
template <>
__device__ __forceinline__ void store_elem<float>(float *p, int64_t i, float v) {
    p[i] = v;
}
template <>
__device__ __forceinline__ void store_elem<bf16>(bf16 *p, int64_t i, float v) {
    const f32x2_t pair = {v, 0.0f};
    const bf16x2_t r = __builtin_convertvector(pair, bf16x2_t);     // round to nearest even
    p[i].bits = (uint16_t)(__builtin_bit_cast(uint32_t, r) & 0xffffu);
}

template <typename T>
__global__ __launch_bounds__(256) void compress_rows(const T *xK, const T *WK, T *codesK, const T *xV,
                                                     const T *WV, T *codesV, int Hkv, int D, int rank) {
    constexpr int EPL = Pack16<T>::N;
    const T *x = blockIdx.y == 0 ? xK : xV;    // grid.y: 0 = keys, 1 = values
    const T *W_enc = blockIdx.y == 0 ? WK : WV;
    T *codes = blockIdx.y == 0 ? codesK : codesV;
    const int bh = blockIdx.x;                 // b * Hkv + h
    const int h = bh % Hkv;
    const int tid = threadIdx.x, sub = tid & 7;
    const int chunks = D / EPL;
    const T *xv = x + (int64_t)bh * D;
    const T *W = W_enc + (int64_t)h * rank * D;
    for (int c0 = 0; c0 < rank; c0 += 256 / 8) {
        const int c = c0 + (tid >> 3);
        const bool real = c < rank;
        float a = 0.0f;
        if (real) {
            for (int ch = sub; ch < chunks; ch += 8) {
                float wf[EPL], xf[EPL];
                Pack16<T>::widen(load16(W + (int64_t)c * D + ch * EPL), wf);
                Pack16<T>::widen(load16(xv + ch * EPL), xf);
#pragma unroll
                for (int i = 0; i < EPL; ++i) a = fmaf(wf[i], xf[i], a);
            }
        }
        a += __shfl_xor(a, 1, kWave);
        a += __shfl_xor(a, 2, kWave);
        a += __shfl_xor(a, 4, kWave);
        if (real && sub == 0) store_elem<T>(codes, (int64_t)bh * rank + c, a);
    }
}

}  // namespace
}  // namespace pikv

using namespace pikv;

extern "C" int pikv_router_penalty(int32_t mode, const int32_t *topk_idx, int32_t rows, int32_t k,
                                   int32_t E, int32_t *load, const int32_t *miss, float coef,
                                   float *bias, void *stream) {
    const int rc = check_penalty(mode, load, miss, coef, bias, E);
    if (rc != PIKV_OK) return rc;
    if (rows < 0 || k < 0) return PIKV_ERR_INVALID;
    if ((int64_t)rows * k > 0 && !topk_idx) return PIKV_ERR_INVALID;
    if ((int64_t)rows * k > 0x7fffffff) return PIKV_ERR_UNSUPPORTED;
    PenaltyParams p;
    p.mode = mode;
    p.topk = topk_idx;
    p.n_sel = rows * k;
    p.E = E;
    p.load = load;
    p.miss = miss;
    p.coef = coef;
    p.bias = bias;
    hipLaunchKernelGGL(router_penalty, dim3(1), dim3(kWave), 0, as_stream(stream), p);
    return launch_status();
}

extern "C" int pikv_compress(const pikv_desc *desc, const void *K_full, const void *Wenc_K,
                             void *K_codes, const void *V_full, const void *Wenc_V, void *V_codes,
                             void *stream) {
    const int rc = check_desc(desc);
    if (rc != PIKV_OK) return rc;
    if (desc->rank == 0 || !K_full || !Wenc_K || !K_codes) return PIKV_ERR_INVALID;
    const bool both = V_full || Wenc_V || V_codes;
    if (both && (!V_full || !Wenc_V || !V_codes)) return PIKV_ERR_INVALID;
    if (desc->B == 0) return PIKV_OK;
    const dim3 grid(desc->B * desc->Hkv, both ? 2 : 1), block(256);
    hipStream_t st = as_stream(stream);
    if (desc->dtype == PIKV_F32)
        hipLaunchKernelGGL(compress_rows<float>, grid, block, 0, st, static_cast<const float *>(K_full),
                           static_cast<const float *>(Wenc_K), static_cast<float *>(K_codes),
                           static_cast<const float *>(V_full), static_cast<const float *>(Wenc_V),
                           static_cast<float *>(V_codes), desc->Hkv, desc->D, desc->rank);
    else
        hipLaunchKernelGGL(compress_rows<bf16>, grid, block, 0, st, static_cast<const bf16 *>(K_full),
                           static_cast<const bf16 *>(Wenc_K), static_cast<bf16 *>(K_codes),
                           static_cast<const bf16 *>(V_full), static_cast<const bf16 *>(Wenc_V),
                           static_cast<bf16 *>(V_codes), desc->Hkv, desc->D, desc->rank);
    return launch_status();
}

extern "C" int pikv_route_round_robin(int32_t rows, int32_t E, int32_t k, int64_t step,
                                      int32_t *topk_idx, float *gates, void *stream) {
    if (rows < 0 || E < 1 || E > 64 || k < 1 || k > E || step < 0) return PIKV_ERR_INVALID;
    if (!topk_idx || !gates) return PIKV_ERR_INVALID;
    if ((int64_t)rows * k > 0x7fffffff) return PIKV_ERR_UNSUPPORTED;
    if (rows == 0) return PIKV_OK;
    const int n = rows * k;
    hipLaunchKernelGGL(route_round_robin, dim3((n + 255) / 256), dim3(256), 0, as_stream(stream), n, E, k,
                       (long long)step, topk_idx, gates);
    return launch_status();
}


extern "C" int pikv_stream_read_probe(const void *const *bufs, int32_t n, size_t bytes_each, int32_t parts,
                                      uint32_t *out, void *stream) {
    if (!bufs || !out || n < 1 || parts < 1 || bytes_each < 16 || bytes_each % 16 != 0) return PIKV_ERR_INVALID;
    if ((int64_t)n * parts > 0x7fffffff) return PIKV_ERR_INVALID;
    size_t span = (bytes_each + parts - 1) / parts;
    span = (span + 4095) / 4096 * 4096;
    if (span * (size_t)(parts - 1) >= bytes_each) return PIKV_ERR_INVALID;      // a part would be empty
    hipLaunchKernelGGL(stream_read_probe, dim3((unsigned)(n * parts)), dim3(256), 0, as_stream(stream),
                       reinterpret_cast<const char *const *>(bufs), bytes_each, span, parts, out);
    return launch_status();
}
