// PiKV scheduling under bounded memory (Algorithm 1, C <- S(C, q_t); Section 3.4) and the
// constant-time insert (Algorithm 1 Insert; Section 3.1 storage invariants).
//
//   evict_select : one block per (sequence, expert).  The entries to drop are the
//                  n - capacity smallest under (utility ascending, slot descending), i.e.
//                  the complement of the `capacity` best under (utility descending, slot
//                  ascending).  An 8-bit most-significant-digit radix select over the
//                  order-preserving integer image of the fp32 utilities finds the cut value
//                  exactly (no floating-point comparison is ever redone in a different
//                  order), then one pass in slot order, driven by block-wide prefix sums,
//                  emits the evicted slots ascending and (optionally) compacts the
//                  utilities in place.
//   evict_move   : one block per (shard, kv head) slides the kept K and V rows down,
//                  chunk by chunk in ascending order (a destination never lies above its
//                  source, so reading a chunk fully before writing it is enough).
//   append_rows  : one block per (sequence, selected expert) writes the new entry.
#include "pikv_common.h"

namespace pikv {
namespace {

constexpr int kEvictThreads = 256;

// Inclusive prefix sum over the 256 threads of the block; *total receives the block sum.
__device__ __forceinline__ int block_scan_incl(int v, int *wave_sums, int *total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int t = __shfl_up(v, off, kWave);
        if (lane >= off) v += t;
    }
    __syncthreads();                      // protects wave_sums from the previous use
    if (lane == kWave - 1) wave_sums[wave] = v;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kEvictThreads / kWave; ++w) {
        const int s = wave_sums[w];
        if (w < wave) before += s;
        all += s;
    }
    *total = all;
    return v + before;
}

struct EvictParams {
    float *utility;
    int32_t *n_valid;
    const int32_t *sel_idx;
    int32_t *evicted_idx;
    int32_t *evicted_cnt;
    int E, S, capacity, sel_k, max_evict, compact;
};

__global__ __launch_bounds__(kEvictThreads) void evict_select(EvictParams p) {
    const int be = blockIdx.x;
    const int b = be / p.E, e = be - b * p.E;
    const int tid = threadIdx.x;

    __shared__ int hist[256];
    __shared__ int wave_sums[kEvictThreads / kWave];
    __shared__ int pick_digit, pick_before;

    bool selected = true;
    if (p.sel_idx) {
        selected = false;
        for (int j = 0; j < p.sel_k; ++j) selected |= (p.sel_idx[(int64_t)b * p.sel_k + j] == e);
    }
    const int n = p.n_valid[be];
    const int ngone = n - p.capacity;
    if (!selected || ngone <= 0 || ngone > p.max_evict) {
        if (tid == 0) p.evicted_cnt[be] = (selected && ngone > p.max_evict) ? -1 : 0;
        return;
    }
    float *u = p.utility + (int64_t)be * p.S;

    if (ngone == 1 && !p.compact) {
        // Streaming case: drop the single worst entry = minimum of (key, then largest slot).
        // One composite 64-bit value per entry orders both at once.
        uint64_t best = ~0ull;
        const int n4 = (p.S % 4 == 0) ? (n / 4) * 4 : 0;   // float4 reads need aligned rows
        for (int i = tid * 4; i < n4; i += kEvictThreads * 4) {
            const float4 v = *reinterpret_cast<const float4 *>(u + i);
            const uint64_t c0 = ((uint64_t)order_key(v.x) << 32) | (uint32_t)(0x7fffffff - i);
            const uint64_t c1 = ((uint64_t)order_key(v.y) << 32) | (uint32_t)(0x7fffffff - (i + 1));
            const uint64_t c2 = ((uint64_t)order_key(v.z) << 32) | (uint32_t)(0x7fffffff - (i + 2));
            const uint64_t c3 = ((uint64_t)order_key(v.w) << 32) | (uint32_t)(0x7fffffff - (i + 3));
            const uint64_t a = c0 < c1 ? c0 : c1, b2 = c2 < c3 ? c2 : c3;
            const uint64_t c = a < b2 ? a : b2;
            best = c < best ? c : best;
        }
        for (int i = n4 + tid; i < n; i += kEvictThreads) {
            const uint64_t c = ((uint64_t)order_key(u[i]) << 32) | (uint32_t)(0x7fffffff - i);
            best = c < best ? c : best;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint64_t o = __shfl_xor(best, off, kWave);
            best = o < best ? o : best;
        }
        __shared__ uint64_t wave_best[kEvictThreads / kWave];
        if ((tid & (kWave - 1)) == 0) wave_best[tid >> 6] = best;
        __syncthreads();
        if (tid == 0) {
            uint64_t m = wave_best[0];
#pragma unroll
            for (int w = 1; w < kEvictThreads / kWave; ++w) m = wave_best[w] < m ? wave_best[w] : m;
            p.evicted_idx[(int64_t)be * p.max_evict] = 0x7fffffff - (int)(uint32_t)(m & 0xffffffffu);
            p.evicted_cnt[be] = 1;
            p.n_valid[be] = p.capacity;
        }
        return;
    }

    // radix select: value of the ngone-th smallest key
    uint32_t prefix = 0, mask = 0;
    int remaining = ngone;   // rank still to locate among the keys matching `prefix`
    int count_eq = 0;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += kEvictThreads) {
            const uint32_t key = order_key(u[i]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 0xff], 1);
        }
        __syncthreads();
        const int mine = hist[tid];
        int total;
        const int incl = block_scan_incl(mine, wave_sums, &total);
        if (incl - mine < remaining && remaining <= incl) {
            pick_digit = tid;
            pick_before = incl - mine;
        }
        __syncthreads();
        prefix |= (uint32_t)pick_digit << shift;
        mask |= 0xffu << shift;
        remaining -= pick_before;
        count_eq = hist[pick_digit];
        __syncthreads();
    }
    const uint32_t cut = prefix;            // keys < cut go; of the keys == cut, the
    const int keep_eq = count_eq - remaining;  // first keep_eq in slot order stay

    int eq_seen = 0, gone_seen = 0;         // running totals over the chunks already done
    for (int base = 0; base < n; base += kEvictThreads) {
        const int i = base + tid;
        float ui = 0.0f;
        int is_eq = 0, is_less = 0;
        if (i < n) {
            ui = u[i];
            const uint32_t key = order_key(ui);
            is_eq = key == cut;
            is_less = key < cut;
        }
        int eq_total, gone_total;
        const int eq_incl = block_scan_incl(is_eq, wave_sums, &eq_total);
        const int eq_rank = eq_seen + eq_incl - is_eq;           // equal keys before slot i
        const int gone = is_less | (is_eq & (eq_rank >= keep_eq));
        const int gone_incl = block_scan_incl(gone, wave_sums, &gone_total);
        const int gone_before = gone_seen + gone_incl - gone;
        if (i < n) {
            if (gone)
                p.evicted_idx[(int64_t)be * p.max_evict + gone_before] = i;
            else if (p.compact && gone_before > 0)
                u[i - gone_before] = ui;    // reads of this chunk finished at the scans' barriers
        }
        eq_seen += eq_total;
        gone_seen += gone_total;
    }
    if (tid == 0) {
        p.evicted_cnt[be] = ngone;
        p.n_valid[be] = p.capacity;
    }
}

struct MoveParams {
    void *const *K;
    void *const *V;
    const int32_t *n_valid;
    const int32_t *evicted_idx;
    const int32_t *evicted_cnt;
    int64_t stride_h_bytes, stride_s_bytes;
    int row_chunks;      // 16-byte chunks per row
    int max_evict;
};

__global__ __launch_bounds__(kEvictThreads) void evict_move(MoveParams p) {
    const int be = blockIdx.x, hk = blockIdx.y;
    const int cnt = p.evicted_cnt[be];
    if (cnt <= 0) return;
    const int n_old = p.n_valid[be] + cnt;
    const int32_t *gone = p.evicted_idx + (int64_t)be * p.max_evict;
    const int rows_per_pass = kEvictThreads / p.row_chunks;
    const int rsub = threadIdx.x / p.row_chunks, csub = threadIdx.x % p.row_chunks;
    char *Kb = static_cast<char *>(p.K[be]) + hk * p.stride_h_bytes + csub * 16;
    char *Vb = static_cast<char *>(p.V[be]) + hk * p.stride_h_bytes + csub * 16;
    for (int base = gone[0]; base < n_old; base += rows_per_pass) {
        const int row = base + rsub;
        const bool active = rsub < rows_per_pass && row < n_old;
        int before = 0;
        bool dropped = false;
        uint4 kv = make_uint4(0, 0, 0, 0), vv = kv;
        if (active) {
            int lo = 0, hi = cnt;            // number of evicted slots < row
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (gone[mid] < row) lo = mid + 1; else hi = mid;
            }
            before = lo;
            dropped = lo < cnt && gone[lo] == row;
            if (!dropped) {
                kv = *reinterpret_cast<const uint4 *>(Kb + row * p.stride_s_bytes);
                vv = *reinterpret_cast<const uint4 *>(Vb + row * p.stride_s_bytes);
            }
        }
        __syncthreads();
        if (active && !dropped && before > 0) {
            *reinterpret_cast<uint4 *>(Kb + (row - before) * p.stride_s_bytes) = kv;
            *reinterpret_cast<uint4 *>(Vb + (row - before) * p.stride_s_bytes) = vv;
        }
        __syncthreads();
    }
}

struct AppendParams {
    const void *K_new;
    const void *V_new;
    const int32_t *topk;
    const int32_t *reuse_idx;
    const int32_t *reuse_cnt;
    void *const *K;
    void *const *V;
    float *utility;
    int32_t *n_valid;
    int64_t stride_h_bytes, stride_s_bytes;
    int E, S, Hkv, k, row_chunks, max_evict;
};

__global__ __launch_bounds__(kEvictThreads) void append_rows(AppendParams p) {
    const int b = blockIdx.x / p.k, j = blockIdx.x - b * p.k;
    const int e = p.topk[(int64_t)b * p.k + j];
    const int be = b * p.E + e;
    const int n = p.n_valid[be];
    int slot = n;
    if (p.reuse_cnt && p.reuse_cnt[be] > 0) slot = p.reuse_idx[(int64_t)be * p.max_evict];
    __syncthreads();                         // every thread has read n before it changes
    if (n >= p.S || slot < 0 || slot >= p.S) return;   // full shard: the entry is dropped
    const int total = p.Hkv * p.row_chunks;
    char *Kd = static_cast<char *>(p.K[be]) + slot * p.stride_s_bytes;
    char *Vd = static_cast<char *>(p.V[be]) + slot * p.stride_s_bytes;
    const char *Ks = static_cast<const char *>(p.K_new) + (int64_t)b * total * 16;
    const char *Vs = static_cast<const char *>(p.V_new) + (int64_t)b * total * 16;
    for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
        const int hk = idx / p.row_chunks, cc = idx - hk * p.row_chunks;
        *reinterpret_cast<uint4 *>(Kd + hk * p.stride_h_bytes + cc * 16) =
            *reinterpret_cast<const uint4 *>(Ks + (int64_t)idx * 16);
        *reinterpret_cast<uint4 *>(Vd + hk * p.stride_h_bytes + cc * 16) =
            *reinterpret_cast<const uint4 *>(Vs + (int64_t)idx * 16);
    }
    if (threadIdx.x == 0) {
        p.utility[(int64_t)be * p.S + slot] = 0.0f;
        p.n_valid[be] = n + 1;
    }
}

}  // namespace
}  // namespace pikv

using namespace pikv;

extern "C" int pikv_evict(const pikv_desc *desc, float *utility, int32_t *n_valid,
                          int32_t capacity, const int32_t *sel_idx, int32_t sel_k,
                          int32_t *evicted_idx, int32_t *evicted_cnt, int32_t max_evict,
                          int32_t compact, void *const *K_shards, void *const *V_shards,
                          void *stream) {
    const int rc = check_desc(desc);
    if (rc != PIKV_OK) return rc;
    if (!utility || !n_valid || !evicted_idx || !evicted_cnt) return PIKV_ERR_INVALID;
    if (capacity < 0 || max_evict < 1) return PIKV_ERR_INVALID;
    if (sel_idx && (sel_k < 1 || sel_k > desc->E)) return PIKV_ERR_INVALID;
    if (compact && (!K_shards || !V_shards)) return PIKV_ERR_INVALID;
    if (desc->B == 0) return PIKV_OK;
    hipStream_t st = as_stream(stream);
    EvictParams p;
    p.utility = utility;
    p.n_valid = n_valid;
    p.sel_idx = sel_idx;
    p.evicted_idx = evicted_idx;
    p.evicted_cnt = evicted_cnt;
    p.E = desc->E;
    p.S = desc->S;
    p.capacity = capacity;
    p.sel_k = sel_k;
    p.max_evict = max_evict;
    p.compact = compact ? 1 : 0;
    hipLaunchKernelGGL(evict_select, dim3(desc->B * desc->E), dim3(kEvictThreads), 0, st, p);
    int lrc = launch_status();
    if (lrc != PIKV_OK || !compact) return lrc;
    MoveParams m;
    m.K = K_shards;
    m.V = V_shards;
    m.n_valid = n_valid;
    m.evicted_idx = evicted_idx;
    m.evicted_cnt = evicted_cnt;
    const int eb = elem_bytes(desc->dtype);
    m.stride_h_bytes = desc->stride_h * eb;
    m.stride_s_bytes = desc->stride_s * eb;
    m.row_chunks = desc_width(desc) * eb / 16;
    m.max_evict = max_evict;
    hipLaunchKernelGGL(evict_move, dim3(desc->B * desc->E, desc->Hkv), dim3(kEvictThreads), 0, st,
                       m);
    return launch_status();
}

extern "C" int pikv_append(const pikv_desc *desc, const void *K_new, const void *V_new,
                           const int32_t *topk_idx, int32_t k, const int32_t *reuse_idx,
                           const int32_t *reuse_cnt, int32_t max_evict, void *const *K_shards,
                           void *const *V_shards, float *utility, int32_t *n_valid,
                           void *stream) {
    const int rc = check_desc(desc);
    if (rc != PIKV_OK) return rc;
    if (!K_new || !V_new || !topk_idx || !K_shards || !V_shards || !utility || !n_valid)
        return PIKV_ERR_INVALID;
    if (k < 1 || k > desc->E) return PIKV_ERR_INVALID;
    if ((reuse_idx == nullptr) != (reuse_cnt == nullptr)) return PIKV_ERR_INVALID;
    if (reuse_idx && max_evict < 1) return PIKV_ERR_INVALID;
    if (desc->B == 0) return PIKV_OK;
    AppendParams p;
    p.K_new = K_new;
    p.V_new = V_new;
    p.topk = topk_idx;
    p.reuse_idx = reuse_idx;
    p.reuse_cnt = reuse_cnt;
    p.K = K_shards;
    p.V = V_shards;
    p.utility = utility;
    p.n_valid = n_valid;
    const int eb = elem_bytes(desc->dtype);
    p.stride_h_bytes = desc->stride_h * eb;
    p.stride_s_bytes = desc->stride_s * eb;
    p.E = desc->E;
    p.S = desc->S;
    p.Hkv = desc->Hkv;
    p.k = k;
    p.row_chunks = desc_width(desc) * eb / 16;
    p.max_evict = max_evict;
    hipLaunchKernelGGL(append_rows, dim3(desc->B * k), dim3(kEvictThreads), 0, as_stream(stream),
                       p);
    return launch_status();
}
