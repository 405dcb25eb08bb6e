// PiKV scheduling under bounded memory (Algorithm 1, C <- S(C, q_t); Section 3.4) and the
// constant-time insert (Algorithm 1 Insert; Section 3.1 storage invariants).
//
//   evict_select : one block per (sequence, expert).  The entries to drop are the
//                  n - capacity smallest under (utility ascending, slot descending), i.e.
//                  the complement of the `capacity` best under (utility descending, slot
//                  ascending).  A bit-by-bit select over the order-preserving integer image
//                  of the fp32 utilities, held in registers, finds the cut value exactly
//                  (no floating-point comparison is ever redone in a different order),
//                  then one pass in slot order, driven by block-wide ranks of one-bit
//                  flags, emits the evicted slots ascending and (optionally) compacts the
//                  utilities in place.
//   evict_move   : one block per (shard, kv head) slides the kept K and V rows down,
//                  a pass of rows at a time in ascending order (a destination never lies
//                  above its source, so holding a pass in registers before writing it is
//                  enough).
//   append_rows  : one block per (sequence, selected expert) writes the new entry.
#include "pikv_common.h"

namespace pikv {
namespace {

constexpr int kEvictThreads = 256;   // evict_move and append_rows
constexpr int kSelThreads = 1024;    // evict_select
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSelCache = 24;        // keys a thread keeps in registers (n <= 24576)

// Block-wide sum of a count every lane of a wave already agrees on.  Two buffers used in
// turn make one barrier per call enough: a buffer is rewritten two calls later, and every
// wave has left the reads of call i before any wave passes the barrier of call i+1.
__device__ __forceinline__ int block_sum_waves(int wave_total, int (*buf)[kSelWaves], int &turn) {
    int *slot = buf[turn & 1];
    ++turn;
    if ((threadIdx.x & (kWave - 1)) == 0) slot[threadIdx.x >> 6] = wave_total;
    __syncthreads();
    int all = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) all += slot[w];
    return all;
}

// Exclusive block-wide rank of a one-bit flag in thread order; *total receives the block sum.
__device__ __forceinline__ int block_rank_flag(bool flag, int (*buf)[kSelWaves], int &turn,
                                               int *total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const uint64_t votes = __ballot(flag);
    const int in_wave = __popcll(votes & ((1ull << lane) - 1ull));
    int *slot = buf[turn & 1];
    ++turn;
    if (lane == 0) slot[wave] = __popcll(votes);
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        const int s = slot[w];
        if (w < wave) before += s;
        all += s;
    }
    *total = all;
    return before + in_wave;
}

struct EvictParams {
    float *utility;
    int32_t *n_valid;
    const int32_t *sel_idx;
    int32_t *evicted_idx;
    int32_t *evicted_cnt;
    int E, S, capacity, sel_k, max_evict, compact;
};

// General case: drop the `ngone` worst of `n` entries.  The cut (the ngone-th smallest key)
// is found one bit at a time from the top: count the candidates whose next bit is 0 and
// step into the half that holds the wanted rank.  With CACHED the keys sit in registers
// (slot i = tid + j * kSelThreads lives in keys[j]), so all 32 steps touch no memory.
template <bool CACHED>
__device__ __forceinline__ void select_many(const EvictParams &p, int be, float *u, int n,
                                            int ngone, int (*buf)[kSelWaves]) {
    const int tid = threadIdx.x;
    const int nchunk = (n + kSelThreads - 1) / kSelThreads;
    uint32_t keys[CACHED ? kSelCache : 1];
    if (CACHED) {
#pragma unroll
        for (int j = 0; j < kSelCache; ++j) {
            const int i = tid + j * kSelThreads;
            keys[j] = (j < nchunk && i < n) ? order_key(u[i]) : 0u;
        }
    }
    int turn = 0;
    uint32_t prefix = 0;
    int remaining = ngone;   // rank still to locate among the keys that match `prefix`
    int cand = n;            // how many keys match `prefix` on the bits decided so far
    for (int bit = 31; bit >= 0; --bit) {
        int zeros = 0;       // wave-uniform: candidates in this wave whose `bit` is 0
        auto tally = [&](uint32_t key, int i) {
            const bool hit = i < n && ((uint64_t)(key ^ prefix) >> (bit + 1)) == 0 &&
                             ((key >> bit) & 1u) == 0;
            zeros += __popcll(__ballot(hit));
        };
        if (CACHED) {
#pragma unroll
            for (int j = 0; j < kSelCache; ++j)
                if (j < nchunk) tally(keys[j], tid + j * kSelThreads);
        } else {
            for (int j = 0; j < nchunk; ++j) {
                const int i = tid + j * kSelThreads;
                tally(i < n ? order_key(u[i]) : 0u, i);
            }
        }
        const int tot0 = block_sum_waves(zeros, buf, turn);
        if (remaining > tot0) {
            remaining -= tot0;
            cand -= tot0;
            prefix |= 1u << bit;
        } else {
            cand = tot0;
        }
    }
    const uint32_t cut = prefix;          // keys < cut go; of the keys == cut (`cand` of
    const int keep_eq = cand - remaining; // them), the first keep_eq in slot order stay

    int eq_seen = 0, gone_seen = 0;       // running totals over the chunks already done
    auto emit = [&](uint32_t key, int i) {
        const bool valid = i < n;
        float ui = 0.0f;
        if (valid && p.compact) ui = u[i];
        const bool is_eq = valid && key == cut, is_less = valid && key < cut;
        int eq_total, gone_total;
        const int eq_rank = eq_seen + block_rank_flag(is_eq, buf, turn, &eq_total);
        const bool gone = is_less || (is_eq && eq_rank >= keep_eq);
        const int gone_before = gone_seen + block_rank_flag(gone, buf, turn, &gone_total);
        if (valid) {
            if (gone) {
                if (gone_before < p.max_evict)
                    p.evicted_idx[(int64_t)be * p.max_evict + gone_before] = i;
            }
            else if (p.compact && gone_before > 0)
                u[i - gone_before] = ui;  // this chunk's reads ended before the barriers above
        }
        eq_seen += eq_total;
        gone_seen += gone_total;
    };
    if (CACHED) {
#pragma unroll
        for (int j = 0; j < kSelCache; ++j)
            if (j < nchunk) emit(keys[j], tid + j * kSelThreads);
    } else {
        for (int j = 0; j < nchunk; ++j) {
            const int i = tid + j * kSelThreads;
            emit(i < n ? order_key(u[i]) : 0u, i);
        }
    }
}

__global__ __launch_bounds__(kSelThreads) void evict_select(EvictParams p) {
    const int be = blockIdx.x;
    const int b = be / p.E, e = be - b * p.E;
    const int tid = threadIdx.x;

    __shared__ int wave_cnt[2][kSelWaves];
    __shared__ uint64_t wave_best[kSelWaves];

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
        for (int i = tid * 4; i < n4; i += kSelThreads * 4) {
            const float4 v = *reinterpret_cast<const float4 *>(u + i);
            const uint64_t c0 = evict_composite(v.x, i), c1 = evict_composite(v.y, i + 1);
            const uint64_t c2 = evict_composite(v.z, i + 2), c3 = evict_composite(v.w, i + 3);
            const uint64_t a = c0 < c1 ? c0 : c1, b2 = c2 < c3 ? c2 : c3;
            const uint64_t c = a < b2 ? a : b2;
            best = c < best ? c : best;
        }
        for (int i = n4 + tid; i < n; i += kSelThreads) {
            const uint64_t c = evict_composite(u[i], i);
            best = c < best ? c : best;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint64_t o = __shfl_xor(best, off, kWave);
            best = o < best ? o : best;
        }
        if ((tid & (kWave - 1)) == 0) wave_best[tid >> 6] = best;
        __syncthreads();
        if (tid == 0) {
            uint64_t m = wave_best[0];
#pragma unroll
            for (int w = 1; w < kSelWaves; ++w) m = wave_best[w] < m ? wave_best[w] : m;
            p.evicted_idx[(int64_t)be * p.max_evict] = evict_composite_slot(m);
            p.evicted_cnt[be] = 1;
            p.n_valid[be] = p.capacity;
        }
        return;
    }

    if (n <= kSelCache * kSelThreads)
        select_many<true>(p, be, u, n, ngone, wave_cnt);
    else
        select_many<false>(p, be, u, n, ngone, wave_cnt);
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
    int row_chunks;      // 16-byte chunks per row, 1..kEvictThreads
    int max_evict;
};

constexpr int kMoveRows = 8;                             // rows a thread carries per pass
constexpr int kMoveFlagWords = kEvictThreads * kMoveRows / 32;
static_assert(kMoveFlagWords == kWave, "one wave ranks the flag words");

__global__ __launch_bounds__(kEvictThreads) void evict_move(MoveParams p) {
    const int be = blockIdx.x, hk = blockIdx.y;
    const int tid = threadIdx.x;
    const int cnt = p.evicted_cnt[be];
    if (cnt <= 0) return;
    const int n_old = p.n_valid[be] + cnt;
    const int32_t *gone = p.evicted_idx + (int64_t)be * p.max_evict;
    const int group_rows = kEvictThreads / p.row_chunks;   // rows covered by one sweep of the block
    const int pass_rows = group_rows * kMoveRows;
    const int rsub = tid / p.row_chunks, csub = tid - rsub * p.row_chunks;
    const bool lane_used = rsub < group_rows;
    char *Kb = static_cast<char *>(p.K[be]) + hk * p.stride_h_bytes + csub * 16;
    char *Vb = static_cast<char *>(p.V[be]) + hk * p.stride_h_bytes + csub * 16;

    // One bit per row of the pass: set = the row is evicted.  The list is ascending, so the
    // evicted rows of a pass are the next entries after the `run` ones already passed.
    __shared__ uint32_t flags[kMoveFlagWords];
    __shared__ int flags_before[kMoveFlagWords + 1];   // set bits in the words below; [last] = all
    int run = 0;
    for (int base = gone[0]; base < n_old; base += pass_rows) {
        if (tid < kMoveFlagWords) flags[tid] = 0u;
        __syncthreads();
        for (int x = tid; x < pass_rows; x += kEvictThreads) {
            if (run + x < cnt) {
                const int off = gone[run + x] - base;
                if (off < pass_rows) atomicOr(&flags[off >> 5], 1u << (off & 31));
            }
        }
        __syncthreads();
        if (tid < kWave) {               // the first wave ranks the 64 words
            const int mine = __popc(flags[tid]);
            int incl = mine;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const int t = __shfl_up(incl, off, kWave);
                if (tid >= off) incl += t;
            }
            flags_before[tid] = incl - mine;
            if (tid == kWave - 1) flags_before[kMoveFlagWords] = incl;
        }
        __syncthreads();
        uint4 kv[kMoveRows], vv[kMoveRows];
        int dst[kMoveRows];
#pragma unroll
        for (int r = 0; r < kMoveRows; ++r) {
            const int off = r * group_rows + rsub;
            const int row = base + off;
            dst[r] = -1;
            kv[r] = make_uint4(0, 0, 0, 0);
            vv[r] = kv[r];
            if (lane_used && row < n_old) {
                const int word = off >> 5, pos = off & 31;
                const uint32_t mine = flags[word];
                const int before = run + flags_before[word] + __popc(mine & ((1u << pos) - 1u));
                if (!((mine >> pos) & 1u) && before > 0) {
                    dst[r] = row - before;
                    kv[r] = *reinterpret_cast<const uint4 *>(Kb + row * p.stride_s_bytes);
                    vv[r] = *reinterpret_cast<const uint4 *>(Vb + row * p.stride_s_bytes);
                }
            }
        }
        const int passed = flags_before[kMoveFlagWords];
        __syncthreads();                 // every row of the pass is in registers
#pragma unroll
        for (int r = 0; r < kMoveRows; ++r) {
            if (dst[r] >= 0) {
                *reinterpret_cast<uint4 *>(Kb + dst[r] * p.stride_s_bytes) = kv[r];
                *reinterpret_cast<uint4 *>(Vb + dst[r] * p.stride_s_bytes) = vv[r];
            }
        }
        run += passed;
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
    const int row_chunks = desc_width(desc) * elem_bytes(desc->dtype) / 16;
    if (compact && (row_chunks < 1 || row_chunks > kEvictThreads)) return PIKV_ERR_UNSUPPORTED;
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
    hipLaunchKernelGGL(evict_select, dim3(desc->B * desc->E), dim3(kSelThreads), 0, st, p);
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
    m.row_chunks = row_chunks;
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
