// PiKV scheduling under bounded memory (Algorithm 1, C <- S(C, q_t); Section 3.4) and the
// constant-time insert (Algorithm 1 Insert; Section 3.1 storage invariants).
//
//   evict_select : one block per (sequence, expert).  The entries to drop are the
//                  n - capacity smallest under (utility ascending, slot descending), i.e.
//                  the complement of the `capacity` best under (utility descending, slot
//                  ascending).  A two-bits-a-step select over the order-preserving integer image
//                  of the fp32 utilities, held in registers, finds the cut value exactly
//                  (no floating-point comparison is ever redone in a different order),
//                  then one pass in slot order, driven by a block-wide prefix sum of the
//                  per-thread counts, emits the evicted slots ascending and (optionally)
//                  compacts the utilities in place.
//   evict_move   : one block per (shard, kv head, K or V, row slice) slides the kept rows down,
//                  a pass of rows at a time in ascending order (a destination never lies
//                  above its source, so holding a pass in registers before writing it is
//                  enough).
//   append_rows  : one block per (sequence, selected expert) writes the new entry.
#include "pikv_common.h"

namespace pikv {
namespace {

constexpr int kEvictThreads = 256;   // every kernel of this file
constexpr int kSelWaves = kEvictThreads / kWave;
constexpr int kSelCache = 128;       // keys a thread can keep in registers (n <= 32768);
                                     // at most 255: the digit counts of a step are bytes

struct SelShared {
    int cnt[2][3 * kSelWaves];       // per-wave digit counts of a select step, two buffers in turn
    int scan[2][kSelWaves];          // per-wave totals of a block scan, two buffers in turn
    uint64_t wave_best[kSelWaves];
};
// Both pairs of buffers are used in turn, which makes one barrier per use enough: a buffer
// is rewritten two uses later, and every wave has left the reads of use i before any wave
// passes the barrier of use i+1.

// Exclusive prefix sum of v over the block in thread order.
__device__ __forceinline__ int block_scan_excl(int v, SelShared &sh, int &turn) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int t = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += t;
    }
    int *slot = sh.scan[turn & 1];
    ++turn;
    if (lane == kWave - 1) slot[wave] = incl;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves - 1; ++w)
        if (w < wave) before += slot[w];
    return before + incl - v;
}

// Exclusive block-wide rank of a one-bit flag in thread order; *total receives the block sum.
__device__ __forceinline__ int block_rank_flag(bool flag, SelShared &sh, int &turn, int *total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const uint64_t votes = __ballot(flag);
    const int in_wave = __popcll(votes & ((1ull << lane) - 1ull));
    int *slot = sh.scan[turn & 1];
    ++turn;
    if (lane == 0) slot[wave] = __popcll(votes);
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        const int c = slot[w];
        if (w < wave) before += c;
        all += c;
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

// fp32 value whose order_key is `key` (a negative zero comes back as positive zero)
__device__ __forceinline__ float key_value(uint32_t key) {
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// Sum over the 64 lanes of a wave, returned in every lane.
__device__ __forceinline__ int wave_sum(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true);    // lane ^ 1
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true);    // lane ^ 2
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true);   // mirror within 8
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true);   // mirror within 16
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}

// The cut of the general case (drop the `ngone` worst of `n`) is the ngone-th smallest key,
// found two bits at a time from the top.  With x = key ^ prefix, the candidates whose next
// digit is below d are exactly the keys with x < d << shift, so three compares per key give
// the cumulative digit counts and the step enters the digit that holds the wanted rank.
struct CutSearch {
    uint32_t prefix = 0;
    int remaining;           // rank still to locate among the keys that match `prefix`
    int cand;                // how many keys match `prefix` on the digits decided so far
    int turn = 0;
    __device__ CutSearch(int n, int ngone) : remaining(ngone), cand(n) {}

    // c1..c3: this thread's candidates with digit < 1, < 2, < 3.  With PACKED the caller
    // promises at most 512 per thread, so a wave's totals fit 16 bits and c1, c2 travel
    // through the lane sums as one word.
    template <bool PACKED>
    __device__ __forceinline__ void step(int shift, int c1, int c2, int c3, SelShared &sh) {
        const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
        if (PACKED) {
            const int c12 = wave_sum(c1 | (c2 << 16));
            c1 = c12 & 0xffff;
            c2 = (int)((uint32_t)c12 >> 16);
        } else {
            c1 = wave_sum(c1);
            c2 = wave_sum(c2);
        }
        c3 = wave_sum(c3);
        int *slot = sh.cnt[turn & 1];
        ++turn;
        if (lane == 0) {
            slot[wave] = c1;
            slot[kSelWaves + wave] = c2;
            slot[2 * kSelWaves + wave] = c3;
        }
        __syncthreads();
        // lanes 0..11 fetch the 3 x 4 counts; quad sums leave the totals in lanes 0, 4, 8
        int v = lane < 3 * kSelWaves ? slot[lane] : 0;
        v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true);
        v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true);
        static_assert(kSelWaves == 4, "quad sums");
        const int C1 = __builtin_amdgcn_readlane(v, 0);
        const int C2 = __builtin_amdgcn_readlane(v, 4);
        const int C3 = __builtin_amdgcn_readlane(v, 8);
        if (remaining <= C1) {
            cand = C1;
        } else if (remaining <= C2) {
            prefix |= 1u << shift;
            remaining -= C1;
            cand = C2 - C1;
        } else if (remaining <= C3) {
            prefix |= 2u << shift;
            remaining -= C2;
            cand = C3 - C2;
        } else {
            prefix |= 3u << shift;
            remaining -= C3;
            cand -= C3;
        }
    }
};

// Keys in registers: thread t owns the `per` consecutive slots from t * per (per a multiple
// of 4, at most NCH), so the 16 steps touch no memory and slot order is thread order.  Slots
// past n hold the largest key: its digit is always 3, which no cumulative count includes.
template <int NCH>
__device__ __forceinline__ void select_cached(const EvictParams &p, int be, float *u, int n,
                                              int ngone, SelShared &sh) {
    const int tid = threadIdx.x;
    const int per = (n + kEvictThreads * 4 - 1) / (kEvictThreads * 4) * 4;
    const int first = tid * per;
    // The row is 16-byte aligned and S is a multiple of 4 (the caller checked), so a group
    // of four that starts below n lies inside the row; groups past n re-read the first one.
    // No branch around the loads: all of them are in flight together.
    uint32_t keys[NCH];
#pragma unroll
    for (int j0 = 0; j0 < NCH; j0 += 4) {
        const int i0 = first + j0;
        const bool any = j0 < per && i0 < n;
        const float4 v = *reinterpret_cast<const float4 *>(u + (any ? i0 : 0));
        keys[j0] = any ? order_key(v.x) : 0xffffffffu;
        keys[j0 + 1] = (any && i0 + 1 < n) ? order_key(v.y) : 0xffffffffu;
        keys[j0 + 2] = (any && i0 + 2 < n) ? order_key(v.z) : 0xffffffffu;
        keys[j0 + 3] = (any && i0 + 3 < n) ? order_key(v.w) : 0xffffffffu;
    }
    CutSearch cs(n, ngone);
    for (int shift = 30; shift >= 0; shift -= 2) {
        // One byte of `acc` per digit value; a key off the prefix has x >> shift >= 4 and is
        // counted with digit 3, which no cumulative count includes.  No compare, no carry.
        uint32_t acc = 0;
#pragma unroll
        for (int j0 = 0; j0 < NCH; j0 += 4) {
            if (j0 < per) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t digit = min((keys[j0 + t] ^ cs.prefix) >> shift, 3u);
                    acc += 1u << (digit << 3);
                }
            }
        }
        const int c1 = acc & 0xff;
        const int c2 = c1 + ((acc >> 8) & 0xff);
        const int c3 = c2 + ((acc >> 16) & 0xff);
        cs.step<true>(shift, c1, c2, c3, sh);
    }
    const uint32_t cut = cs.prefix;               // keys < cut go; of the keys == cut (`cand`
    const int keep_eq = cs.cand - cs.remaining;   // of them) the first keep_eq in slot order stay

    constexpr int kWords = (NCH + 31) / 32;
    uint32_t gone[kWords];
#pragma unroll
    for (int w = 0; w < kWords; ++w) gone[w] = 0;
    int n_eq = 0, n_gone = 0;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        const bool valid = j < per && first + j < n;
        const bool g = valid && (keys[j] < cut || (keep_eq == 0 && keys[j] == cut));
        gone[j >> 5] |= (g ? 1u : 0u) << (j & 31);
        n_gone += g;
        n_eq += valid && keys[j] == cut;
    }
    if (keep_eq > 0) {                            // ties at the cut: the earliest keep_eq stay
        int eq_rank = block_scan_excl(n_eq, sh, cs.turn);
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const bool valid = j < per && first + j < n;
            if (valid && keys[j] == cut) {
                if (eq_rank >= keep_eq) {
                    gone[j >> 5] |= 1u << (j & 31);
                    ++n_gone;
                }
                ++eq_rank;
            }
        }
    }
    int rank = block_scan_excl(n_gone, sh, cs.turn);   // evicted slots before my first slot
    int32_t *out = p.evicted_idx + (int64_t)be * p.max_evict;
    // In-place compaction is safe here: every utility is already held as a key.
#pragma unroll
    for (int j0 = 0; j0 < NCH; j0 += 4) {
        if (j0 < per) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int j = j0 + t, i = first + j;
                if (i < n) {
                    if ((gone[j >> 5] >> (j & 31)) & 1u) {
                        if (rank < p.max_evict) out[rank] = i;
                        ++rank;
                    } else if (p.compact && rank > 0) {
                        u[i - rank] = key_value(keys[j]);
                    }
                }
            }
        }
    }
}

// More keys than the registers hold: every step re-reads them (slot i = tid + j * 256).
__device__ __forceinline__ void select_stream(const EvictParams &p, int be, float *u, int n,
                                              int ngone, SelShared &sh) {
    const int tid = threadIdx.x;
    const int nchunk = (n + kEvictThreads - 1) / kEvictThreads;
    CutSearch cs(n, ngone);
    for (int shift = 30; shift >= 0; shift -= 2) {
        const uint32_t t1 = 1u << shift, t2 = 2u << shift, t3 = 3u << shift;
        int c1 = 0, c2 = 0, c3 = 0;
        for (int j = 0; j < nchunk; ++j) {
            const int i = tid + j * kEvictThreads;
            const uint32_t x = (i < n ? order_key(u[i]) : 0xffffffffu) ^ cs.prefix;
            c1 += x < t1;
            c2 += x < t2;
            c3 += x < t3;
        }
        cs.step<false>(shift, c1, c2, c3, sh);
    }
    const uint32_t cut = cs.prefix;
    const int keep_eq = cs.cand - cs.remaining;
    int32_t *out = p.evicted_idx + (int64_t)be * p.max_evict;
    int eq_seen = 0, gone_seen = 0;       // running totals over the chunks already done
    for (int j = 0; j < nchunk; ++j) {
        const int i = tid + j * kEvictThreads;
        const bool valid = i < n;
        const float ui = valid ? u[i] : 0.0f;
        const uint32_t key = order_key(ui);
        const bool is_eq = valid && key == cut, is_less = valid && key < cut;
        int eq_total, gone_total;
        const int eq_rank = eq_seen + block_rank_flag(is_eq, sh, cs.turn, &eq_total);
        const bool gone = is_less || (is_eq && eq_rank >= keep_eq);
        const int gone_before = gone_seen + block_rank_flag(gone, sh, cs.turn, &gone_total);
        if (valid) {
            if (gone) {
                if (gone_before < p.max_evict) out[gone_before] = i;
            } else if (p.compact && gone_before > 0) {
                u[i - gone_before] = ui;  // this chunk's reads ended before the barriers above
            }
        }
        eq_seen += eq_total;
        gone_seen += gone_total;
    }
}

__global__ __launch_bounds__(kEvictThreads) void evict_select(EvictParams p) {
    const int be = blockIdx.x;
    const int b = be / p.E, e = be - b * p.E;
    const int tid = threadIdx.x;

    __shared__ SelShared sh;

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
            const uint64_t c0 = evict_composite(v.x, i), c1 = evict_composite(v.y, i + 1);
            const uint64_t c2 = evict_composite(v.z, i + 2), c3 = evict_composite(v.w, i + 3);
            const uint64_t a = c0 < c1 ? c0 : c1, b2 = c2 < c3 ? c2 : c3;
            const uint64_t c = a < b2 ? a : b2;
            best = c < best ? c : best;
        }
        for (int i = n4 + tid; i < n; i += kEvictThreads) {
            const uint64_t c = evict_composite(u[i], i);
            best = c < best ? c : best;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint64_t o = __shfl_xor(best, off, kWave);
            best = o < best ? o : best;
        }
        if ((tid & (kWave - 1)) == 0) sh.wave_best[tid >> 6] = best;
        __syncthreads();
        if (tid == 0) {
            uint64_t m = sh.wave_best[0];
#pragma unroll
            for (int w = 1; w < kSelWaves; ++w) m = sh.wave_best[w] < m ? sh.wave_best[w] : m;
            p.evicted_idx[(int64_t)be * p.max_evict] = evict_composite_slot(m);
            p.evicted_cnt[be] = 1;
            p.n_valid[be] = p.capacity;
        }
        return;
    }

    // keys held per thread: the next size that covers n; beyond the largest, re-read them
    const bool vec = p.S % 4 == 0 && (reinterpret_cast<uintptr_t>(p.utility) & 15) == 0;
    if (!vec || n > kSelCache * kEvictThreads) select_stream(p, be, u, n, ngone, sh);
    else if (n <= 8 * kEvictThreads) select_cached<8>(p, be, u, n, ngone, sh);
    else if (n <= 32 * kEvictThreads) select_cached<32>(p, be, u, n, ngone, sh);
    else select_cached<kSelCache>(p, be, u, n, ngone, sh);
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
    int row_chunks;      // 16-byte chunks of a row that one block moves, 1..kEvictThreads
    int max_evict;
};

constexpr int kMoveRows = 8;                             // rows a thread carries per pass
constexpr int kMoveFlagWords = kEvictThreads * kMoveRows / 32;
static_assert(kMoveFlagWords == kWave, "one wave ranks the flag words");

__global__ __launch_bounds__(kEvictThreads) void evict_move(MoveParams p) {
    // blockIdx.z: bit 0 picks K or V, the rest picks the column slice of the row
    const int be = blockIdx.x, hk = blockIdx.y;
    const bool is_v = blockIdx.z & 1;
    const int slice = blockIdx.z >> 1;
    const int tid = threadIdx.x;
    const int cnt = p.evicted_cnt[be];
    if (cnt <= 0) return;
    const int n_old = p.n_valid[be] + cnt;
    const int32_t *gone = p.evicted_idx + (int64_t)be * p.max_evict;
    const int group_rows = kEvictThreads / p.row_chunks;   // rows covered by one sweep of the block
    const int pass_rows = group_rows * kMoveRows;
    const int rsub = tid / p.row_chunks, csub = tid - rsub * p.row_chunks;
    const bool lane_used = rsub < group_rows;
    char *Xb = static_cast<char *>(is_v ? p.V[be] : p.K[be]) + hk * p.stride_h_bytes +
               (slice * p.row_chunks + csub) * 16;

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
        uint4 held[kMoveRows];
        int dst[kMoveRows];
#pragma unroll
        for (int r = 0; r < kMoveRows; ++r) {
            const int off = r * group_rows + rsub;
            const int row = base + off;
            dst[r] = -1;
            held[r] = make_uint4(0, 0, 0, 0);
            if (lane_used && row < n_old) {
                const int word = off >> 5, pos = off & 31;
                const uint32_t mine = flags[word];
                const int before = run + flags_before[word] + __popc(mine & ((1u << pos) - 1u));
                if (!((mine >> pos) & 1u) && before > 0) {
                    dst[r] = row - before;
                    held[r] = *reinterpret_cast<const uint4 *>(Xb + row * p.stride_s_bytes);
                }
            }
        }
        const int passed = flags_before[kMoveFlagWords];
        __syncthreads();                 // every row of the pass is in registers
#pragma unroll
        for (int r = 0; r < kMoveRows; ++r) {
            if (dst[r] >= 0) *reinterpret_cast<uint4 *>(Xb + dst[r] * p.stride_s_bytes) = held[r];
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
    // K and V move in separate blocks; rows of 256 bytes or more are also cut in two slices
    const int slices = (row_chunks >= 16 && row_chunks % 2 == 0) ? 2 : 1;
    m.row_chunks = row_chunks / slices;
    m.max_evict = max_evict;
    hipLaunchKernelGGL(evict_move, dim3(desc->B * desc->E, desc->Hkv, 2 * slices),
                       dim3(kEvictThreads), 0, st, m);
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
