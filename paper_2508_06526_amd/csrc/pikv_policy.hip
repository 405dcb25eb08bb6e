// PiKV scheduling policies other than H2O (Section 3.4, Table 3 rows SL, LRU, LRU+): per-entry
// utilities formed from integer bookkeeping - the step an entry was inserted at, the step
// it was last accessed at, and how often it has been accessed - and handed to the same
// eviction (evict_select reads a utility array, whoever wrote it).
//
//   policy_stamp   : bookkeeping of the entry the next insert writes (Algorithm 1 Insert):
//                    birth = last access = now, access count 0.  One block per (sequence,
//                    selected position), same slot rule as append_rows.
//   policy_utility : one thread per live entry; reads three ints, writes one float.
//   policy_compact : after an eviction that compacted a shard, one block per shard slides the
//                    three arrays' kept entries down the same way (a pass of 256 slots at a
//                    time, read before written; a slot's shift is the number of evicted
//                    slots below it, found in the ascending list by binary search).
#include "pikv_common.h"
#include "pikv_policy_dev.h"

#include <math.h>

namespace pikv {
namespace {

constexpr int kPolicyThreads = 256;

struct StampParams {
    const int32_t *topk;
    const int32_t *reuse_idx;
    const int32_t *reuse_cnt;
    const int32_t *n_valid;
    int32_t *birth;
    int32_t *last_access;
    int32_t *freq;
    int E, S, k, max_evict, now, rows;
};

__global__ __launch_bounds__(kWave) void policy_stamp(StampParams p) {
    const int r = blockIdx.x * kWave + threadIdx.x;     // (sequence, selected position)
    if (r >= p.rows) return;
    const int b = r / p.k;
    const int e = p.topk[r];
    const int64_t be = (int64_t)b * p.E + e;
    const int n = p.n_valid[be];
    int slot = n;
    if (p.reuse_cnt && p.reuse_cnt[be] > 0) slot = p.reuse_idx[be * p.max_evict];
    if (n >= p.S || slot < 0 || slot >= p.S) return;    // full shard: the insert drops the entry
    const int64_t at = be * p.S + slot;
    p.birth[at] = p.now;
    p.last_access[at] = p.now;
    p.freq[at] = 0;
}

struct PolicyParams {
    const int32_t *n_valid;
    const float *h2o;
    float *out;
    int S, tiles;
    PolicyView v;
};

__global__ __launch_bounds__(kPolicyThreads) void policy_utility(PolicyParams p) {
    const int be = blockIdx.x / p.tiles, tile = blockIdx.x - be * p.tiles;
    const int i = tile * kPolicyThreads + threadIdx.x;
    if (i >= p.n_valid[be]) return;
    const int64_t at = (int64_t)be * p.S + i;
    p.out[at] = policy_value(p.v, at, p.h2o);
}

struct CompactParams {
    const int32_t *evicted_idx;
    const int32_t *evicted_cnt;
    const int32_t *n_valid;     // after the eviction
    int32_t *arrays[3];
    int S, max_evict;
};

__global__ __launch_bounds__(kPolicyThreads) void policy_compact(CompactParams p) {
    const int be = blockIdx.x, tid = threadIdx.x;
    const int cnt = p.evicted_cnt[be];
    if (cnt <= 0) return;
    const int n_old = p.n_valid[be] + cnt;
    const int32_t *gone = p.evicted_idx + (int64_t)be * p.max_evict;
    for (int base = gone[0]; base < n_old; base += kPolicyThreads) {   // slots below the first hole stay
        const int i = base + tid;
        int before = 0;
        bool kept = false;
        int32_t v[3] = {0, 0, 0};
        if (i < n_old) {
            int lo = 0, hi = cnt;            // number of evicted slots < i
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (gone[mid] < i) lo = mid + 1; else hi = mid;
            }
            before = lo;
            kept = !(lo < cnt && gone[lo] == i);
            if (kept)
#pragma unroll
                for (int a = 0; a < 3; ++a) v[a] = p.arrays[a][(int64_t)be * p.S + i];
        }
        __syncthreads();                     // the pass is in registers before anything moves
        if (kept && before > 0)
#pragma unroll
            for (int a = 0; a < 3; ++a) p.arrays[a][(int64_t)be * p.S + i - before] = v[a];
        __syncthreads();
    }
}

}  // namespace
}  // namespace pikv

using namespace pikv;

extern "C" int pikv_policy_compact(const pikv_desc *desc, const int32_t *evicted_idx,
                                   const int32_t *evicted_cnt, int32_t max_evict,
                                   const int32_t *n_valid, int32_t *birth, int32_t *last_access,
                                   int32_t *freq, void *stream) {
    const int rc = check_desc(desc);
    if (rc != PIKV_OK) return rc;
    if (!evicted_idx || !evicted_cnt || !n_valid || !birth || !last_access || !freq)
        return PIKV_ERR_INVALID;
    if (max_evict < 1) return PIKV_ERR_INVALID;
    if (desc->B == 0) return PIKV_OK;
    CompactParams p;
    p.evicted_idx = evicted_idx;
    p.evicted_cnt = evicted_cnt;
    p.n_valid = n_valid;
    p.arrays[0] = birth;
    p.arrays[1] = last_access;
    p.arrays[2] = freq;
    p.S = desc->S;
    p.max_evict = max_evict;
    hipLaunchKernelGGL(policy_compact, dim3(desc->B * desc->E), dim3(kPolicyThreads), 0,
                       as_stream(stream), p);
    return launch_status();
}

extern "C" int pikv_policy_stamp(const pikv_desc *desc, const int32_t *topk_idx, int32_t k,
                                 const int32_t *reuse_idx, const int32_t *reuse_cnt,
                                 int32_t max_evict, const int32_t *n_valid, int32_t now,
                                 int32_t *birth, int32_t *last_access, int32_t *freq,
                                 void *stream) {
    const int rc = check_desc(desc);
    if (rc != PIKV_OK) return rc;
    if (!topk_idx || !n_valid || !birth || !last_access || !freq) return PIKV_ERR_INVALID;
    if (k < 1 || k > desc->E) return PIKV_ERR_INVALID;
    if ((reuse_idx == nullptr) != (reuse_cnt == nullptr)) return PIKV_ERR_INVALID;
    if (reuse_idx && max_evict < 1) return PIKV_ERR_INVALID;
    if (desc->route_rows_per_seq != 1) return PIKV_ERR_UNSUPPORTED;   // one insert per sequence
    if (desc->B == 0) return PIKV_OK;
    StampParams p;
    p.topk = topk_idx;
    p.reuse_idx = reuse_idx;
    p.reuse_cnt = reuse_cnt;
    p.n_valid = n_valid;
    p.birth = birth;
    p.last_access = last_access;
    p.freq = freq;
    p.E = desc->E;
    p.S = desc->S;
    p.k = k;
    p.max_evict = max_evict;
    p.now = now;
    p.rows = desc->B * k;
    hipLaunchKernelGGL(policy_stamp, dim3((p.rows + kWave - 1) / kWave), dim3(kWave), 0,
                       as_stream(stream), p);
    return launch_status();
}

extern "C" int pikv_policy_utility(const pikv_desc *desc, int32_t policy, const int32_t *n_valid,
                                   int32_t now, float lambda, int32_t window, int32_t protect,
                                   const int32_t *birth, const int32_t *last_access,
                                   const int32_t *freq, const float *h2o, float *out,
                                   void *stream) {
    const int rc = check_desc(desc);
    if (rc != PIKV_OK) return rc;
    if (!n_valid || !out) return PIKV_ERR_INVALID;
    const int prc = check_policy(policy, window, protect, lambda, birth, last_access, freq, h2o);
    if (prc != PIKV_OK) return prc;
    if (desc->B == 0) return PIKV_OK;
    PolicyParams p;
    p.n_valid = n_valid;
    p.h2o = h2o;
    p.out = out;
    p.S = desc->S;
    p.tiles = (desc->S + kPolicyThreads - 1) / kPolicyThreads;
    p.v.policy = policy;
    p.v.now = now;
    p.v.window = window;
    p.v.protect = protect;
    p.v.lambda = lambda;
    p.v.threshold = 0.0f;
    p.v.birth = const_cast<int32_t *>(birth);
    p.v.last_access = const_cast<int32_t *>(last_access);
    p.v.freq = const_cast<int32_t *>(freq);
    const int64_t blocks = (int64_t)desc->B * desc->E * p.tiles;
    if (blocks > 0x7fffffff) return PIKV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(policy_utility, dim3((unsigned)blocks), dim3(kPolicyThreads), 0,
                       as_stream(stream), p);
    return launch_status();
}
