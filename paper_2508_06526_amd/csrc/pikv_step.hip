// One decode step of PiKV's hot path as three launches (Algorithm 1, one iteration of the
// loop: route, insert the new entry under bounded memory, attend, score):
//
//   step_pre   : per (sequence, selected position), a 1024-thread block routes the query
//                (Section 3.2), then for its selected shard evicts the minimum-utility entry
//                if the shard is full (Section 3.4) and inserts the new token's K/V rows in
//                O(1) (Section 3.1).  Everything that depends only on the selected expert id
//                (entry count, table pointers, the shard's utilities) is fetched in one round
//                trip; the new rows are fetched before the router result exists.
//   attention  : the split flash-decode pass over the selected shards (pikv_attn.hip).
//   step_post  : merge of the split partials with the router gates and the utility update
//                u <- decay * u + attention mass (Section 3.4, Table 3 H2O), in one launch.
//
// With a scheduling policy (Table 3 rows SL, LRU, LRU+) step_pre takes its minimum over the
// policy's value, computed on the fly from the per-entry stamps and counts, and stamps the
// new entry; step_post marks the entries whose attention mass exceeds the access threshold.
//
// On MI355X even an empty kernel occupies the queue for ~1.5 us and each small kernel is a
// chain of dependent memory round trips; six launches cost more in dispatch and latency than
// in work next to a ~20 us attention pass.  The step is defined as exactly the sequence of
// the separate C-ABI calls and shares every reduction order with them (bit-identical).
#include "pikv_common.h"
#include "pikv_combine_dev.h"
#include "pikv_route_dev.h"
#include "pikv_policy_dev.h"
#include "pikv_penalty_dev.h"

namespace pikv {
namespace {

struct PreParams {
    const void *x;
    const void *W_r;
    const float *bias;
    int32_t *topk;
    float *gates;
    const void *K_new;
    const void *V_new;
    void *const *K;
    void *const *V;
    float *utility;
    int32_t *n_valid;
    int32_t *evicted_idx;
    int32_t *evicted_cnt;
    int64_t stride_h_bytes, stride_s_bytes;
    int64_t x_stride;    // elements between the routed vectors of consecutive sequences (>= d_r)
    int d_r, E, cpr, k, S, Hkv, row_chunks, do_insert;
    int EP;              // 0: rows of W_r are aligned 16-byte chunks (cpr of them); else E rounded up to a power of two
    int use_policy;      // the entry to evict is chosen by pol (Table 3) instead of the utility
    PolicyView pol;      // its arrays, when given, are also stamped for the new entry
};

// Minimum of a 64-bit key over the wavefront, every lane ends with it; the four low lane bits
// are exchanged inside the 16-lane rows (no LDS traffic).
__device__ __forceinline__ uint64_t wave_min_u64(uint64_t v) {
    auto step = [&](auto bit) {
        constexpr int BIT = decltype(bit)::value;
        const uint32_t lo = __float_as_uint(lane_xchg<BIT>(__uint_as_float((uint32_t)v)));
        const uint32_t hi = __float_as_uint(lane_xchg<BIT>(__uint_as_float((uint32_t)(v >> 32))));
        const uint64_t o = ((uint64_t)hi << 32) | lo;
        v = o < v ? o : v;
    };
    step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{});
    step(std::integral_constant<int, 3>{});
    step(std::integral_constant<int, 4>{});
    step(std::integral_constant<int, 5>{});
    return v;
}

// Grid: (sequence b, selected position j).  Every block of a sequence recomputes the routing
// decision (W_r is L2-resident and tiny next to the cache) so that the k evict/insert jobs
// run on k compute units at once instead of one after the other; block j == 0 publishes the
// decision.
template <typename T>
__global__ __launch_bounds__(kRouteThreads) void step_pre(PreParams p) {
    constexpr int kWaves = kRouteThreads / kWave;
    const int b = blockIdx.x / p.k, j = blockIdx.x - b * p.k;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;

    __shared__ float red[kWaves][64];
    __shared__ uint64_t wave_best[kWaves];

    // neither the router's additive term, nor the entry counts of the sequence's shards (lane e
    // takes shard e's; the selected one is picked out of the register once the router has
    // spoken), nor the new rows depend on anything: requested now
    const float bias_e = route_bias_of_lane(p.bias, p.E, lane);
    const int n_of_lane = p.n_valid[(int64_t)b * p.E + min(lane, p.E - 1)];
    const int new_chunks = p.Hkv * p.row_chunks;
    uint4 knew = make_uint4(0, 0, 0, 0), vnew = knew;
    if (p.do_insert && tid < new_chunks) {
        knew = load16(static_cast<const char *>(p.K_new) + ((int64_t)b * new_chunks + tid) * 16);
        vnew = load16(static_cast<const char *>(p.V_new) + ((int64_t)b * new_chunks + tid) * 16);
    }

    if (p.EP == 0)
        route_logits_vec<T>(static_cast<const T *>(p.x) + (int64_t)b * p.x_stride,
                            static_cast<const T *>(p.W_r), p.bias, p.d_r, p.E, p.cpr, red);
    else      // any E, any alignment: the stand-alone router's generic form, same bits
        route_logits_generic<T>(static_cast<const T *>(p.x) + (int64_t)b * p.x_stride,
                                static_cast<const T *>(p.W_r), p.d_r, p.E, p.EP, &red[0][0]);
    // The first wave ranks the experts and tells the others which shard is the block's (one LDS
    // word and a barrier): sixteen waves doing it side by side, four to a SIMD, take twice as
    // long as one wave alone plus the barrier.  The ranks come first - the shard to scan hangs
    // off them alone - and the softmax and the gates are formed, by that wave of the sequence's
    // first block, while the scan's requests are in flight.
    __shared__ int block_expert;
    float logit = 0.0f;
    int rank = 64;
    if (wave == 0) {
        logit = p.EP == 0 ? route_logit_of_lane(red, bias_e, p.E, lane)
                          : route_logit_generic_of_lane(&red[0][0], bias_e, p.E, lane);
        rank = route_rank(logit, lane, p.E);
        const uint64_t owner = __ballot(rank == j);      // taken with every lane of the wave active
        if (lane == 0) block_expert = __builtin_ctzll(owner);
    }
    auto publish = [&]() {
        if (j == 0 && wave == 0) route_gates(logit, rank, lane, b, p.E, p.k, p.topk, p.gates, nullptr);
    };
    if (!p.do_insert) {
        publish();
        return;
    }
    __syncthreads();
    const int e = __builtin_amdgcn_readfirstlane(block_expert);
    const int n = __builtin_amdgcn_readlane(n_of_lane, e);
    const int64_t be = (int64_t)b * p.E + e;
    char *Kd = static_cast<char *>(p.K[be]);
    char *Vd = static_cast<char *>(p.V[be]);
    const float *u = p.utility + be * p.S;
    uint64_t best = ~0ull;
    if (p.use_policy) {
        publish();
        if (policy_vec_ok(p.pol, p.utility, p.S)) {
            for (int i = tid * 4; i < p.S; i += kRouteThreads * 4) {
                float v[4];
                policy_value4(p.pol, be * p.S + i, p.utility, v);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint64_t c0 = evict_composite(v[t], i + t);
                    best = c0 < best ? c0 : best;
                }
            }
        } else {
            for (int i = tid; i < p.S; i += kRouteThreads) {
                const uint64_t c0 = evict_composite(policy_value(p.pol, be * p.S + i, p.utility), i);
                best = c0 < best ? c0 : best;
            }
        }
    } else if ((p.S & 3) == 0) {
        // two 16-byte loads per thread and pass, both requested before either is used: up to
        // 8192 slots are one trip to memory, not one per 4096
        // (the first pass's requests are in flight while the gates are formed and published)
        constexpr int kScanLoads = 2;
        float4 v[kScanLoads];
        auto request = [&](int i0) {
#pragma unroll
            for (int t = 0; t < kScanLoads; ++t) {
                const int i = i0 + t * kRouteThreads * 4;
                v[t] = i < p.S ? *reinterpret_cast<const float4 *>(u + i) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        };
        request(tid * 4);
        publish();
        for (int i0 = tid * 4; i0 < p.S; i0 += kRouteThreads * 4 * kScanLoads) {
            if (i0 != tid * 4) request(i0);
            // The block's 16 waves share 4 vector units, so this phase costs its instruction
            // count times 16 cycles.  Where no value of the wave has its sign bit set (utilities
            // are sums of probabilities), the keys' order is the order of the raw bits and the
            // thread's slots ascend: one compare and two selects per value ("<=": of equal
            // values the higher slot goes) instead of building and comparing 64-bit composites
            // - the same minimum.  (Loads past the shard's end hold zeros and are left out; the
            // thread's first load is always inside.)
            uint32_t signs = 0;
#pragma unroll
            for (int t = 0; t < kScanLoads; ++t)
                signs |= (__float_as_uint(v[t].x) | __float_as_uint(v[t].y)) |
                         (__float_as_uint(v[t].z) | __float_as_uint(v[t].w));
            if (!__any((int)signs < 0)) {
                uint32_t low = 0xffffffffu;
                int at = 0;              // offset of the lowest value's slot from i0
                auto take = [&](bool inside, float value, int offset) {
                    const uint32_t bits = __float_as_uint(value);
                    const bool le = inside && bits <= low;
                    low = le ? bits : low;
                    at = le ? offset : at;
                };
#pragma unroll
                for (int t = 0; t < kScanLoads; ++t) {
                    const bool inside = i0 + t * kRouteThreads * 4 < p.S;
                    take(inside, v[t].x, t * kRouteThreads * 4);
                    take(inside, v[t].y, t * kRouteThreads * 4 + 1);
                    take(inside, v[t].z, t * kRouteThreads * 4 + 2);
                    take(inside, v[t].w, t * kRouteThreads * 4 + 3);
                }
                const uint64_t c0 = evict_composite(__uint_as_float(low), i0 + at);
                best = c0 < best ? c0 : best;
                continue;
            }
#pragma unroll
            for (int t = 0; t < kScanLoads; ++t) {
                const int i = i0 + t * kRouteThreads * 4;
                if (i < p.S) {
                    uint64_t c0 = evict_composite(v[t].x, i), c1 = evict_composite(v[t].y, i + 1);
                    uint64_t c2 = evict_composite(v[t].z, i + 2), c3 = evict_composite(v[t].w, i + 3);
                    c0 = c0 < c1 ? c0 : c1;
                    c2 = c2 < c3 ? c2 : c3;
                    c0 = c0 < c2 ? c0 : c2;
                    best = c0 < best ? c0 : best;
                }
            }
        }
    } else {
        publish();
        for (int i = tid; i < p.S; i += kRouteThreads) {
            const uint64_t c0 = evict_composite(u[i], i);
            best = c0 < best ? c0 : best;
        }
    }
    best = wave_min_u64(best);
    if (lane == 0) wave_best[wave] = best;
    __syncthreads();
    // what is left - the new rows and the bookkeeping - takes the block's first waves only: the
    // others leave, and with them their share of the SIMDs' issue slots
    if (wave != 0 && wave * kWave >= new_chunks) return;
    static_assert(kWaves <= 16, "one LDS word per lane of a row");
    uint64_t m = wave_min_u64(wave_best[lane & (kWaves - 1)]);
    const bool full = n >= p.S;
    const int slot = full ? evict_composite_slot(m) : n;

    // insert the new entry's rows (one 16-byte chunk per thread and pass)
    Kd += slot * p.stride_s_bytes;
    Vd += slot * p.stride_s_bytes;
    for (int idx = tid; idx < new_chunks; idx += kRouteThreads) {
        uint4 kv = knew, vv = vnew;
        if (idx >= kRouteThreads) {
            kv = load16(static_cast<const char *>(p.K_new) + ((int64_t)b * new_chunks + idx) * 16);
            vv = load16(static_cast<const char *>(p.V_new) + ((int64_t)b * new_chunks + idx) * 16);
        }
        const int hk = idx / p.row_chunks, cc = idx - hk * p.row_chunks;
        *reinterpret_cast<uint4 *>(Kd + hk * p.stride_h_bytes + cc * 16) = kv;
        *reinterpret_cast<uint4 *>(Vd + hk * p.stride_h_bytes + cc * 16) = vv;
    }
    if (tid == 0) {
        if (full) p.evicted_idx[be] = slot;
        p.evicted_cnt[be] = full ? 1 : 0;
        p.utility[be * p.S + slot] = 0.0f;
        p.n_valid[be] = full ? p.S : n + 1;
        // the new entry's bookkeeping (Algorithm 1 Insert)
        if (p.pol.birth) p.pol.birth[be * p.S + slot] = p.pol.now;
        if (p.pol.last_access) p.pol.last_access[be * p.S + slot] = p.pol.now;
        if (p.pol.freq) p.pol.freq[be * p.S + slot] = 0;
    }
    // experts nobody selected report "nothing evicted" (block 0 of the sequence)
    if (j == 0 && tid < p.E && rank >= p.k) p.evicted_cnt[(int64_t)b * p.E + tid] = 0;
}

// Post-attention stage of the fused step: the merge of the split partials (one block per
// query head, as in the stand-alone combine kernel) and the utility update in ONE launch.
// A utility block (256 slots of a visited shard x 4 groups of heads) cannot wait for the merge
// blocks, so it recomputes the per-head softmax statistics itself from the (max, sum) pairs of
// the partials - a few KiB from L2 and the same arithmetic, hence the same bits - while its
// score loads are already in flight.
constexpr int kPostMaxShards = 2048;   // Hq * k
// From this many query rows per sequence on (a multi-query step of 8 drafts x 32 heads) the merge
// and the utility update run as two launches: every utility block of the single launch re-derives
// the statistics of all Hq * k (head, shard) pairs from their partials - 128 KiB per block at 256
// rows and 4 shards - while the stand-alone utility kernel reads the merge's (shift, coef) pairs.
// Measured, 256 rows: 18.2 us in one launch, 5.3 + 9.4 us in two; 128 rows: 11.4 us either way.
constexpr int kPostSplitRows = 256;
constexpr int kPostPrefetchHeads = 8;  // score loads each thread issues before the statistics
constexpr int kPostMaxTiles = 8;       // slot tiles one utility block walks through
constexpr int kPostStatsAhead = 4;     // many-pairs shape: passes of statistics whose loads are in flight
// Shapes of the kernel (template MODE): one slot tile per utility block and straight-line code;
// several tiles per block; many (head, shard) pairs or many heads per thread.
constexpr int kPostSingle = 0, kPostMulti = 1, kPostMany = 2;

struct PostParams {
    CombineParams c;
    const float *scores;
    const int32_t *n_valid;
    const int32_t *topk;
    float *utility;
    int B, E, S;
    int tiles;            // utility blocks per selected shard
    int tiles_per_block;  // consecutive slot tiles each of them covers
    int util_first;       // the utility blocks take the grid's first block ids (they start first)
    float decay;
    int track;            // access bookkeeping: mass above pol.threshold stamps and counts the entry
    PolicyView pol;
    int small_scores;     // Hq * k * S < 2^31: a sequence's scores are addressed with 32-bit offsets
    int feedback;         // the grid's last block runs the router's penalty update (fb)
    PenaltyParams fb;
};

// LDS of a utility block: statistics of the Hq * k (head, shard) pairs, the gates, and two
// buffers of per-(head group, slot) sums used in turn.
inline __host__ __device__ int post_pairs_pad(int pairs) { return (pairs + 3) & ~3; }
inline size_t post_smem_bytes(int threads, int np, int pairs) {
    const size_t util = (size_t)(4 * post_pairs_pad(pairs) + 64 + 2 * threads) * 4;
    const size_t comb = combine_smem_bytes(threads, np);
    return util > comb ? util : comb;
}

// B*Hq blocks merge one query head each (the grid's first ids, or with util_first those after
// the utility blocks); the others update the utilities of
// tiles_per_block tiles of THREADS/4 slots of the j-th selected shard of a sequence.  THREADS
// is the merge's block size (combine_threads), so that the merge is bit-identical to the
// stand-alone kernel.
template <typename T, int THREADS, int MODE>
__global__ __launch_bounds__(THREADS) void step_post(PostParams p) {
    constexpr int kSlots = THREADS / 4;
    const int ntiles = MODE != kPostSingle ? p.tiles_per_block : 1;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // post_smem_bytes()
    const int Hq = p.c.Hq, k = p.c.k, nsplit = p.c.nsplit;
    const int ncomb = p.B * Hq;
    // Blocks are dispatched in id order.  With hundreds of query rows the utility blocks are
    // the long ones and a CU holds one block of either kind: they then take the first ids,
    // so that they do not queue behind the merge blocks (kPostMany only).
    const bool util_first = MODE == kPostMany && p.util_first;
    const int mb = util_first ? (int)blockIdx.x - p.B * k * p.tiles : (int)blockIdx.x;
    if (mb >= 0 && mb < ncomb) {
        combine_head<T, THREADS>(p.c, mb, smem);
        return;
    }
    if (p.feedback && blockIdx.x == gridDim.x - 1) {   // Table 1 penalty for the next step
        if (threadIdx.x < kWave) penalty_wave(p.fb, threadIdx.x);
        return;
    }
    const int np = k * nsplit;
    int bid = util_first ? (int)blockIdx.x : (int)blockIdx.x - ncomb;
    const int tile = bid % p.tiles;
    bid /= p.tiles;
    const int j = bid % k;
    const int b = bid / k;
    const int tid = threadIdx.x;
    // Order of the requests: loads come back in the order they were issued, a value the
    // compiler knows to be the same in all lanes is waited for where it is loaded (it goes to a
    // scalar register at once), and nothing that is needed early may queue behind something
    // slow.  So the sequence's selections, entry counts and gates are read one per lane, first
    // (lane l takes selection l, shard l's count and gate l; the block's own are picked out of
    // the registers after the statistics); then the (max, sum) pairs of the statistics; then
    // the scores - a trip to memory, with the shard's capacity as the bound: slots past the
    // entry count are masked when they are used, and a block past the shard's end leaves after
    // the statistics.
    const int lane_id = tid & (kWave - 1);
    const int sel_of_lane = p.topk[(int64_t)b * k + min(lane_id, k - 1)];
    const int n_of_lane = p.n_valid[(int64_t)b * p.E + min(lane_id, p.E - 1)];
    const float gate_of_thread = (p.c.gates != nullptr && tid < k) ? p.c.gates[(int64_t)b * k + tid] : 1.0f;
    const int i0 = tile * kSlots * ntiles;

    const int pairs = post_pairs_pad(Hq * k);
    float *Mj_s = reinterpret_cast<float *>(smem), *Zj_s = Mj_s + pairs;
    float *shift_s = Zj_s + pairs, *coef_s = shift_s + pairs;
    float *g_s = coef_s + pairs;               // [64]
    float *part_s = g_s + 64;                  // [2][4][kSlots]

    // thread = (slot, head group); the heads are cut into 4 consecutive groups, each summed in
    // ascending order, the groups joined as (g0 + g1) + (g2 + g3) - the order the stand-alone
    // utility kernel uses too
    const int slot = tid & (kSlots - 1), hg = tid / kSlots;
    const int gsize = (Hq + 3) / 4;
    const int h_lo = hg * gsize, h_hi = min(Hq, h_lo + gsize);
    float sc[kPostPrefetchHeads];
    // (unconditional loads from clamped, always valid addresses: heads past the group's end and
    // slots past the limit are masked where the values are used.  Loads under a lane-dependent
    // branch would make every later wait a wait for ALL loads in flight.)
    // Addresses = the sequence's block of scores (one 64-bit base, the same in every thread) plus
    // 32-bit element offsets built with adds and selects: as eight independent 64-bit products
    // they took some 130 instructions per wave, many of them quarter-rate multiplies, in front of
    // the block's first requests - and a block's 16 waves issue four to a SIMD, one after another.
    // (p.small_scores: a sequence's scores span less than 2^31 elements; else the long form.)
    const float *seq_scores = p.scores + (int64_t)b * Hq * k * p.S;
    const int h_first = min(h_lo, Hq - 1), t_last = Hq - 1 - h_first;
    const uint32_t kS = (uint32_t)k * (uint32_t)p.S;
    const uint32_t off_first = ((uint32_t)h_first * (uint32_t)k + (uint32_t)j) * (uint32_t)p.S;
    const uint32_t off_last = off_first + (uint32_t)t_last * kS;
    auto fetch = [&](int i, int limit, bool first) {
        const int ic = min(i, limit - 1);
        // (the later tiles' requests keep the long form: its bases are set up once, after the
        // first requests have gone out, and a tile then costs one add per head; the shape with
        // several tiles per block keeps it throughout - there both forms side by side measured
        // 0.5-0.9 us slower on the streaming workload)
        if (MODE != kPostMulti && first && p.small_scores) {  // block-uniform
#pragma unroll
            for (int t = 0; t < kPostPrefetchHeads; ++t) {
                const uint32_t off = (t < t_last ? off_first + (uint32_t)t * kS : off_last) + (uint32_t)ic;
                sc[t] = seq_scores[off];
            }
        } else {
#pragma unroll
            for (int t = 0; t < kPostPrefetchHeads; ++t) {
                const int h = min(h_lo + t, Hq - 1);
                sc[t] = p.scores[(((int64_t)b * Hq + h) * k + j) * p.S + ic];
            }
        }
    };
    int i = i0 + slot;
    // softmax statistics of every (head, selected shard): 8 lanes each, pairs read from L2.  The
    // pairs of the first pass are requested before the scores: loads come back in order, and the
    // statistics must not wait for the scores' trip to memory
    const float *ml = p.c.part_ml + (int64_t)b * Hq * np * 2;
    const int pair0 = tid / 8;
    auto pair_of = [&](int t) {
        return [=](int sp) { return *reinterpret_cast<const float2 *>(ml + 2 * ((int64_t)t * nsplit + sp)); };
    };
    // With more pairs than groups of 8 lanes the statistics take several passes (kPostMany: 8
    // at 256 rows and 4 shards), each a round trip to L2 if taken one after the other: the
    // pairs of kPostStatsAhead passes are requested ahead, and a pass that is done requests
    // those of the pass kPostStatsAhead later.
    constexpr int kAhead = MODE == kPostMany ? kPostStatsAhead : 1;
    constexpr int kPairsPerPass = THREADS / 8;
    const int npairs = Hq * k;
    auto load_pass = [&](int pass) {
        const int t = pass * kPairsPerPass + pair0;
        return shard_pairs_load(t < npairs ? nsplit : 0, tid & 7, pair_of(min(t, npairs - 1)));
    };
    ShardPairs held[kAhead];
#pragma unroll
    for (int a = 0; a < kAhead; ++a) held[a] = load_pass(a);
    fetch(i, p.S, true);

    const int passes = (npairs + kPairsPerPass - 1) / kPairsPerPass;
    for (int pass0 = 0; pass0 < passes; pass0 += kAhead) {
#pragma unroll
        for (int a = 0; a < kAhead; ++a) {
            const int pass = pass0 + a;
            if (pass < passes) {                 // block-uniform
                const int t = pass * kPairsPerPass + pair0;
                const bool real = t < npairs;
                float M, Z;
                if (MODE == kPostMany || pass == 0)
                    shard_stats8(held[a], real ? nsplit : 0, tid & 7, pair_of(t), &M, &Z);
                else
                    shard_stats8(real ? nsplit : 0, tid & 7, pair_of(t), &M, &Z);
                if (real && (tid & 7) == 0) {
                    Mj_s[t] = M;
                    Zj_s[t] = Z;
                }
                if (MODE == kPostMany && pass + kAhead < passes) held[a] = load_pass(pass + kAhead);
            }
        }
    }
    const int e = __builtin_amdgcn_readlane(sel_of_lane, j);
    const int n = __builtin_amdgcn_readlane(n_of_lane, e);
    if (i0 >= n) return;     // block-uniform: no entries in this block's slots
    float *urow = p.utility + ((int64_t)b * p.E + e) * p.S;
    float u_old = (i < n && hg == 0) ? urow[i] : 0.0f;
    if (p.c.gates != nullptr && tid < k) g_s[tid] = gate_of_thread;
    __syncthreads();
    // (shift, coef) of every (head, shard) pair: an aligned group of kp lanes per head
    const int kp = pow2_at_least(k);
    for (int h0 = 0; h0 < Hq; h0 += THREADS / kp) {
        const int h = h0 + tid / kp, jj = tid & (kp - 1);
        // a wave holds 64 / kp whole heads: one whose first head is past the end has nothing to
        // do and leaves the SIMD to the waves that have (wave-uniform branch)
        if (__builtin_amdgcn_readfirstlane(h) >= Hq) break;
        const bool mine = h < Hq && jj < k;
        const HeadWeights hw = head_weights(kp, mine ? Mj_s[h * k + jj] : 0.0f, mine ? Zj_s[h * k + jj] : 0.0f,
                                            (mine && p.c.gates) ? g_s[jj] : 1.0f, p.c.combine);
        if (mine) {
            shift_s[h * k + jj] = hw.shift;
            coef_s[h * k + jj] = hw.coef;
        }
    }
    __syncthreads();
    for (int it = 0; it < ntiles; ++it) {
        const bool live = i < n;
        float a = 0.0f;
        // the prefetched heads, without branches: the group's head range is the same in the whole
        // wave (a scalar compare picks the sum or leaves it), heads past its end read a clamped,
        // valid pair, and lanes past the entry count compute on their clamped scores for nothing
        const int held_heads = __builtin_amdgcn_readfirstlane(h_hi - h_lo);
#pragma unroll
        for (int t = 0; t < kPostPrefetchHeads; ++t) {
            const int h = min(h_lo + t, Hq - 1);
            const float with = fmaf(coef_s[h * k + j], __expf(sc[t] - shift_s[h * k + j]), a);
            a = t < held_heads ? with : a;
        }
        if (live) {
            // more heads per group than were prefetched: batches of loads, same ascending order
            for (int hb = h_lo + kPostPrefetchHeads; hb < h_hi; hb += kPostPrefetchHeads) {
                float more[kPostPrefetchHeads];
#pragma unroll
                for (int t = 0; t < kPostPrefetchHeads; ++t)
                    more[t] = hb + t < h_hi ? p.scores[(((int64_t)b * Hq + hb + t) * k + j) * p.S + i] : 0.0f;
#pragma unroll
                for (int t = 0; t < kPostPrefetchHeads; ++t) {
                    const int h = hb + t;
                    if (h < h_hi) a = fmaf(coef_s[h * k + j], __expf(more[t] - shift_s[h * k + j]), a);
                }
            }
        }
        // the next tile's loads go out before this tile's sums meet in LDS
        const int i_next = i + kSlots;
        const float u_cur = u_old;
        if (it + 1 < ntiles) {
            fetch(i_next, n, false);
            u_old = (i_next < n && hg == 0) ? urow[i_next] : 0.0f;
        }
        float *part = part_s + (it & 1) * 4 * kSlots;    // rewritten two tiles later, after a barrier
        part[hg * kSlots + slot] = a;
        __syncthreads();
        if (hg == 0 && live) {
            const float total = (part[slot] + part[kSlots + slot]) +
                                (part[2 * kSlots + slot] + part[3 * kSlots + slot]);
            urow[i] = fmaf(p.decay, u_cur, total);
            if (p.track && total > p.pol.threshold) {
                const int64_t at = ((int64_t)b * p.E + e) * p.S + i;
                p.pol.last_access[at] = p.pol.now;
                p.pol.freq[at] += 1;
            }
        }
        i = i_next;
    }
}

}  // namespace
}  // namespace pikv

using namespace pikv;

static int decode_step(const pikv_desc *desc, const void *q, const void *W_r, const float *bias,
                       const void *K_new, const void *V_new, void *const *K_shards,
                       void *const *V_shards, const void *U_K, const void *U_V, int32_t *n_valid,
                       float *utility, int32_t k, int32_t combine, float scale, float decay,
                       int32_t *topk_idx, float *gates, int32_t *evicted_idx, int32_t *evicted_cnt,
                       float *y, float *row_max, float *row_norm, float *scores, float *slot_coef,
                       void *workspace, size_t workspace_bytes, void *stream,
                       const pikv_policy_args *pa, const pikv_router_feedback *fb) {
    const int rc = check_desc(desc);
    if (rc != PIKV_OK) return rc;
    PolicyView pol = {};
    bool use_policy = false, track = false;
    if (pa != nullptr) {
        const int prc = check_policy(pa->policy, pa->window, pa->protect, pa->lambda, pa->birth,
                                     pa->last_access, pa->freq, utility);
        if (prc != PIKV_OK) return prc;
        track = pa->last_access != nullptr && pa->freq != nullptr;
        if (track && !(pa->threshold >= 0.0f)) return PIKV_ERR_INVALID;
        pol.policy = pa->policy;
        pol.now = pa->now;
        pol.window = pa->window;
        pol.protect = pa->protect;
        pol.lambda = pa->lambda;
        pol.threshold = pa->threshold;
        pol.birth = pa->birth;
        pol.last_access = pa->last_access;
        pol.freq = pa->freq;
        use_policy = pa->policy != PIKV_POLICY_H2O || pa->protect > 0;
    }
    if (!q || !W_r || !K_shards || !V_shards || !n_valid || !utility || !topk_idx || !gates || !y ||
        !scores || !slot_coef)
        return PIKV_ERR_INVALID;
    PenaltyParams pen = {};
    if (fb != nullptr) {
        const int frc = check_penalty(fb->mode, fb->load, fb->miss, fb->coef, fb->bias, desc->E);
        if (frc != PIKV_OK) return frc;
        pen.mode = fb->mode;
        pen.topk = topk_idx;
        pen.n_sel = desc->B * k;
        pen.E = desc->E;
        pen.load = fb->load;
        pen.miss = fb->miss;
        pen.coef = fb->coef;
        pen.bias = fb->bias;
    }
    if ((K_new == nullptr) != (V_new == nullptr)) return PIKV_ERR_INVALID;
    if (K_new && (!evicted_idx || !evicted_cnt)) return PIKV_ERR_INVALID;
    if (k < 1 || k > desc->E) return PIKV_ERR_INVALID;
    if (!(decay >= 0.0f) || decay > 3.0e38f) return PIKV_ERR_INVALID;
    if (combine != PIKV_COMBINE_LSE && combine != PIKV_COMBINE_LOCAL) return PIKV_ERR_INVALID;
    if (desc->route_rows_per_seq != 1) return PIKV_ERR_UNSUPPORTED;
    int cpr = 0, EP = 0;
    if (!route_vec_ok(W_r, desc->E, desc->dtype, &cpr)) {
        EP = 1;
        while (EP < desc->E) EP <<= 1;
    }
    // the attention pass's own checks come before the first launch as well: a rejected call
    // leaves the cache (rows, utilities, entry counts, policy arrays) exactly as it was
    AttnPlan checked;
    const int arc = check_attn_args(desc, q, K_shards, V_shards, U_K, U_V, n_valid, topk_idx, k, combine,
                                    scale, y, workspace, workspace_bytes, &checked);
    if (arc != PIKV_OK) return arc;
    hipStream_t st = as_stream(stream);
    if (profile_events_set()) {
        // an event record inside a captured graph would replay with every launch of the graph
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cs) != hipSuccess) return PIKV_ERR_HIP;
        if (cs != hipStreamCaptureStatusNone) return PIKV_ERR_INVALID;
    }
    if (desc->B == 0) return PIKV_OK;

    PreParams p;
    p.x = q;
    p.W_r = W_r;
    p.bias = bias;
    p.topk = topk_idx;
    p.gates = gates;
    p.K_new = K_new;
    p.V_new = V_new;
    p.K = K_shards;
    p.V = V_shards;
    p.utility = utility;
    p.n_valid = n_valid;
    p.evicted_idx = evicted_idx;
    p.evicted_cnt = evicted_cnt;
    const int eb = elem_bytes(desc->dtype);
    p.stride_h_bytes = desc->stride_h * eb;
    p.stride_s_bytes = desc->stride_s * eb;
    // a multi-query step is routed by its first query alone: the leading d_r values of q[b]
    const int tq = desc->tq > 1 ? desc->tq : 1;
    if (desc->Hq % tq != 0) return PIKV_ERR_UNSUPPORTED;
    p.d_r = desc->Hq / tq * desc->D;
    p.x_stride = (int64_t)desc->Hq * desc->D;
    p.E = desc->E;
    p.cpr = cpr;
    p.EP = EP;
    p.k = k;
    p.S = desc->S;
    p.Hkv = desc->Hkv;
    p.row_chunks = desc_width(desc) * eb / 16;
    p.do_insert = K_new != nullptr;
    p.use_policy = use_policy;
    p.pol = pol;
    if (desc->dtype == PIKV_F32)
        hipLaunchKernelGGL(step_pre<float>, dim3(desc->B * k), dim3(kRouteThreads), 0, st, p);
    else
        hipLaunchKernelGGL(step_pre<bf16>, dim3(desc->B * k), dim3(kRouteThreads), 0, st, p);
    int lrc = launch_status();
    if (lrc != PIKV_OK) return lrc;
    AttnPlan plan;
    CombineParams c;
    lrc = launch_attn_partial(desc, q, K_shards, V_shards, U_K, U_V, n_valid, topk_idx, gates, k,
                              combine, scale, y, row_max, row_norm, scores, slot_coef, workspace,
                              workspace_bytes, stream, &plan, &c);
    if (lrc != PIKV_OK) return lrc;
    if ((int64_t)desc->Hq * k > kPostMaxShards || desc->Hq >= kPostSplitRows) {
        // too many partials to restage per utility block: separate merge and utility launches
        lrc = pikv_sharded_attn_merge(desc, &c, stream);
        if (lrc != PIKV_OK) return lrc;
        if (track)
            lrc = pikv_update_utility_tracked(desc, scores, slot_coef, n_valid, topk_idx, k, decay,
                                              utility, pol.threshold, pol.now, pol.last_access,
                                              pol.freq, stream);
        else
            lrc = pikv_update_utility(desc, scores, slot_coef, n_valid, topk_idx, k, decay, utility,
                                      stream);
        if (lrc != PIKV_OK || fb == nullptr) return lrc;
        return pikv_router_penalty(fb->mode, topk_idx, desc->B, k, desc->E, fb->load, fb->miss, fb->coef,
                                   fb->bias, stream);
    }
    PostParams pp;
    pp.c = c;
    pp.scores = scores;
    pp.n_valid = n_valid;
    pp.topk = topk_idx;
    pp.utility = utility;
    pp.track = track;
    pp.pol = pol;
    pp.small_scores = (int64_t)desc->Hq * k * desc->S < ((int64_t)1 << 31);
    pp.B = desc->B;
    pp.E = desc->E;
    pp.S = desc->S;
    const int np = k * plan.nsplit;
    const int threads = combine_threads(np);
    // Utility blocks: enough of them to fill the GPU once (256 CUs x the blocks a CU holds),
    // each walking through several slot tiles rather than a new block per tile - the
    // statistics of the sequence's (head, shard) pairs are then computed once per block.
    const int64_t slot_tiles = (desc->S + threads / 4 - 1) / (threads / 4);
    const int64_t want_blocks = threads == 256 ? 1024 : 256;
    int64_t tpb = ((int64_t)desc->B * k * slot_tiles + want_blocks - 1) / want_blocks;
    if (tpb < 1) tpb = 1;
    if (tpb > kPostMaxTiles) tpb = kPostMaxTiles;
    pp.tiles_per_block = (int)tpb;
    pp.tiles = (int)((slot_tiles + tpb - 1) / tpb);
    // many (head, shard) pairs per utility block, or many heads per thread: the kernel shape
    // that keeps several passes of statistics in flight and starts the utility blocks first
    const bool many = desc->Hq * k > 2 * (threads / 8) || (desc->Hq + 3) / 4 > 2 * kPostPrefetchHeads;
    pp.util_first = many ? 1 : 0;
    pp.decay = decay;
    pp.feedback = fb != nullptr;
    pp.fb = pen;
    const int64_t blocks = (int64_t)desc->B * desc->Hq + (int64_t)desc->B * k * pp.tiles + (fb ? 1 : 0);
    if (blocks > 0x7fffffff) return PIKV_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)blocks);
    const bool f32 = desc->dtype == PIKV_F32;
    const size_t lds = post_smem_bytes(threads, np, desc->Hq * k);
    const bool multi = tpb > 1;
#define PIKV_LAUNCH_POST(T, TH)                                                                          \
    do {                                                                                                 \
        if (many) hipLaunchKernelGGL((step_post<T, TH, kPostMany>), grid, dim3(TH), lds, st, pp);        \
        else if (multi) hipLaunchKernelGGL((step_post<T, TH, kPostMulti>), grid, dim3(TH), lds, st, pp); \
        else hipLaunchKernelGGL((step_post<T, TH, kPostSingle>), grid, dim3(TH), lds, st, pp);           \
    } while (0)
    if (threads == 256) {
        if (f32) PIKV_LAUNCH_POST(float, 256);
        else PIKV_LAUNCH_POST(bf16, 256);
    } else {
        if (f32) PIKV_LAUNCH_POST(float, 1024);
        else PIKV_LAUNCH_POST(bf16, 1024);
    }
#undef PIKV_LAUNCH_POST
    return launch_status();
}

extern "C" int pikv_decode_step(const pikv_desc *desc, const void *q, const void *W_r,
                                const float *bias, const void *K_new, const void *V_new,
                                void *const *K_shards, void *const *V_shards, const void *U_K,
                                const void *U_V, int32_t *n_valid, float *utility, int32_t k,
                                int32_t combine, float scale, float decay, int32_t *topk_idx,
                                float *gates, int32_t *evicted_idx, int32_t *evicted_cnt, float *y,
                                float *row_max, float *row_norm, float *scores, float *slot_coef,
                                void *workspace, size_t workspace_bytes, void *stream) {
    return decode_step(desc, q, W_r, bias, K_new, V_new, K_shards, V_shards, U_K, U_V, n_valid, utility,
                       k, combine, scale, decay, topk_idx, gates, evicted_idx, evicted_cnt, y, row_max,
                       row_norm, scores, slot_coef, workspace, workspace_bytes, stream, nullptr, nullptr);
}

extern "C" int pikv_decode_step_policy(const pikv_desc *desc, const void *q, const void *W_r,
                                       const float *bias, const void *K_new, const void *V_new,
                                       void *const *K_shards, void *const *V_shards, const void *U_K,
                                       const void *U_V, int32_t *n_valid, float *utility, int32_t k,
                                       int32_t combine, float scale, float decay, int32_t *topk_idx,
                                       float *gates, int32_t *evicted_idx, int32_t *evicted_cnt,
                                       float *y, float *row_max, float *row_norm, float *scores,
                                       float *slot_coef, void *workspace, size_t workspace_bytes,
                                       void *stream, const pikv_policy_args *policy,
                                       const pikv_router_feedback *feedback) {
    return decode_step(desc, q, W_r, bias, K_new, V_new, K_shards, V_shards, U_K, U_V, n_valid, utility,
                       k, combine, scale, decay, topk_idx, gates, evicted_idx, evicted_cnt, y, row_max,
                       row_norm, scores, slot_coef, workspace, workspace_bytes, stream, policy, feedback);
}

