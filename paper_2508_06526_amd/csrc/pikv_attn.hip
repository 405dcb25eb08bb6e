// Routed attention over the selected expert shards (PiKV Algorithm 1, the f_attn step over
// C[g_t]; Section 3.2: only the k selected shards are fetched; Section 3.3: rank-r codes are
// decoded inside the kernel) as a split flash-decode for gfx950:
//
//   attn_partial : grid over (sequence, head group, selected shard, split).  Each wave64
//                  streams whole K rows and V rows with 16-byte lane loads (a wave load is
//                  1 KiB of consecutive bytes), keeps a running max / sum / output in fp32
//                  registers and never revisits a byte.  A block of 4 waves merges its
//                  waves through LDS and writes one (max, sum, acc[width]) partial.
//   attn_combine : one block per (sequence, query head) merges the k * nsplit partials with
//                  the router gates, applies the value decoder for rank-r codes, and emits
//                  y, the row statistics and the (shift, coef) pairs the utility pass needs.
//
// Low-rank entries are never materialised: s_i = scale * <U_K q, code_i> and
// y = (sum_i p_i code_i) U_V, so the streamed bytes are the codes and the decode costs
// O(rank) per entry (the paper's T_decode is linear in the compressed width, eq. 2).
#include "pikv_common.h"
#include "pikv_combine_dev.h"

#include <math.h>

namespace pikv {

namespace {

constexpr int kWavesPerBlock = 4;

// Shape of the plain-ALU kernel by row size and heads per block.  16-byte loads each lane keeps
// in flight per K (or V) tile: 8, or kShortRowLoads for one head over rows of at most 128 bytes (rank-r codes):
// that kernel then fits 128 registers, a CU holds four of its 4-wave blocks instead of three, and
// 1024 (sequence, head, shard) units run in one round of resident blocks instead of one and a third.
constexpr int kShortRowLoads = 4;
constexpr bool plain_short_rows(int row_bytes, int gb) { return gb == 1 && row_bytes <= 128; }
constexpr int plain_loads_per_tile(int row_bytes, int gb) { return plain_short_rows(row_bytes, gb) ? kShortRowLoads : 8; }

struct AttnParams {
    const void *q;
    const void *const *K;
    const void *const *V;
    const void *U_K;
    const int32_t *n_valid;
    const int32_t *topk;
    float *part_acc;
    float *part_ml;
    float *scores;
    int B, Hq, G, D, E, S, k, rr, rank;
    int64_t stride_h, stride_s;
    int nsplit, chunk;
    int tq;             // draft queries per sequence: q is [B, tq, Hq / tq, D] (1: plain [B, Hq, D])
    int stage_scores;   // keep the block's scores in LDS, write them in one burst at the end
    int stream_scores;  // ... with non-temporal stores
    float scale;
};

// Raw scores of at most this many bytes per block are staged in LDS (plain-ALU kernel).
constexpr int kScoreStageBytes = 16384;
// LDS the matrix-core kernel's blocks hold for their tile staging (K tile, two P tiles, rescale
// factors and wave statistics of 4 waves); their score stage comes on top
constexpr size_t kGqaStaticLds = 4 * (32 * 272 + 2 * 16 * 80 + 16 * 4 + 2 * 16 * 4);

// Resolve the j-th selected shard of a routing row with ONE round trip to memory: the
// expert id is fetched while lanes 0..E-1 fetch the entry count and the K/V base address of
// every expert of the sequence; the selected lane's values are then broadcast.
struct ShardRef {
    int e, n;
    const char *K, *V;
};
__device__ __forceinline__ ShardRef resolve_shard(const AttnParams &p, int b, int route_row, int j,
                                                  int lane) {
    const int l = min(lane, p.E - 1);
    const int64_t s = (int64_t)b * p.E + l;
    const int nv = p.n_valid[s];
    const uint64_t kp = reinterpret_cast<uint64_t>(p.K[s]);
    const uint64_t vp = reinterpret_cast<uint64_t>(p.V[s]);
    const int e = __builtin_amdgcn_readfirstlane(p.topk[(int64_t)route_row * p.k + j]);
    ShardRef out;
    out.e = e;
    out.n = __builtin_amdgcn_readlane(nv, e);
    const uint32_t klo = __builtin_amdgcn_readlane((int)(uint32_t)kp, e);
    const uint32_t khi = __builtin_amdgcn_readlane((int)(uint32_t)(kp >> 32), e);
    const uint32_t vlo = __builtin_amdgcn_readlane((int)(uint32_t)vp, e);
    const uint32_t vhi = __builtin_amdgcn_readlane((int)(uint32_t)(vp >> 32), e);
    out.K = reinterpret_cast<const char *>(((uint64_t)khi << 32) | klo);
    out.V = reinterpret_cast<const char *>(((uint64_t)vhi << 32) | vlo);
    return out;
}

// Where the caller keeps the query of internal row h of sequence b, in rows of D values.
// Internally the rows of a sequence are ordered (kv head, draft query, head of the group), so
// that all rows reading one kv head are adjacent; the caller's q is [B, tq, heads, D].
__device__ __forceinline__ int64_t query_row(const AttnParams &p, int b, int h) {
    if (p.tq <= 1) return (int64_t)b * p.Hq + h;
    const int heads = p.Hq / p.tq;             // query heads of one draft query
    const int g = p.G / p.tq;                  // of them, per kv head
    const int hk = h / p.G, rem = h - hk * p.G;
    const int t = rem / g, gg = rem - t * g;
    return ((int64_t)b * p.tq + t) * heads + hk * g + gg;
}

// 4-wave blocks of the plain-ALU kernel that one CU holds: its register footprint grows with the
// heads per block (about 150 VGPRs at one head, 180-240 at two and four, all 256 at eight).
// The launch bounds hold the compiler to it and the split plan counts resident blocks with it.
constexpr int plain_blocks_per_cu(int row_bytes, int gb) {
    return plain_short_rows(row_bytes, gb) ? 4 : gb == 1 ? 3 : (gb <= 4 ? 2 : 1);
}

template <typename T, int W, int GB>
__global__ __launch_bounds__(kWavesPerBlock *kWave, plain_blocks_per_cu(W * (int)sizeof(T), GB)) void attn_partial(
    AttnParams p) {
    constexpr int EPL = Pack16<T>::N;        // elements per lane per load
    constexpr int LPR = W / EPL;             // lanes covering one row
    constexpr int RPL = kWave / LPR;         // rows covered by one wave load
    constexpr int NL = plain_loads_per_tile(W * (int)sizeof(T), GB);
    constexpr int TILE = RPL * NL;           // rows per wave iteration
    constexpr int CB = ilog2(LPR);           // lane bits that index the column chunk
    static_assert(LPR >= 1 && LPR <= 32 && (LPR & (LPR - 1)) == 0, "row must be 16..512 bytes");

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int c = lane & (LPR - 1);
    const int r = lane >> CB;

    int bid = blockIdx.x;
    const int split = bid % p.nsplit;
    bid /= p.nsplit;
    const int j = bid % p.k;
    bid /= p.k;
    const int hgroups = p.Hq / GB;
    const int hg = bid % hgroups;
    const int b = bid / hgroups;
    const int h0 = hg * GB;
    const int hk = h0 / p.G;
    const int route_row = b * p.rr + (p.rr == 1 ? 0 : h0);
    const ShardRef sh = resolve_shard(p, b, route_row, j, lane);
    const int n = sh.n;
    const int r0 = split * p.chunk;
    const int r1 = min(n, r0 + p.chunk);

    __shared__ float q_s[GB][W];
    __shared__ float sm_acc[kWavesPerBlock][GB][W];
    __shared__ float sm_m[kWavesPerBlock][GB];
    __shared__ float sm_l[kWavesPerBlock][GB];
    // Raw scores of the block's rows, [GB][chunk], when p.stage_scores: scattered 128-byte
    // score writes in the middle of the K/V stream cost far more HBM time than their bytes
    // (each one turns a channel around); one contiguous burst per block at the end does not.
    extern __shared__ __attribute__((aligned(16))) float score_stage[];

    const int64_t part_base = (((int64_t)b * p.Hq + h0) * p.k + j) * p.nsplit + split;
    const int64_t part_head_stride = (int64_t)p.k * p.nsplit;

    if (r0 >= r1) {  // nothing valid in this split (short or empty shard)
        for (int idx = tid; idx < GB * W; idx += blockDim.x) {
            const int g = idx / W, d = idx - g * W;
            p.part_acc[(part_base + g * part_head_stride) * W + d] = 0.0f;
            if (d == 0) {
                p.part_ml[(part_base + g * part_head_stride) * 2 + 0] = -INFINITY;
                p.part_ml[(part_base + g * part_head_stride) * 2 + 1] = 0.0f;
            }
        }
        return;
    }

    const T *Kb = reinterpret_cast<const T *>(sh.K) + (int64_t)hk * p.stride_h + c * EPL;
    const T *Vb = reinterpret_cast<const T *>(sh.V) + (int64_t)hk * p.stride_h + c * EPL;

    // A wave owns tiles t0, t0 + 4*TILE, ... of the block's row range.  The loads of a tile
    // are issued one phase ahead of their use (K of the next tile while the softmax of this
    // one runs, V of the next tile after this tile's PV), so every wave always has 8 KiB in
    // flight; the first tile's loads go out before the query is staged.
    uint4 kr[NL], vr[NL];
    auto load_tile = [&](uint4(&dst)[NL], const T *base, int t0) {
#pragma unroll
        for (int t = 0; t < NL; ++t) {
            // rows past the end are clamped onto the last valid row (always in bounds) and
            // masked out of the softmax below, so the loads need no branches
            const int row = min(t0 + t * RPL + r, r1 - 1);
            dst[t] = load16_stream(base + (int64_t)row * p.stride_s);
        }
    };
    int t0 = r0 + wave * TILE;
    if (t0 < r1) {
        load_tile(kr, Kb, t0);
        load_tile(vr, Vb, t0);
    }

    // Stage the (scaled) query in LDS; for rank-r codes it is the projected query U_K q.
    const T *qp = static_cast<const T *>(p.q) + ((int64_t)b * p.Hq + h0) * p.D;
    if (p.rank == 0) {
        for (int idx = tid; idx < GB * W; idx += blockDim.x)
            q_s[idx / W][idx % W] = p.scale * load_scalar<T>(qp, idx);   // W == D here
    } else {
        // 8 lanes per (head, code column): 16-byte loads of the decoder row and of q, all
        // independent, joined by an xor butterfly (fixed order)
        const T *U = static_cast<const T *>(p.U_K) + (int64_t)hk * p.rank * p.D;
        const int chunks = p.D / EPL;
        const int sub = tid & 7;
        for (int idx0 = 0; idx0 < GB * W; idx0 += (kWavesPerBlock * kWave) / 8) {
            const int idx = idx0 + (tid >> 3);
            const bool real = idx < GB * W;
            const int g = real ? idx / W : 0, col = real ? idx - g * W : 0;
            float a = 0.0f;
            for (int ch = sub; ch < chunks; ch += 8) {
                float uf[EPL], qv[EPL];
                Pack16<T>::widen(load16(U + (int64_t)col * p.D + ch * EPL), uf);
                Pack16<T>::widen(load16(qp + (int64_t)g * p.D + ch * EPL), qv);
#pragma unroll
                for (int i = 0; i < EPL; ++i) a = fmaf(uf[i], qv[i], a);
            }
            a += __shfl_xor(a, 1, kWave);
            a += __shfl_xor(a, 2, kWave);
            a += __shfl_xor(a, 4, kWave);
            if (real && sub == 0) q_s[g][col] = p.scale * a;
        }
    }
    __syncthreads();

    float qf[GB][EPL];
#pragma unroll
    for (int g = 0; g < GB; ++g)
#pragma unroll
        for (int i = 0; i < EPL; ++i) qf[g][i] = q_s[g][c * EPL + i];

    float m[GB], l[GB], acc[GB][EPL];
#pragma unroll
    for (int g = 0; g < GB; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.0f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[g][i] = 0.0f;
    }

    for (; t0 < r1; t0 += kWavesPerBlock * TILE) {
        const int tnext = t0 + kWavesPerBlock * TILE;

        // scores: each lane's partial dot over its EPL columns, summed over the row's lanes
        float s[NL][GB];
#pragma unroll
        for (int t = 0; t < NL; ++t) {
            float kf[EPL];
            Pack16<T>::widen(kr[t], kf);
            const bool valid = (t0 + t * RPL + r) < r1;
#pragma unroll
            for (int g = 0; g < GB; ++g) {
                float d = 0.0f;
#pragma unroll
                for (int i = 0; i < EPL; ++i) d = fmaf(qf[g][i], kf[i], d);
                d = bits_sum<0, CB>(d);
                s[t][g] = valid ? d : -INFINITY;
            }
        }
        if (tnext < r1) load_tile(kr, Kb, tnext);

        if (p.scores != nullptr) {  // raw scores for the utility pass, one row per lane
#pragma unroll
            for (int g = 0; g < GB; ++g) {
                float *dst = p.scores + (((int64_t)b * p.Hq + h0 + g) * p.k + j) * p.S;
#pragma unroll
                for (int u = 0; u < NL; u += LPR) {
                    float v = s[u][g];
#pragma unroll
                    for (int t = 1; t < LPR && u + t < NL; ++t) v = (c == t) ? s[u + t][g] : v;
                    const int row = t0 + (u + c) * RPL + r;
                    if (u + c < NL && row < r1) {
                        if (p.stage_scores) score_stage[g * p.chunk + row - r0] = v;
                        else dst[row] = v;
                    }
                }
            }
        }

        // online softmax update (wave-uniform running max per head)
#pragma unroll
        for (int g = 0; g < GB; ++g) {
            float tm = s[0][g];
#pragma unroll
            for (int t = 1; t < NL; ++t) tm = fmaxf(tm, s[t][g]);
            tm = bits_max<CB, 6>(tm);
            const float mn = fmaxf(m[g], tm);
            const float corr = __expf(m[g] - mn);
            m[g] = mn;
            l[g] *= corr;
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[g][i] *= corr;
#pragma unroll
            for (int t = 0; t < NL; ++t) {
                const float pt = __expf(s[t][g] - mn);
                s[t][g] = pt;
                l[g] += pt;
            }
        }

        // acc += p * V rows
#pragma unroll
        for (int t = 0; t < NL; ++t) {
            float vf[EPL];
            Pack16<T>::widen(vr[t], vf);
#pragma unroll
            for (int g = 0; g < GB; ++g)
#pragma unroll
                for (int i = 0; i < EPL; ++i) acc[g][i] = fmaf(s[t][g], vf[i], acc[g][i]);
        }
        if (tnext < r1) load_tile(vr, Vb, tnext);
    }

    // merge the row groups of the wave (same column chunk c, different r) ...
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
        for (int g = 0; g < GB; ++g) {
            l[g] += __shfl_xor(l[g], off, kWave);
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[g][i] += __shfl_xor(acc[g][i], off, kWave);
        }
    }
    if (r == 0) {
#pragma unroll
        for (int g = 0; g < GB; ++g)
#pragma unroll
            for (int i = 0; i < EPL; ++i) sm_acc[wave][g][c * EPL + i] = acc[g][i];
    }
    if (lane == 0) {
#pragma unroll
        for (int g = 0; g < GB; ++g) {
            sm_m[wave][g] = m[g];
            sm_l[wave][g] = l[g];
        }
    }
    __syncthreads();

    if (p.scores != nullptr && p.stage_scores) {   // the block's scores, one contiguous burst
        const int rows = r1 - r0;
#pragma unroll
        for (int g = 0; g < GB; ++g) {
            float *dst = p.scores + (((int64_t)b * p.Hq + h0 + g) * p.k + j) * p.S + r0;
            const float *src = score_stage + g * p.chunk;
            if ((p.S & 3) == 0 && (reinterpret_cast<uintptr_t>(p.scores) & 15) == 0) {   // r0, chunk: multiples of the tile
                const int rows4 = rows & ~3;
                // Bursts that land while later blocks still stream K/V (more than one round
                // of blocks) go out non-temporally: a dirty line parked in L2 is evicted on
                // its own later and interrupts a read stream each time.  With a single round
                // all bursts come at the very end and ordinary stores are cheaper.
                if (p.stream_scores) {
                    for (int i = tid * 4; i < rows4; i += blockDim.x * 4)
                        store16_stream(dst + i, *reinterpret_cast<const uint4 *>(src + i));
                } else {
                    for (int i = tid * 4; i < rows4; i += blockDim.x * 4)
                        *reinterpret_cast<float4 *>(dst + i) = *reinterpret_cast<const float4 *>(src + i);
                }
                if (tid < rows - rows4) dst[rows4 + tid] = src[rows4 + tid];
            } else {
                for (int i = tid; i < rows; i += blockDim.x) dst[i] = src[i];
            }
        }
    }

    // ... then the waves of the block, and write the block's partial.
    for (int idx = tid; idx < GB * W; idx += blockDim.x) {
        const int g = idx / W, d = idx - g * W;
        float M = sm_m[0][g];
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w) M = fmaxf(M, sm_m[w][g]);
        float a = 0.0f, L = 0.0f;
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) {
            const float f = sm_m[w][g] == -INFINITY ? 0.0f : __expf(sm_m[w][g] - M);
            a = fmaf(sm_acc[w][g][d], f, a);
            L = fmaf(sm_l[w][g], f, L);
        }
        p.part_acc[(part_base + g * part_head_stride) * W + d] = a;
        if (d == 0) {
            p.part_ml[(part_base + g * part_head_stride) * 2 + 0] = M;
            p.part_ml[(part_base + g * part_head_stride) * 2 + 1] = L;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Grouped-query variant on the matrix cores (bf16 rows of 128 values, one routing decision
// per token, 2..64 query rows per kv head: the heads of the group times the draft queries of
// a multi-query step).  With G query rows sharing every K/V byte the plain-ALU kernel above
// spends ~G times more instructions per byte and stops being memory-bound; here the G rows
// (padded to whole tiles of 16) form the second dimension of 16x16x32 bf16 MFMA tiles, so the
// instruction count per byte does not depend on G within a row tile.
//
// Per wave and per tile of 32 entries:
//   * K and V rows arrive with the same coalesced 16-byte lane loads as above; lane
//     (r = lane/16, c = lane%16) takes rows 8r..8r+7 and byte chunk c of each.
//   * scores, transposed: S^T[entry][head] = K . Q^T.  The MFMA wants lane%16 to index the
//     entry, so the K registers make one trip through a padded wave-private LDS tile
//     (write row-major, read one entry per lane); Q sits in registers as the other operand.
//     Result: lane (head c, group r) holds 8 entries of head c - the softmax is lane-local
//     except for two cross-group steps.
//   * probabilities go back through LDS (as a bf16 high part plus a bf16 residual, so the
//     product is exact to ~2^-17) into the row-operand layout: lane (head c, group r) gets
//     P[head c][entries 8r..8r+7].
//   * output: O[head][d] += P . V.  V needs no transpose at all: for output column set i the
//     column operand of lane (c, r) is V[entries 8r..8r+7][d = 8c + i], i.e. the i-th value
//     of each of its own 8 loaded rows, packed by byte-permutes.
constexpr int kGqaTile = 32;
// Bytes per staged K row: 256 + 16 of padding, so that the 16 lanes reading one 16-byte column
// of 16 different rows do not all start in the same bank.  The pass waits on memory, not on LDS:
// a pitch of 288, which halves the bank-conflict cycles the counters report, runs in the same
// time to the nanosecond, so the smaller pitch stays.
constexpr int kGqaKPitch = 272;
constexpr int kGqaPPitch = 80;    // bytes per staged P row (32 bf16 + 16 pad)

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void wave_lds_order() {
    // LDS operations of one wave execute in order; this only stops the compiler from moving
    // them across the point where another lane's data is expected.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// RT = number of 16-row tiles the query group occupies (group rows = query heads per kv head
// times the draft queries of a multi-query step): 1, 2 or 4.  Every row tile reuses the K tile
// staged in LDS and the V rows in registers, so the streamed bytes do not grow with RT; the
// accumulators do (32 registers per row tile), which is why a CU holds 3 blocks at RT = 1 and 2
// above.  For RT = 4 the query operands live in LDS instead of registers.
template <int RT>
struct GqaShape {
    static constexpr int kBlocksPerCU = RT == 1 ? 3 : 2;
    static constexpr bool kQueryInLds = RT > 2;
    // RT = 4: the 128 accumulator registers leave no room to hold the next K tile across the
    // whole tile's arithmetic; K is then loaded where it is used and the CU's other waves hide
    // the latency (at four row tiles the kernel is bound by the matrix cores, not by memory).
    static constexpr bool kPrefetchK = RT < 4;
};

// SC: what happens to the raw scores - kScoresNone (not asked for), kScoresStaged (kept in LDS,
// one burst per row at the block's end) or kScoresDirect (written from the loop).  A template
// parameter and not a run-time branch: each form costs registers, and a value spilled for one
// of them is reloaded inside the loop by a scratch load, which the wait counters cannot tell
// from the tile loads in flight - the wave then waits for all of them.
constexpr int kScoresNone = 0, kScoresStaged = 1, kScoresDirect = 2;
template <int RT, int SC>
__global__ __launch_bounds__(kWavesPerBlock *kWave, GqaShape<RT>::kBlocksPerCU) void attn_partial_gqa128(
    AttnParams p) {
    constexpr int W = 128;
    constexpr bool QLDS = GqaShape<RT>::kQueryInLds;
    constexpr bool KPRE = GqaShape<RT>::kPrefetchK;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int c = lane & 15;
    const int r = lane >> 4;
    const int gb = p.G;                       // rows per block = the whole query group

    // Workgroups go to the 8 XCDs round-robin by id.  Giving each XCD a contiguous range of
    // work items - whole (kv head, shard) units, whose splits share score rows and partial
    // lines - measures 1.3 % faster here than spreading neighbours over all XCDs; the
    // plain-ALU kernel above measures 2.6 % slower with it and keeps the round-robin order.
    int bid = blockIdx.x;
    if (gridDim.x % 8 == 0) bid = (bid % 8) * (gridDim.x / 8) + bid / 8;
    const int split = bid % p.nsplit;
    bid /= p.nsplit;
    const int j = bid % p.k;
    bid /= p.k;
    const int hgroups = p.Hq / gb;
    const int hk = bid % hgroups;
    const int b = bid / hgroups;
    const int h0 = hk * gb;
    const ShardRef sh = resolve_shard(p, b, b, j, lane);
    const int n = sh.n;
    const int r0 = split * p.chunk;
    const int r1 = min(n, r0 + p.chunk);

    __shared__ __attribute__((aligned(16))) unsigned char lds_k[kWavesPerBlock][kGqaTile * kGqaKPitch];
    __shared__ __attribute__((aligned(16))) unsigned char lds_p[kWavesPerBlock][2][16 * kGqaPPitch];
    __shared__ __attribute__((aligned(16))) float lds_corr[kWavesPerBlock][16];
    __shared__ float sm_m[kWavesPerBlock][16];
    __shared__ float sm_l[kWavesPerBlock][16];
    __shared__ __attribute__((aligned(16))) unsigned char lds_q[QLDS ? RT * 16 * kGqaKPitch : 16];
    // Raw scores of the block's rows, [rows of the group][chunk], when p.stage_scores (see
    // attn_partial): written to memory in one contiguous burst per row after the streaming loop.
    extern __shared__ __attribute__((aligned(16))) float gqa_stage[];

    const int64_t part_base = (((int64_t)b * p.Hq + h0) * p.k + j) * p.nsplit + split;
    const int64_t part_head_stride = (int64_t)p.k * p.nsplit;

    if (r0 >= r1) {
        for (int idx = tid; idx < gb * W; idx += blockDim.x) {
            const int g = idx / W, d = idx - g * W;
            p.part_acc[(part_base + g * part_head_stride) * W + d] = 0.0f;
            if (d == 0) {
                p.part_ml[(part_base + g * part_head_stride) * 2 + 0] = -INFINITY;
                p.part_ml[(part_base + g * part_head_stride) * 2 + 1] = 0.0f;
            }
        }
        return;
    }

    const int64_t row_bytes = p.stride_s * 2;
    const char *Kb = sh.K + (int64_t)hk * p.stride_h * 2;
    const char *Vb = sh.V + (int64_t)hk * p.stride_h * 2;
    // lane part of every address: rows 8r.. of the tile, byte chunk c (fits 32 bits)
    const uint32_t lane_off = (uint32_t)(8 * r) * (uint32_t)row_bytes + 16u * c;

    uint4 kr[8], vr[8];
    auto load_tile = [&](uint4(&dst)[8], const char *base, int t0) {
        if (t0 + kGqaTile <= r1) {     // full tile: wave-uniform base + constant lane offset
            const char *bp = base + (int64_t)t0 * row_bytes;
#pragma unroll
            for (int t = 0; t < 8; ++t) dst[t] = load16_stream(bp + t * row_bytes + lane_off);
        } else {                        // ragged tail: clamp onto the last valid row, mask later
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int row = min(t0 + 8 * r + t, r1 - 1);
                dst[t] = load16_stream(base + (int64_t)row * row_bytes + 16 * c);
            }
        }
    };
    int t0 = r0 + __builtin_amdgcn_readfirstlane(wave) * kGqaTile;
    if (t0 < r1) {
        if constexpr (KPRE) load_tile(kr, Kb, t0);
        load_tile(vr, Vb, t0);
    }

    // query operand of row tile rt: lane (row c, group r) holds Q[row rt*16 + c][32 s + 8 r .. +7],
    // s = 0..3 (zero for rows past the group).  The group's rows are the query rows
    // h0 .. h0 + gb - 1 of the sequence; query_row() maps a group row to where the caller keeps it.
    bf16x8_t qop[QLDS ? 1 : RT][4];
    if constexpr (QLDS) {
        for (int idx = tid; idx < RT * 16 * 16; idx += blockDim.x) {     // (row, 16-byte chunk)
            const int row = idx >> 4, ch = idx & 15;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row < gb) v = load16(static_cast<const bf16 *>(p.q) + query_row(p, b, h0 + row) * W + 8 * ch);
            *reinterpret_cast<uint4 *>(lds_q + row * kGqaKPitch + 16 * ch) = v;
        }
        __syncthreads();
    } else {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const int row = rt * 16 + c;
            const bf16 *qrow = static_cast<const bf16 *>(p.q) + query_row(p, b, h0 + min(row, gb - 1)) * W;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                uint4 v = load16(qrow + 32 * s + 8 * r);
                if (row >= gb) v = make_uint4(0, 0, 0, 0);
                qop[rt][s] = __builtin_bit_cast(bf16x8_t, v);
            }
        }
    }

    float m[RT], lsum[RT];                  // running max / partial sum of row rt*16 + c
    f32x4_t oacc[RT][8];                    // oacc[rt][i][x] = O[row rt*16 + 4r + x][d = 8c + i]
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        m[rt] = -INFINITY;
        lsum[rt] = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) oacc[rt][i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    unsigned char *kst = lds_k[wave];
    unsigned char *pst_hi = lds_p[wave][0];
    unsigned char *pst_lo = lds_p[wave][1];

    for (; t0 < r1; t0 += kWavesPerBlock * kGqaTile) {
        const int tnext = t0 + kWavesPerBlock * kGqaTile;

        // K rows -> LDS (row-major, padded), then the next tile's K loads reuse the registers
        if constexpr (!KPRE) {
            // K where it is used: the clamped form for every tile (one code path, no branch
            // between the loads and their use), with 32-bit byte offsets from the kv head's base
            // (the host admits this kernel only for less than 4 GiB per kv head of a shard)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const unsigned row = (unsigned)min(t0 + 8 * r + t, r1 - 1);
                kr[t] = load16_stream(Kb + (size_t)(row * (unsigned)row_bytes + 16u * (unsigned)c));
            }
        }
#pragma unroll
        for (int t = 0; t < 8; ++t)
            *reinterpret_cast<uint4 *>(kst + (8 * r + t) * kGqaKPitch + 16 * c) = kr[t];
        if constexpr (KPRE) {
            if (tnext < r1) load_tile(kr, Kb, tnext);
        }
        wave_lds_order();

#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            if (rt * 16 >= gb) break;        // row tiles past the group (wave-uniform)
            // S^T = K Q^T for the two 16-entry halves of the tile
            f32x4_t sc[2];
#pragma unroll
            for (int hb = 0; hb < 2; ++hb) {
                sc[hb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const uint4 a = *reinterpret_cast<const uint4 *>(kst + (16 * hb + c) * kGqaKPitch + 64 * s + 16 * r);
                    bf16x8_t qv;
                    if constexpr (QLDS)
                        qv = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(
                                                              lds_q + (rt * 16 + c) * kGqaKPitch + 64 * s + 16 * r));
                    else
                        qv = qop[rt][s];
                    sc[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), qv, sc[hb],
                                                                    0, 0, 0);
                }
            }
            // lane (row c, group r): sc[hb][x] is the score of entry t0 + 16 hb + 4 r + x
            const int row_g = rt * 16 + c;   // row of the group this lane's scores belong to
            float sv[8];
#pragma unroll
            for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int row = t0 + 16 * hb + 4 * r + x;
                    sv[hb * 4 + x] = row < r1 ? sc[hb][x] * p.scale : -INFINITY;
                }
            if (SC == kScoresStaged && row_g < gb) {
                // [row of the group][row of the block]: chunk is a multiple of the tile, so the
                // float4 stores stay aligned
                float *dst = gqa_stage + row_g * p.chunk + (t0 - r0) + 4 * r;
#pragma unroll
                for (int hb = 0; hb < 2; ++hb)
                    *reinterpret_cast<float4 *>(dst + 16 * hb) =
                        make_float4(sv[hb * 4], sv[hb * 4 + 1], sv[hb * 4 + 2], sv[hb * 4 + 3]);
            } else if (SC == kScoresDirect && row_g < gb) {
                float *dst = p.scores + (((int64_t)b * p.Hq + h0 + row_g) * p.k + j) * p.S + t0 + 4 * r;
#pragma unroll
                for (int hb = 0; hb < 2; ++hb) {
                    const int row = t0 + 16 * hb + 4 * r;
                    if (row + 4 <= r1 && (p.S & 3) == 0) {
                        *reinterpret_cast<float4 *>(dst + 16 * hb) =
                            make_float4(sv[hb * 4], sv[hb * 4 + 1], sv[hb * 4 + 2], sv[hb * 4 + 3]);
                    } else {
#pragma unroll
                        for (int x = 0; x < 4; ++x)
                            if (row + x < r1) dst[16 * hb + x] = sv[hb * 4 + x];
                    }
                }
            }

            // online softmax for row c of this tile (entries are spread over the 4 lane groups)
            float tm = sv[0];
#pragma unroll
            for (int x = 1; x < 8; ++x) tm = fmaxf(tm, sv[x]);
            tm = fmaxf(tm, __shfl_xor(tm, 16, kWave));
            tm = fmaxf(tm, __shfl_xor(tm, 32, kWave));
            const float mn = fmaxf(m[rt], tm);
            const float corr = __expf(m[rt] - mn);
            m[rt] = mn;
            lsum[rt] *= corr;
            float pv[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                pv[x] = __expf(sv[x] - mn);
                lsum[rt] += pv[x];
            }
            // probabilities as bf16 high part + bf16 residual, 4 consecutive entries per store
#pragma unroll
            for (int hb = 0; hb < 2; ++hb) {
                uint32_t hi2[2], lo2[2];
#pragma unroll
                for (int q2 = 0; q2 < 2; ++q2) {
                    const f32x2_t v = {pv[hb * 4 + 2 * q2], pv[hb * 4 + 2 * q2 + 1]};
                    const bf16x2_t hi = __builtin_convertvector(v, bf16x2_t);
                    const f32x2_t back = {(float)hi[0], (float)hi[1]};
                    const bf16x2_t lo = __builtin_convertvector(v - back, bf16x2_t);
                    hi2[q2] = __builtin_bit_cast(uint32_t, hi);
                    lo2[q2] = __builtin_bit_cast(uint32_t, lo);
                }
                const int off = c * kGqaPPitch + (16 * hb + 4 * r) * 2;
                *reinterpret_cast<uint2 *>(pst_hi + off) = make_uint2(hi2[0], hi2[1]);
                *reinterpret_cast<uint2 *>(pst_lo + off) = make_uint2(lo2[0], lo2[1]);
            }
            if (r == 0) lds_corr[wave][c] = corr;
            wave_lds_order();

            // row operands P[row c][entries 8r..8r+7] and the rescale factors of rows 4r..4r+3
            const bf16x8_t p_hi = __builtin_bit_cast(
                bf16x8_t, *reinterpret_cast<const uint4 *>(pst_hi + c * kGqaPPitch + 16 * r));
            const bf16x8_t p_lo = __builtin_bit_cast(
                bf16x8_t, *reinterpret_cast<const uint4 *>(pst_lo + c * kGqaPPitch + 16 * r));
            const float4 cr = *reinterpret_cast<const float4 *>(&lds_corr[wave][4 * r]);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                oacc[rt][i][0] *= cr.x;
                oacc[rt][i][1] *= cr.y;
                oacc[rt][i][2] *= cr.z;
                oacc[rt][i][3] *= cr.w;
            }
            // O += P V, output column set i takes the i-th value of each of the lane's 8 V rows
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
                uint32_t w[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const uint4 &v = vr[t];
                    w[t] = (i >> 1) == 0 ? v.x : (i >> 1) == 1 ? v.y : (i >> 1) == 2 ? v.z : v.w;
                }
                const uint4 packed = make_uint4(__builtin_amdgcn_perm(w[1], w[0], sel),
                                                __builtin_amdgcn_perm(w[3], w[2], sel),
                                                __builtin_amdgcn_perm(w[5], w[4], sel),
                                                __builtin_amdgcn_perm(w[7], w[6], sel));
                const bf16x8_t vop = __builtin_bit_cast(bf16x8_t, packed);
                oacc[rt][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(p_hi, vop, oacc[rt][i], 0, 0, 0);
                oacc[rt][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(p_lo, vop, oacc[rt][i], 0, 0, 0);
            }
            wave_lds_order();                // the P tiles are rewritten by the next row tile
        }
        if constexpr (KPRE) {
            if (tnext < r1) load_tile(vr, Vb, tnext);
        } else {
            // the next tile's V rows, requested on the loop's own path (its exit test comes first)
            // rather than under a condition inside it
            if (tnext >= r1) break;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const unsigned row = (unsigned)min(tnext + 8 * r + t, r1 - 1);
                vr[t] = load16_stream(Vb + (size_t)(row * (unsigned)row_bytes + 16u * (unsigned)c));
            }
        }
    }

    __syncthreads();
    if (SC == kScoresStaged) {   // the block's scores: one burst per row of the group
        const int rows = r1 - r0, rows4 = rows & ~3;
        for (int g = 0; g < gb; ++g) {
            float *dst = p.scores + (((int64_t)b * p.Hq + h0 + g) * p.k + j) * p.S + r0;
            const float *src = gqa_stage + g * p.chunk;
            if ((p.S & 3) == 0 && (reinterpret_cast<uintptr_t>(p.scores) & 15) == 0) {
                for (int i = tid * 4; i < rows4; i += blockDim.x * 4)
                    *reinterpret_cast<float4 *>(dst + i) = *reinterpret_cast<const float4 *>(src + i);
                if (tid < rows - rows4) dst[rows4 + tid] = src[rows4 + tid];
            } else {
                for (int i = tid; i < rows; i += blockDim.x) dst[i] = src[i];
            }
        }
    }

    // per row tile: wave results -> LDS (the wave's own K staging area is free now), then merge
    // the waves and write the block's partial
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        if (rt * 16 >= gb) break;
        const int rows_here = min(16, gb - rt * 16);
        float ls = lsum[rt];
        ls += __shfl_xor(ls, 16, kWave);
        ls += __shfl_xor(ls, 32, kWave);
        float *wacc = reinterpret_cast<float *>(kst);          // [16][128] floats = 8 KiB
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int head = 4 * r + x;
            if (head < rows_here) {
                *reinterpret_cast<float4 *>(wacc + head * W + 8 * c) =
                    make_float4(oacc[rt][0][x], oacc[rt][1][x], oacc[rt][2][x], oacc[rt][3][x]);
                *reinterpret_cast<float4 *>(wacc + head * W + 8 * c + 4) =
                    make_float4(oacc[rt][4][x], oacc[rt][5][x], oacc[rt][6][x], oacc[rt][7][x]);
            }
        }
        if (r == 0) {
            sm_m[wave][c] = m[rt];
            sm_l[wave][c] = ls;
        }
        __syncthreads();
        for (int idx = tid; idx < rows_here * W; idx += blockDim.x) {
            const int g = idx / W, d = idx - g * W;
            float M = sm_m[0][g];
#pragma unroll
            for (int w2 = 1; w2 < kWavesPerBlock; ++w2) M = fmaxf(M, sm_m[w2][g]);
            float a = 0.0f, L = 0.0f;
#pragma unroll
            for (int w2 = 0; w2 < kWavesPerBlock; ++w2) {
                const float f = sm_m[w2][g] == -INFINITY ? 0.0f : __expf(sm_m[w2][g] - M);
                a = fmaf(reinterpret_cast<const float *>(lds_k[w2])[g * W + d], f, a);
                L = fmaf(sm_l[w2][g], f, L);
            }
            const int64_t at = part_base + (rt * 16 + g) * part_head_stride;
            p.part_acc[at * W + d] = a;
            if (d == 0) {
                p.part_ml[at * 2 + 0] = M;
                p.part_ml[at * 2 + 1] = L;
            }
        }
        if (rt + 1 < RT) __syncthreads();    // the staging areas are rewritten by the next row tile
    }
}

template <typename T, int THREADS>
__global__ __launch_bounds__(THREADS) void attn_combine(CombineParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // combine_smem_bytes()
    combine_head<T, THREADS>(p, blockIdx.x, smem);
}

template <typename T, int W>
int launch_partial_w(int gb, const AttnParams &p, int blocks, hipStream_t st) {
    const dim3 grid(blocks), block(kWavesPerBlock * kWave);
    const size_t lds = p.stage_scores ? (size_t)gb * p.chunk * sizeof(float) : 0;
    switch (gb) {
        case 1: hipLaunchKernelGGL((attn_partial<T, W, 1>), grid, block, lds, st, p); break;
        case 2: hipLaunchKernelGGL((attn_partial<T, W, 2>), grid, block, lds, st, p); break;
        case 4: hipLaunchKernelGGL((attn_partial<T, W, 4>), grid, block, lds, st, p); break;
        case 8: hipLaunchKernelGGL((attn_partial<T, W, 8>), grid, block, lds, st, p); break;
        default: return PIKV_ERR_UNSUPPORTED;
    }
    return launch_status();
}

template <typename T>
int launch_partial(int width, int gb, const AttnParams &p, int blocks, hipStream_t st) {
    switch (width) {
        case 16: return launch_partial_w<T, 16>(gb, p, blocks, st);
        case 32: return launch_partial_w<T, 32>(gb, p, blocks, st);
        case 64: return launch_partial_w<T, 64>(gb, p, blocks, st);
        case 128: return launch_partial_w<T, 128>(gb, p, blocks, st);
        default: return PIKV_ERR_UNSUPPORTED;
    }
}

}  // namespace

static int g_split_override = 0;   // tuning hook, see pikv_set_attn_split
static hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;   // see pikv_set_profile_events
void g_split_override_set(int v) { g_split_override = v > 0 ? v : 0; }

int make_attn_plan(const pikv_desc *d, int k, AttnPlan *plan) {
    const int rc = check_desc(d);
    if (rc != PIKV_OK) return rc;
    if (k < 1 || k > d->E) return PIKV_ERR_INVALID;
    const int W = desc_width(d);
    const int G = d->Hq / d->Hkv;
    int gb = 1;
    if (d->route_rows_per_seq == 1 && (G == 2 || G == 4 || G == 8)) gb = G;
    const bool gqa_mfma = d->route_rows_per_seq == 1 && d->dtype == PIKV_BF16 && d->rank == 0 &&
                          d->D == 128 && G >= 2 && G <= 64 &&
                          (int64_t)d->S * d->stride_s * 2 < ((int64_t)1 << 32);
    if (gqa_mfma) gb = G;
    const int tq = d->tq > 1 ? d->tq : 1;
    // draft queries are folded into the query group of the matrix-core kernel only
    if (tq > 1 && (!gqa_mfma || d->Hq % tq != 0 || G % tq != 0)) return PIKV_ERR_UNSUPPORTED;
    const int row_tiles = !gqa_mfma ? 0 : (G <= 16 ? 1 : (G <= 32 ? 2 : 4));
    const int epl = 16 / elem_bytes(d->dtype);
    const int lpr = W / epl;
    if (lpr < 1 || lpr > 32) return PIKV_ERR_UNSUPPORTED;
    const int row_bytes = W * elem_bytes(d->dtype);
    const int tile = gqa_mfma ? kGqaTile : (kWave / lpr) * plain_loads_per_tile(row_bytes, gb);
    const int64_t units = (int64_t)d->B * (d->Hq / gb) * k;
    // One round of resident blocks: 256 CUs times the 4-wave blocks a CU holds at this
    // kernel's register footprint.  Fewer, longer blocks keep the per-wave prefetch chain
    // busy and shrink the partials that the combine pass has to merge.
    int resident = gqa_mfma ? (row_tiles == 1 ? 3 : 2) : plain_blocks_per_cu(row_bytes, gb);
    int64_t nsplit = 1;
    int chunk = 0;
    auto split_for = [&](int res) {
        nsplit = units > 0 ? (int64_t)256 * res / units : 1;
        // No finer than two tiles per wave: with one, nothing is in flight while a wave computes,
        // and a block of uneven waves (2, 2, 1, 1 tiles) runs as long as one of twice the rows.
        // (Few units, short passes: 64 MiB over 16 units 14.0 -> 12.8 us, 32 MiB over 8 units
        // 8.6 -> 7.9 us, and fewer partials for the merge.)  A forced count is only held to one tile.
        int64_t max_split = d->S / (2 * kWavesPerBlock * tile);
        if (g_split_override > 0) {
            nsplit = g_split_override;
            max_split = (d->S + tile - 1) / tile;
        }
        if (max_split < 1) max_split = 1;
        if (nsplit > max_split) nsplit = max_split;
        if (nsplit > kMaxPartialsPerHead / k) nsplit = kMaxPartialsPerHead / k;
        if (nsplit < 1) nsplit = 1;
        chunk = (int)((d->S + nsplit - 1) / nsplit);
        chunk = (chunk + tile - 1) / tile * tile;
        nsplit = (d->S + chunk - 1) / chunk;
        // Matrix-core kernel: when that leaves the waves of a block uneven tile counts (c3: 11
        // tiles, 3 + 3 + 3 + 2) and blocks of exactly two tiles per wave are at most a third more
        // blocks, in whole multiples of the 256 CUs, take those.  The extra blocks form a short
        // last round, and a wave whose first tile is served late has one tile left instead of two
        // (c3: 24 -> 32 splits, pass 23.4 -> 23.1 us).  Longer even blocks in a partial round
        // measured slower (k = 16: 8 splits of 8 tiles per wave against 6 splits, +3.7 %).
        const int even = 2 * kWavesPerBlock * tile;
        const int64_t fine = d->S / even;
        if (gqa_mfma && g_split_override == 0 && chunk % (kWavesPerBlock * tile) != 0 && d->S % even == 0 &&
            fine > nsplit && fine * 3 <= nsplit * 4 && fine <= kMaxPartialsPerHead / k &&
            (units * fine) % 256 == 0) {
            nsplit = fine;
            chunk = even;
        }
    };
    split_for(resident);
    size_t stage = (size_t)gb * chunk * sizeof(float);      // the block's raw scores, staged in LDS
    if (gqa_mfma && gb < 8) {
        // few rows per kv head: the score writes are ~3 % of the bytes and staging them measures
        // no faster (its LDS stores collide with the tile staging)
        stage = 0;
    } else if (gqa_mfma) {
        // The matrix-core kernel's tile staging takes kGqaStaticLds per block (plus the query
        // tile at four row tiles): the score stage must fit beside it as often as a CU holds
        // blocks - three times with one row tile, or twice with longer blocks - or is left out.
        const size_t lds_cu = 160 * 1024;
        const size_t fixed = kGqaStaticLds + (row_tiles == 4 ? (size_t)64 * kGqaKPitch : 0);
        if ((size_t)resident * (fixed + stage) > lds_cu || stage > 64 * 1024 - 256) {
            bool fits = false;
            if (resident == 3) {
                split_for(2);
                stage = (size_t)gb * chunk * sizeof(float);
                fits = 2 * (fixed + stage) <= lds_cu && stage <= 64 * 1024 - 256;
                if (fits) resident = 2;
            }
            if (!fits) {
                split_for(resident);
                stage = 0;
            }
        }
    } else if (stage > (size_t)kScoreStageBytes) {
        stage = 0;
    }
    const int64_t target_blocks = 256 * resident;
    plan->gqa_mfma = gqa_mfma;
    plan->heads_per_block = gb;
    plan->row_tiles = row_tiles;
    plan->head_blocks = d->Hq / gb;
    plan->tile_rows = tile;
    plan->chunk = chunk;
    plan->nsplit = (int)nsplit;
    plan->resident_blocks = (int)target_blocks;
    plan->score_stage_bytes = stage;
    plan->acc_floats = (size_t)d->B * d->Hq * k * nsplit * W;
    plan->ml_floats = (size_t)d->B * d->Hq * k * nsplit * 2;
    return PIKV_OK;
}

}  // namespace pikv

using namespace pikv;

extern "C" void pikv_set_attn_split(int32_t nsplit) { pikv::g_split_override_set(nsplit); }

namespace pikv {
void g_profile_events_set(void *start, void *stop) {
    g_prof_start = static_cast<hipEvent_t>(start);
    g_prof_stop = static_cast<hipEvent_t>(stop);
}
}  // namespace pikv

extern "C" void pikv_set_profile_events(void *start, void *stop) {
    pikv::g_profile_events_set(start, stop);
}

extern "C" size_t pikv_attn_workspace_bytes(const pikv_desc *desc, int32_t k) {
    AttnPlan plan;
    if (make_attn_plan(desc, k, &plan) != PIKV_OK) return 0;
    const size_t acc = (plan.acc_floats * sizeof(float) + 255) / 256 * 256;
    const size_t ml = (plan.ml_floats * sizeof(float) + 255) / 256 * 256;
    return acc + ml + 256;
}

namespace pikv {

// Every host-side check of the attention call and its split plan; launches nothing.
int check_attn_args(const pikv_desc *desc, const void *q, const void *const *K_shards,
                    const void *const *V_shards, const void *U_K, const void *U_V,
                    const int32_t *n_valid, const int32_t *topk_idx, int32_t k, int32_t combine,
                    float scale, const float *y, const void *workspace, size_t workspace_bytes,
                    AttnPlan *plan_out) {
    AttnPlan plan;
    const int rc = make_attn_plan(desc, k, &plan);
    if (rc != PIKV_OK) return rc;
    if (!q || !K_shards || !V_shards || !n_valid || !topk_idx || !y) return PIKV_ERR_INVALID;
    if (desc->rank > 0 && (!U_K || !U_V)) return PIKV_ERR_INVALID;
    if (combine != PIKV_COMBINE_LSE && combine != PIKV_COMBINE_LOCAL) return PIKV_ERR_INVALID;
    if (!(scale == scale)) return PIKV_ERR_INVALID;
    *plan_out = plan;
    if (desc->B == 0) return PIKV_OK;
    const size_t need = pikv_attn_workspace_bytes(desc, k);
    if (!workspace || workspace_bytes < need) return PIKV_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return PIKV_ERR_INVALID;
    if ((int64_t)desc->B * plan.head_blocks * k * plan.nsplit > 0x7fffffff) return PIKV_ERR_UNSUPPORTED;
    return PIKV_OK;
}

bool profile_events_set() { return g_prof_start != nullptr || g_prof_stop != nullptr; }

// Validate, plan and launch the split pass only; fills the parameters of the merge pass.
int launch_attn_partial(const pikv_desc *desc, const void *q, const void *const *K_shards,
                        const void *const *V_shards, const void *U_K, const void *U_V,
                        const int32_t *n_valid, const int32_t *topk_idx, const float *gates,
                        int32_t k, int32_t combine, float scale, float *y, float *row_max,
                        float *row_norm, float *scores, float *slot_coef, void *workspace,
                        size_t workspace_bytes, void *stream, AttnPlan *plan_out,
                        CombineParams *c_out) {
    AttnPlan plan;
    const int rc = check_attn_args(desc, q, K_shards, V_shards, U_K, U_V, n_valid, topk_idx, k, combine,
                                   scale, y, workspace, workspace_bytes, &plan);
    if (rc != PIKV_OK) return rc;
    *plan_out = plan;
    if (desc->B == 0) return PIKV_OK;

    const int W = desc_width(desc);
    float *part_acc = static_cast<float *>(workspace);
    float *part_ml = part_acc + (plan.acc_floats * sizeof(float) + 255) / 256 * 64;

    AttnParams p;
    p.q = q;
    p.K = K_shards;
    p.V = V_shards;
    p.U_K = U_K;
    p.n_valid = n_valid;
    p.topk = topk_idx;
    p.part_acc = part_acc;
    p.part_ml = part_ml;
    p.scores = scores;
    p.B = desc->B;
    p.Hq = desc->Hq;
    p.G = desc->Hq / desc->Hkv;
    p.D = desc->D;
    p.E = desc->E;
    p.S = desc->S;
    p.k = k;
    p.rr = desc->route_rows_per_seq;
    p.rank = desc->rank;
    p.tq = desc->tq > 1 ? desc->tq : 1;
    p.stride_h = desc->stride_h;
    p.stride_s = desc->stride_s;
    p.nsplit = plan.nsplit;
    p.chunk = plan.chunk;
    p.stage_scores = scores != nullptr && plan.score_stage_bytes > 0;
    p.scale = scale > 0.0f ? scale : 1.0f / sqrtf((float)desc->D);

    const int64_t blocks64 = (int64_t)desc->B * plan.head_blocks * k * plan.nsplit;
    p.stream_scores = blocks64 > plan.resident_blocks;
    hipStream_t st = as_stream(stream);
    int lrc;
    if (g_prof_start) (void)hipEventRecord(g_prof_start, st);
    if (plan.gqa_mfma) {
        const size_t lds = p.stage_scores ? plan.score_stage_bytes : 0;
        const dim3 grid((unsigned)blocks64), block(kWavesPerBlock * kWave);
        switch (plan.row_tiles) {
#define PIKV_LAUNCH_GQA(RT)                                                                                 \
    do {                                                                                                    \
        if (p.scores == nullptr)                                                                            \
            hipLaunchKernelGGL((attn_partial_gqa128<RT, kScoresNone>), grid, block, lds, st, p);            \
        else if (p.stage_scores)                                                                            \
            hipLaunchKernelGGL((attn_partial_gqa128<RT, kScoresStaged>), grid, block, lds, st, p);          \
        else                                                                                                \
            hipLaunchKernelGGL((attn_partial_gqa128<RT, kScoresDirect>), grid, block, lds, st, p);          \
    } while (0)
            case 1: PIKV_LAUNCH_GQA(1); break;
            case 2: PIKV_LAUNCH_GQA(2); break;
            default: PIKV_LAUNCH_GQA(4); break;
#undef PIKV_LAUNCH_GQA
        }
        lrc = launch_status();
    } else {
        lrc = desc->dtype == PIKV_F32
                  ? launch_partial<float>(W, plan.heads_per_block, p, (int)blocks64, st)
                  : launch_partial<bf16>(W, plan.heads_per_block, p, (int)blocks64, st);
    }
    if (g_prof_stop) (void)hipEventRecord(g_prof_stop, st);
    if (lrc != PIKV_OK) return lrc;

    CombineParams c;
    c.part_acc = part_acc;
    c.part_ml = part_ml;
    c.gates = gates;
    c.U_V = U_V;
    c.y = y;
    c.row_max = row_max;
    c.row_norm = row_norm;
    c.slot_coef = slot_coef;
    c.Hq = desc->Hq;
    c.G = p.G;
    c.D = desc->D;
    c.W = W;
    c.k = k;
    c.rr = p.rr;
    c.rank = desc->rank;
    c.value_bias = (desc->flags & PIKV_DESC_VALUE_BIAS) ? 1 : 0;
    c.tq = p.tq;
    c.nsplit = plan.nsplit;
    c.combine = combine;
    *c_out = c;
    return PIKV_OK;
}

}  // namespace pikv

namespace pikv {
int pikv_sharded_attn_merge(const pikv_desc *desc, const CombineParams *c, void *stream) {
    const dim3 cgrid(desc->B * desc->Hq);
    hipStream_t st = as_stream(stream);
    const bool f32 = desc->dtype == PIKV_F32;
    const int np = c->k * c->nsplit;
    if (combine_threads(np) == 256) {
        const size_t lds = combine_smem_bytes(256, np);
        if (f32) hipLaunchKernelGGL((attn_combine<float, 256>), cgrid, dim3(256), lds, st, *c);
        else hipLaunchKernelGGL((attn_combine<bf16, 256>), cgrid, dim3(256), lds, st, *c);
    } else {
        const size_t lds = combine_smem_bytes(1024, np);
        if (f32) hipLaunchKernelGGL((attn_combine<float, 1024>), cgrid, dim3(1024), lds, st, *c);
        else hipLaunchKernelGGL((attn_combine<bf16, 1024>), cgrid, dim3(1024), lds, st, *c);
    }
    return launch_status();
}
}  // namespace pikv

extern "C" int pikv_sharded_attn(const pikv_desc *desc, const void *q, const void *const *K_shards,
                                 const void *const *V_shards, const void *U_K, const void *U_V,
                                 const int32_t *n_valid, const int32_t *topk_idx,
                                 const float *gates, int32_t k, int32_t combine, float scale,
                                 float *y, float *row_max, float *row_norm, float *scores,
                                 float *slot_coef, void *workspace, size_t workspace_bytes,
                                 void *stream) {
    AttnPlan plan;
    CombineParams c;
    const int rc = launch_attn_partial(desc, q, K_shards, V_shards, U_K, U_V, n_valid, topk_idx, gates,
                                       k, combine, scale, y, row_max, row_norm, scores, slot_coef,
                                       workspace, workspace_bytes, stream, &plan, &c);
    if (rc != PIKV_OK || desc->B == 0) return rc;
    return pikv_sharded_attn_merge(desc, &c, stream);
}

// ---------------------------------------------------------------------------------------
// The same call for callers that cannot allocate (code under HIP graph capture, tight serving
// loops): the split partials live in a file-scope device array instead of a caller workspace.
namespace {

constexpr size_t kStaticScratchBytes = PIKV_NOALLOC_SCRATCH_BYTES;   // per GPU, held until the process ends
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Address of this GPU's copy of `scratch` (every device holds its own copy at its own address),
// looked up once per device with that device current.  In host code the array's name is only a
// handle for this lookup, never an address to pass to a kernel.
int static_scratch(void **out) {
    static void *ptr_of_device[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PIKV_ERR_HIP;
    if (ptr_of_device[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return PIKV_ERR_HIP;
        ptr_of_device[dev] = ptr;
    }
    *out = ptr_of_device[dev];
    return PIKV_OK;
}

}  // namespace

extern "C" int pikv_sharded_attn_noalloc(const pikv_desc *desc, const void *q, const void *const *K_shards,
                                         const void *const *V_shards, const void *U_K, const void *U_V,
                                         const int32_t *n_valid, const int32_t *topk_idx,
                                         const float *gates, int32_t k, int32_t combine, float scale,
                                         float *y, float *row_max, float *row_norm, float *scores,
                                         float *slot_coef, void *stream) {
    const size_t need = pikv_attn_workspace_bytes(desc, k);
    if (need > kStaticScratchBytes) return PIKV_ERR_WORKSPACE;   // geometry too large for the fixed array
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != PIKV_OK) return rc;
    // Every partial the merge reads is written by the split pass of the same call (empty splits
    // write an empty partial), so nothing in the array has to start at zero.
    return pikv_sharded_attn(desc, q, K_shards, V_shards, U_K, U_V, n_valid, topk_idx, gates, k, combine,
                             scale, y, row_max, row_norm, scores, slot_coef, ws, kStaticScratchBytes, stream);
}
