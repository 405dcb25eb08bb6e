/*
 * pikv.h - C ABI of the MI355X (gfx950) implementation of PiKV's decode-step hot path
 * (arxiv 2508.06526): route -> attend over the top-k expert KV shards -> combine ->
 * update per-entry utility -> evict / append.
 *
 * General conventions
 *   - Every pointer argument is a DEVICE pointer unless the comment says "host".  The
 *     descriptor (pikv_desc) is a host struct passed by const pointer.
 *   - The caller owns every buffer.  The library allocates nothing, frees nothing and
 *     keeps no state between calls; scratch space is passed in as `workspace`.  The only
 *     exceptions are the two process-wide measurement hooks at the end of this file
 *     (pikv_set_attn_split, pikv_set_profile_events), both off by default.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work and return; they never synchronise.
 *   - Return value: a pikv_status.  Argument errors are detected on the host before
 *     anything is launched and leave all outputs untouched; HIP launch failures map to
 *     PIKV_ERR_HIP.  Nothing is printed, nothing aborts.
 *   - Layout of one expert shard (one (sequence b, expert e) pair): rows
 *         shard[h' * stride_h + slot * stride_s + 0 .. width)
 *     for kv head h' in [0,Hkv), slot in [0,S); width = D (dense) or rank (codes); the
 *     last dimension is contiguous; strides are in elements; every row must start on a
 *     16-byte boundary.  K_shards / V_shards are device arrays of B*E device pointers,
 *     entry b*E+e.  The valid entries of a shard are the prefix 0 .. n_valid[b][e]-1.
 *   - Outputs that are probabilities, gates, utilities or attention results are float32
 *     whatever the storage dtype.
 *   - Routing decisions come in rows: row = b (route_rows_per_seq == 1, one decision per
 *     token) or row = b*Hq + h (route_rows_per_seq == Hq, one decision per token and head).
 */
#ifndef PIKV_H
#define PIKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PIKV_OK = 0,
    PIKV_ERR_INVALID = -1,      /* bad argument (null pointer, size out of range, ...)   */
    PIKV_ERR_UNSUPPORTED = -2,  /* valid in principle, no kernel for this shape          */
    PIKV_ERR_WORKSPACE = -3,    /* workspace_bytes smaller than pikv_attn_workspace_bytes */
    PIKV_ERR_HIP = -4           /* the HIP runtime refused a launch                      */
} pikv_status;

typedef enum { PIKV_F32 = 0, PIKV_BF16 = 1 } pikv_dtype;

/* How the per-shard attention results are merged (Algorithm 1, f_attn over C[g_t], with
 * the router's gate weights supplied by the caller):
 *   LSE   - one softmax over the union of the selected shards, each entry weighted by its
 *           shard's gate: p_i = g_e exp(s_i) / sum.  With gates == NULL this is the paper's
 *           0/1 mask (Section 3.2) and k == E reproduces dense attention.
 *   LOCAL - softmax inside each shard, outputs mixed by the gates renormalised over the
 *           non-empty selected shards: y = sum_e g_e o_e / sum_e g_e.                      */
typedef enum { PIKV_COMBINE_LSE = 0, PIKV_COMBINE_LOCAL = 1 } pikv_combine;

/* Geometry of one layer's expert-sharded cache (Section 3.1: E shards of capacity S per
 * sequence).  Plain data, host memory.                                                    */
typedef struct pikv_desc {
    int32_t B;        /* sequences (decode streams)                                        */
    int32_t Hq;       /* query heads, <= 256                                               */
    int32_t Hkv;      /* kv heads, Hq % Hkv == 0; query head h reads kv head h / (Hq/Hkv)  */
    int32_t D;        /* head dimension: 16, 32, 64 or 128                                 */
    int32_t E;        /* expert shards per sequence, 1..64                                 */
    int32_t S;        /* slot capacity of every shard                                      */
    int32_t rank;     /* 0: rows hold D values; r in {16,32,64}: rows hold rank-r codes    */
    int32_t dtype;    /* pikv_dtype of q, K/V (or codes), U_K/U_V                          */
    int64_t stride_h; /* elements between kv heads inside a shard buffer                   */
    int64_t stride_s; /* elements between slots (>= width, multiple of 16 bytes)           */
    int32_t route_rows_per_seq; /* 1 or Hq                                                 */
    int32_t flags;    /* 0, or PIKV_DESC_VALUE_BIAS (rank > 0 only)                        */
    int32_t tq;       /* draft queries per sequence in a multi-query step; 0 or 1: one query */
    int32_t reserved; /* must be 0                                                         */
} pikv_desc;

/* Multi-query (speculative decoding) steps: tq > 1 draft queries of a sequence attend the same
 * selected shards in one pass, so every K/V byte is streamed once for all of them.  Hq then
 * counts ALL query rows of a sequence, Hq = tq * (query heads of the model), and q, y, row_max
 * and row_norm are laid out [B, tq, Hq / tq, ...] - the natural layout of tq consecutive
 * tokens.  pikv_decode_step makes one routing decision per sequence, from the FIRST query of
 * the tile alone - q[b][0], the token that is certain to be kept, the others being drafts -
 * so W_r keeps the shape it has for single-query steps, [(Hq / tq) * D, E].  (pikv_route is
 * unaware of tq: it routes whatever rows it is given.)
 * Each row attends all valid entries of the selected shards; the causal
 * part among the drafts themselves is the caller's (row_max / row_norm let it merge them).
 * Supported for bfloat16 rows of D = 128 values (rank 0) with per-token routing and at most 64
 * query rows per kv head (Hq / Hkv <= 64); UNSUPPORTED otherwise.
 * scores and slot_coef stay internal scratch in every case.                               */

/* desc->flags.  PIKV_DESC_VALUE_BIAS: the value decoder has the additive term of Table 2's
 * LoRA++ row (reconstruction W_d W_u x + b): U_V then holds rank + 1 rows of D values per kv
 * head, [Hkv, rank + 1, D], the last row being b, and every decoded value - hence every output
 * row with a non-empty selection - gains b[h'].  (The same term on the key side would shift all
 * scores of a head equally and cancel in the softmax, so U_K never carries one.)             */
#define PIKV_DESC_VALUE_BIAS 1

/* Section 3.2, Table 1 "TopK softmax" router (with the table's additive per-expert
 * penalty as `bias`): logits = x W_r + bias, p = softmax over the E experts, the mask has
 * ones at the k largest logits.
 *   x      [rows, d_r]  dtype      query vectors being routed
 *   W_r    [d_r, E]     dtype      router weights, row-major
 *   bias   [E] float32 or NULL
 *   topk_idx [rows, k] int32  out  selected experts, descending logit; equal logits:
 *                                  lower expert index first; NaN logits rank as -inf
 *   gates  [rows, k] float32  out  p restricted to the selection, renormalised to sum 1
 *   probs  [rows, E] float32  out  full softmax, or NULL
 * Errors: INVALID for null x/W_r/topk_idx/gates, rows < 0, d_r < 1, E not in 1..64,
 * k not in 1..E, unknown dtype.  rows == 0 is a no-op.                                     */
int pikv_route(const void *x, const void *W_r, const float *bias, int32_t rows, int32_t d_r,
               int32_t E, int32_t k, int32_t dtype, int32_t *topk_idx, float *gates,
               float *probs, void *stream);

/* Bytes of scratch pikv_sharded_attn needs for this geometry and k (host computation;
 * 0 if the descriptor is invalid).  The workspace must be 256-byte aligned.              */
size_t pikv_attn_workspace_bytes(const pikv_desc *desc, int32_t k);

/* Algorithm 1, y_t = f_attn(q_t, C[g_t]): attention of each query head over the valid
 * entries of its selected shards only (Section 3.2: the fetch is 2*B*L*h*k, not ...*E).
 * Scores s_i = scale * <q_h, K_i>.  With rank > 0 the stored rows are codes and the
 * entries are K_i = code_i U_K[h'], V_i = code_i U_V[h'] (Section 3.3, decoder of the
 * rank-r compressor, fused into the kernel: the codes are what is streamed from HBM).
 *   q        [B,Hq,D] dtype
 *   U_K,U_V  [Hkv,rank,D] dtype   (rank > 0 only, else ignored; U_V is [Hkv,rank+1,D] with
 *                                  PIKV_DESC_VALUE_BIAS)
 *   n_valid  [B,E] int32
 *   topk_idx [rows,k] int32       selected experts per routing row (distinct within a row)
 *   gates    [rows,k] float32 or NULL (NULL: every gate is 1)
 *   combine  pikv_combine
 *   scale    <= 0 selects 1/sqrt(D)
 *   y        [B,Hq,D] float32 out  (0 where every selected shard is empty)
 *   row_max  [B,Hq] float32 out or NULL: max score over the non-empty selected shards
 *   row_norm [B,Hq] float32 out or NULL: the normaliser y was divided by
 *                (LSE: sum_e g_e sum_i exp(s_i - row_max); LOCAL: sum_e g_e)
 *   scores   [B,Hq,k,S] float32 out or NULL: raw s_i of entry i of the j-th selected shard
 *   slot_coef [B,Hq,k,2] float32 out or NULL: (shift, coef) such that the attention
 *                probability of entry i is coef * exp(s_i - shift); coef = 0 for an empty
 *                shard.  scores + slot_coef are what pikv_update_utility consumes.
 * Errors: INVALID / UNSUPPORTED per the descriptor limits above, k not in 1..E, null
 * required pointer; WORKSPACE if workspace_bytes is too small.  B == 0 is a no-op.         */
int pikv_sharded_attn(const pikv_desc *desc, const void *q, const void *const *K_shards,
                      const void *const *V_shards, const void *U_K, const void *U_V,
                      const int32_t *n_valid, const int32_t *topk_idx, const float *gates,
                      int32_t k, int32_t combine, float scale, float *y, float *row_max,
                      float *row_norm, float *scores, float *slot_coef, void *workspace,
                      size_t workspace_bytes, void *stream);

/* pikv_sharded_attn for callers that cannot allocate device memory or cannot carry a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments and results, but the split partials go to a fixed array of
 * PIKV_NOALLOC_SCRATCH_BYTES inside the library's device image (one copy per GPU, held until
 * the process ends) instead of a caller workspace.  The call allocates and frees nothing.
 * All calls on one GPU share that array: calls that overlap on one GPU (different streams,
 * different threads) race; serialise them.  The first call on each GPU looks the array's
 * address up (no stream work); make that call outside graph capture.
 * Errors: as pikv_sharded_attn; WORKSPACE when pikv_attn_workspace_bytes(desc, k) exceeds
 * PIKV_NOALLOC_SCRATCH_BYTES (use pikv_sharded_attn with a workspace then); HIP if the array's
 * address cannot be resolved.                                                              */
#define PIKV_NOALLOC_SCRATCH_BYTES (4u << 20)
int pikv_sharded_attn_noalloc(const pikv_desc *desc, const void *q, const void *const *K_shards,
                              const void *const *V_shards, const void *U_K, const void *U_V,
                              const int32_t *n_valid, const int32_t *topk_idx, const float *gates,
                              int32_t k, int32_t combine, float scale, float *y, float *row_max,
                              float *row_norm, float *scores, float *slot_coef, void *stream);

/* Section 3.4, Table 3 row H2O (u_i = a_i, the attention an entry received), kept as a
 * running score: for every shard that at least one query head selected this step and
 * every valid slot i:  u_i <- decay * u_i + sum over those heads of p_{h,i}.
 * decay == 1 accumulates; decay < 1 gives the exponentially decayed score.  Shards nobody
 * selected are not touched.  `scores`, `slot_coef`, `topk_idx`, `k` are those of the
 * pikv_sharded_attn call of the same step.
 *   utility [B,E,S] float32, in place.
 * Errors: INVALID for null pointers, k out of range, decay < 0 or not finite.              */
int pikv_update_utility(const pikv_desc *desc, const float *scores, const float *slot_coef,
                        const int32_t *n_valid, const int32_t *topk_idx, int32_t k,
                        float decay, float *utility, void *stream);

/* Algorithm 1, C <- S(C, q_t) under bounded memory (Section 3.4): every processed shard
 * holding n > capacity entries keeps the `capacity` entries that come first in the order
 * (utility descending, slot ascending) and evicts the other n - capacity.
 *   sel_idx  [B,sel_k] int32 or NULL: process only the shards listed for each sequence
 *            (e.g. this step's topk_idx under per-token routing); NULL: all B*E shards
 *   evicted_idx [B,E,max_evict] int32 out: evicted slots, ascending
 *   evicted_cnt [B,E] int32 out: number evicted (0 for shards skipped or within capacity;
 *            -1, and the shard is left untouched, if n - capacity > max_evict)
 *   compact  != 0: move the kept rows of K, V (all kv heads) and utility down to slots
 *            0..capacity-1 in ascending original order (K_shards/V_shards required).
 *            A moved utility keeps its value; a negative zero may come back as +0.
 *            == 0: rows stay where they are; the evicted slots are holes the caller must
 *            refill with pikv_append (reuse_idx) before the next attention call.
 *   n_valid  [B,E] int32, in place: becomes capacity for shards that evicted.
 * Errors: INVALID for null utility/n_valid/evicted_*, capacity < 0, max_evict < 1,
 * sel_k not in 1..E when sel_idx is given, compact without shard tables; UNSUPPORTED for
 * compact with rows wider than 4096 bytes.                                                  */
int pikv_evict(const pikv_desc *desc, float *utility, int32_t *n_valid, int32_t capacity,
               const int32_t *sel_idx, int32_t sel_k, int32_t *evicted_idx,
               int32_t *evicted_cnt, int32_t max_evict, int32_t compact,
               void *const *K_shards, void *const *V_shards, void *stream);

/* Algorithm 1, Insert into C[e][s]; Section 3.1 storage invariants (fixed-capacity buffer,
 * O(1) insertion, no reallocation): for each sequence b and each expert e = topk_idx[b][j]
 * the new entry's rows (one per kv head) are written to slot
 *     reuse_idx[b][e][0]  if reuse_cnt != NULL and reuse_cnt[b][e] > 0 (a slot pikv_evict
 *                         just freed), else n_valid[b][e];
 * its utility is set to 0 and n_valid[b][e] grows by one.  A shard that is already full
 * (n_valid == S) is skipped: the entry is dropped for that shard.
 *   K_new,V_new [B,Hkv,width] dtype;  topk_idx [B,k] int32 (distinct within a row)
 *   reuse_idx [B,E,max_evict] int32, reuse_cnt [B,E] int32, or both NULL
 * Errors: INVALID for null required pointers, k not in 1..E.                               */
int pikv_append(const pikv_desc *desc, const void *K_new, const void *V_new,
                const int32_t *topk_idx, int32_t k, const int32_t *reuse_idx,
                const int32_t *reuse_cnt, int32_t max_evict, void *const *K_shards,
                void *const *V_shards, float *utility, int32_t *n_valid, void *stream);

/* One iteration of Algorithm 1's loop in three launches instead of six (four from 256 query
 * rows per sequence on, where the merge and the utility update are faster apart; per-token routing
 * only): route q -> for every selected shard that is full evict its minimum-utility entry
 * (order: utility ascending, then higher slot first) -> insert the new token's rows there
 * (or at slot n_valid if the shard has room) -> attention over the selected shards (new
 * entry included) -> utility update.  Results are exactly those of the call sequence
 *   pikv_route(q as [B, Hq*D], W_r, bias, ...);          (tq > 1: q[:, 0] as [B, (Hq/tq)*D])
 *   pikv_evict(capacity = S-1, sel_idx = topk_idx, max_evict = 1, compact = 0);
 *   pikv_append(K_new, V_new, topk_idx, reuse = the evict outputs);
 *   pikv_sharded_attn(...); pikv_update_utility(...);
 * with the same argument meanings.  K_new == V_new == NULL skips the evict/insert stage
 * (evicted_* may then be NULL).  evicted_idx is [B,E,1], evicted_cnt [B,E]; scores and
 * slot_coef are required.  Errors: as for the separate calls, every one of them detected
 * before the first launch (a rejected call leaves the cache untouched); INVALID while a
 * profiling event pair is installed (pikv_set_profile_events) and `stream` is being captured
 * into a graph; UNSUPPORTED when route_rows_per_seq != 1.  (Rows of W_r that are a power-of-two
 * number of aligned 16-byte chunks - E * sizeof(element) in {16,32,64,128,256} - take the fast
 * form of the router, any other E the generic one, as in pikv_route.)                       */
int pikv_decode_step(const pikv_desc *desc, const void *q, const void *W_r, const float *bias,
                     const void *K_new, const void *V_new, void *const *K_shards,
                     void *const *V_shards, const void *U_K, const void *U_V, int32_t *n_valid,
                     float *utility, int32_t k, int32_t combine, float scale, float decay,
                     int32_t *topk_idx, float *gates, int32_t *evicted_idx, int32_t *evicted_cnt,
                     float *y, float *row_max, float *row_norm, float *scores, float *slot_coef,
                     void *workspace, size_t workspace_bytes, void *stream);

/* Section 3.2, Table 1 row B: the base round-robin router (no scores, O(1)).  The k selections
 * of routed row r at step `step` are the experts ((step + r) * k + j) mod E, j = 0..k-1, gate
 * 1/k each: consecutive (step, row) pairs take consecutive groups of k experts, so every
 * expert is chosen equally often.  Outputs as pikv_route (topk_idx [rows,k], gates [rows,k]).
 * Errors: INVALID for rows < 0, E not in 1..64, k not in 1..E, step < 0, null outputs.       */
int pikv_route_round_robin(int32_t rows, int32_t E, int32_t k, int64_t step, int32_t *topk_idx,
                           float *gates, void *stream);

/* Section 3.2, Table 1, column "Penalty Term": the additive per-expert term of the penalised
 * routers, kept on the device so that routing feeds back into itself without the host:
 *   PIKV_PENALTY_LOAD_BALANCE (row LB):  bias_e = -coef * (load_e - mean_e' load_e')
 *   PIKV_PENALTY_CACHE_AWARE  (row P):   bias_e = -coef * log(1 + miss_e)
 *   PIKV_PENALTY_ENTROPY      (row E):   bias_e = -coef * (h_e - mean_e' h_e'), h_e = -p_e ln p_e,
 *                                        p_e = load_e / sum_e' load_e' the expert's share of all
 *                                        selections so far (0 ln 0 = 0; zero under uniform load)
 * `load` [E] int32 is a running count of how often each expert was selected; the call first
 * adds this step's selections topk_idx [rows,k] to it (rows*k may be 0), then writes
 * bias [E] float32, to be passed as `bias` to the next pikv_route / pikv_decode_step.
 * `miss` [E] int32 (cache-aware mode only) is maintained by the caller.
 * Errors: INVALID for unknown mode, null load/bias, E not in 1..64, null miss in cache-aware
 * mode, NaN coef.                                                                          */
typedef enum {
    PIKV_PENALTY_LOAD_BALANCE = 0, PIKV_PENALTY_CACHE_AWARE = 1, PIKV_PENALTY_ENTROPY = 2
} pikv_penalty;
int pikv_router_penalty(int32_t mode, const int32_t *topk_idx, int32_t rows, int32_t k, int32_t E,
                        int32_t *load, const int32_t *miss, float coef, float *bias, void *stream);

/* Algorithm 1, (K^, V^) <- C_cmp(K_t, V_t) for the rank-r linear compressor (Section 3.3,
 * Table 2 LoRA rows): codes[b][h'][c] = sum_d x[b][h'][d] * W_enc[h'][c][d], fp32 accumulate,
 * rounded once to the storage dtype (bf16: nearest even), for the new token's keys and - in the
 * same launch, when the three V arguments are given - values.  The codes are what pikv_append /
 * pikv_decode_step insert when desc->rank > 0.
 *   K_full, V_full [B,Hkv,D] dtype;  Wenc_K, Wenc_V [Hkv,rank,D] dtype;
 *   K_codes, V_codes [B,Hkv,rank] dtype out.  V_full = Wenc_V = V_codes = NULL: keys only.
 * Errors: descriptor errors, INVALID for rank == 0, null K arguments, partly given V arguments. */
int pikv_compress(const pikv_desc *desc, const void *K_full, const void *Wenc_K, void *K_codes,
                  const void *V_full, const void *Wenc_V, void *V_codes, void *stream);

/* Section 3.4, Table 3: scheduling policies other than H2O.  Their utilities come from
 * integer bookkeeping per cache entry, all [B,E,S] int32 device arrays owned by the caller:
 *   birth        the step the entry was inserted at
 *   last_access  the step the entry was last accessed at
 *   freq         how often the entry has been accessed
 * `now` is the caller's step counter.  An entry is accessed in a step when the attention
 * mass it received in that step, a_i = sum over the query heads that read it of its
 * probability, exceeds `threshold` (>= 0).  Slots are stable under pikv_evict with
 * compact == 0; after a pikv_evict with compact != 0 call pikv_policy_compact with that call's
 * evicted_idx / evicted_cnt / max_evict and the n_valid it left, and the three arrays' kept
 * entries move down the same way (shards with evicted_cnt <= 0 are left alone).
 *
 * pikv_policy_stamp: bookkeeping of the entry the next pikv_append writes (Algorithm 1
 * Insert) - call it BEFORE that pikv_append, with the same topk_idx / reuse_idx / reuse_cnt /
 * n_valid; the slot rule is the append's (first freed slot, else slot n, nothing if the shard
 * is full): birth = last_access = now, freq = 0.  UNSUPPORTED for per-head routing.
 *
 * pikv_update_utility_tracked: pikv_update_utility plus the access bookkeeping in the same pass
 * over the scores.  utility may be NULL (bookkeeping only).
 *
 * pikv_policy_utility: out[b][e][i] for i < n_valid[b][e] (float32 [B,E,S], other slots untouched):
 *   PIKV_POLICY_H2O       h2o[b][e][i] (the accumulated attention, copied through)
 *   PIKV_POLICY_SL        1 if now - birth < window, else 0 (row SL with t_i the insertion step
 *                         and the threshold tau = now - window)
 *   PIKV_POLICY_LRU       -(now - last_access)
 *   PIKV_POLICY_LRU_PLUS  -(now - last_access) + lambda * freq, one fused multiply-add in fp32
 * protect > 0: entries with now - birth < protect get +inf (never evicted while others remain).
 * Pass `out` as the utility of pikv_evict.  Arrays a policy does not read may be NULL.
 * Errors: descriptor errors; INVALID for null required arrays, unknown policy, negative
 * window / protect / threshold, NaN lambda.                                                   */
typedef enum {
    PIKV_POLICY_H2O = 0, PIKV_POLICY_SL = 1, PIKV_POLICY_LRU = 2, PIKV_POLICY_LRU_PLUS = 3
} pikv_policy;
int pikv_policy_stamp(const pikv_desc *desc, const int32_t *topk_idx, int32_t k,
                      const int32_t *reuse_idx, const int32_t *reuse_cnt, int32_t max_evict,
                      const int32_t *n_valid, int32_t now, int32_t *birth, int32_t *last_access,
                      int32_t *freq, void *stream);
int pikv_update_utility_tracked(const pikv_desc *desc, const float *scores, const float *slot_coef,
                                const int32_t *n_valid, const int32_t *topk_idx, int32_t k,
                                float decay, float *utility, float threshold, int32_t now,
                                int32_t *last_access, int32_t *freq, void *stream);
int pikv_policy_utility(const pikv_desc *desc, int32_t policy, const int32_t *n_valid, int32_t now,
                        float lambda, int32_t window, int32_t protect, const int32_t *birth,
                        const int32_t *last_access, const int32_t *freq, const float *h2o,
                        float *out, void *stream);
/* Router feedback inside the fused step: with a pikv_router_feedback the step's last launch also
 * does what pikv_router_penalty(mode, this step's topk_idx, ...) would do after the step - adds
 * the selections to `load` and writes the penalty for the NEXT step to `bias` - so that closing
 * the loop costs no launch of its own.  `bias` may be the array the step itself was given as its
 * routing bias (it is read by the step's first launch and written by its last).              */
typedef struct {
    int32_t mode;          /* pikv_penalty */
    float coef;
    int32_t *load;         /* [E] device, running selection counts, in place */
    const int32_t *miss;   /* [E] device, PIKV_PENALTY_CACHE_AWARE only */
    float *bias;           /* [E] device, out */
} pikv_router_feedback;

/* pikv_decode_step with a scheduling policy and / or router feedback (same arguments, plus
 * `policy` and `feedback`; NULL, NULL = exactly pikv_decode_step).  With a policy it is the sequence
 *   pikv_route; pikv_policy_utility(policy, ...) into a scratch utility;
 *   pikv_evict(scratch, capacity = S-1, sel_idx = topk_idx, max_evict = 1, compact = 0);
 *   pikv_policy_stamp; pikv_append; pikv_sharded_attn;
 *   pikv_update_utility_tracked(decay, utility, threshold, now, last_access, freq)
 * in the same three launches as pikv_decode_step, with no scratch utility: the entry to evict
 * is chosen on the policy's value computed on the fly (bit-identical to the separate calls).
 * Arrays the policy does not read may be NULL; the new entry is stamped in those given; access
 * bookkeeping runs when last_access and freq are both given (threshold >= 0).  `utility` keeps
 * accumulating the attention (H2O) whatever the policy.
 * With feedback the sequence ends with pikv_router_penalty (bit-identical to that call).
 * Errors: as pikv_decode_step, pikv_policy_utility and pikv_router_penalty.                  */
typedef struct {
    int32_t policy;        /* pikv_policy */
    int32_t now;           /* the caller's step counter */
    float lambda;          /* PIKV_POLICY_LRU_PLUS */
    int32_t window;        /* PIKV_POLICY_SL */
    int32_t protect;       /* > 0: entries younger than this many steps are never evicted */
    float threshold;       /* attention mass above which an entry counts as accessed */
    int32_t *birth;        /* [B,E,S] device arrays */
    int32_t *last_access;
    int32_t *freq;
} pikv_policy_args;
int pikv_decode_step_policy(const pikv_desc *desc, const void *q, const void *W_r, const float *bias,
                            const void *K_new, const void *V_new, void *const *K_shards,
                            void *const *V_shards, const void *U_K, const void *U_V, int32_t *n_valid,
                            float *utility, int32_t k, int32_t combine, float scale, float decay,
                            int32_t *topk_idx, float *gates, int32_t *evicted_idx, int32_t *evicted_cnt,
                            float *y, float *row_max, float *row_norm, float *scores, float *slot_coef,
                            void *workspace, size_t workspace_bytes, void *stream,
                            const pikv_policy_args *policy, const pikv_router_feedback *feedback);
int pikv_policy_compact(const pikv_desc *desc, const int32_t *evicted_idx, const int32_t *evicted_cnt,
                        int32_t max_evict, const int32_t *n_valid, int32_t *birth,
                        int32_t *last_access, int32_t *freq, void *stream);

/* Tuning hook: force the number of row-range splits per (head group, selected shard) used
 * by pikv_sharded_attn and pikv_attn_workspace_bytes (process-wide; 0 restores the built-in
 * choice of one round of resident blocks).  Change it only between calls, and size the
 * workspace after changing it.                                                             */
void pikv_set_attn_split(int32_t nsplit);

/* Profiling hook: two hipEvent_t (created with timing enabled, passed as void*) that every
 * later pikv_sharded_attn / pikv_decode_step call records on its stream immediately before and
 * after launching the split attention pass - the kernel that streams the K/V bytes - so that a
 * caller can time exactly that kernel in its real context with hipEventElapsedTime.  NULL, NULL
 * switches it off (the default).  Process-wide, not thread-safe.  While a pair is installed
 * pikv_decode_step refuses (INVALID) a stream that is being captured into a graph: the records
 * would replay with the graph.                                                             */
void pikv_set_profile_events(void *start_event, void *stop_event);

/* Measurement hook, no part of the method: reads n device buffers of bytes_each bytes once,
 * each cut into `parts` spans (one block of 4 waves per span), with the attention pass's load
 * shape (1 KiB of consecutive bytes per wave load, non-temporal, 16 loads of a wave in flight)
 * and no arithmetic, and writes the xor of each span's 32-bit words to out [n * parts] (buffer-major;
 * span = bytes_each / parts rounded up to 4096 bytes, the last one shorter).  bench.py times
 * it over the same K/V bytes as a step to report what a pass that only has to read them reaches
 * on the machine at hand.  bufs: device array of n device pointers, 16-byte aligned buffers.
 * Errors: INVALID for null pointers, n < 1, parts < 1, bytes_each not a positive multiple of
 * 16, or so many parts that one would be empty.                                              */
int pikv_stream_read_probe(const void *const *bufs, int32_t n, size_t bytes_each, int32_t parts,
                           uint32_t *out, void *stream);

/* Static description of a status code (host string, never NULL).                          */
const char *pikv_strerror(int status);

/* Library version: major*10000 + minor*100 + patch.                                        */
int pikv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PIKV_H */
