/*
 * PiKV decode-step oracle: plain, slow, direct CPU arithmetic in double precision.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check
 * and the benchmark's "cpu_baseline" leg may call it.  It shares no code, header,
 * table or helper with the HIP library and knows nothing about how the GPU path
 * blocks, splits or reorders the work.
 *
 * What it computes (PiKV, arxiv 2508.06526):
 *   route    - Section 3.2: R(q) is a 0/1 mask over E experts with exactly k ones;
 *              Table 1 row "TopK softmax" (optionally with an additive per-expert
 *              penalty, the "Penalty Term" column of the same table).
 *   attend   - Algorithm 1, the f_attn step: attention of the query over the cache
 *              entries of the selected expert shards only; Section 3.3: entries may be
 *              stored as width-d' codes and decoded (here: rank-r linear decoder,
 *              Table 2 rows LoRA / LoRA++ without the bias) before use.
 *   utility  - Section 3.4 / Table 3 row H2O: u_i = a_i, the attention mass an entry
 *              received, accumulated over steps (decay 1) or with a decay < 1.
 *   evict    - Algorithm 1, the scheduling step under bounded memory (Section 3.4):
 *              keep the `capacity` highest-utility entries of a shard.
 *   append   - Algorithm 1, Insert: constant-time write of one new entry per selected
 *              shard into a fixed-capacity buffer (Section 3.1, storage invariants).
 *   policies - Section 3.4 / Table 3 rows SL, LRU, LRU+: utilities from per-entry
 *              insertion / last-access stamps and access counts, fed to the same evict.
 *
 * Every sum is a double; inputs (float or bfloat16 bit patterns) are widened exactly;
 * each output is rounded to float once.  No online softmax, no split reductions, no
 * absorbed projections: a reader can check each loop against the definitions above.
 *
 * Pins (tests marked "not gpu"): softmax/sigmoid closed forms, brute-force sorts,
 * k = E routed attention == dense attention computed by an independent numpy routine,
 * constant-V / zero-q special cases, GQA replication, crop-decoder == zero padding,
 * utility mass conservation, brute-force eviction, LRU == sort by access stamp, the
 * sliding-window property, exact small-integer LRU+ values.  Nothing in the paper prints a
 * worked numeric example, so the choice between readings of the paper (which vector is
 * routed, how gates enter, utility granularity, decay form) is pinned by the task
 * statement only; the arithmetic of each reading is pinned as listed.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_COMBINE_LSE = 0, ORACLE_COMBINE_LOCAL = 1 };

static double load_elem(const void *base, int64_t i, int dtype) {
    if (dtype == ORACLE_F32) return (double)((const float *)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static size_t elem_size(int dtype) { return dtype == ORACLE_F32 ? 4u : 2u; }

/* ------------------------------------------------------------------ route */
/* Section 3.2, Table 1 "TopK softmax": logits = x W_r (+ penalty), p = softmax over
 * all E experts, the mask g has ones at the k largest logits (ties: lower expert index
 * first), listed in descending order; gate weights are p renormalised over the k.     */
typedef struct { double logit; int e; } route_key;

static int route_cmp(const void *a, const void *b) {
    const route_key *x = a, *y = b;
    if (x->logit > y->logit) return -1;
    if (x->logit < y->logit) return 1;
    return (x->e > y->e) - (x->e < y->e);
}

int pikv_oracle_route(const void *x, const void *W_r, const float *bias, int rows, int d_r,
                      int E, int k, int dtype, int32_t *topk_idx, float *gates,
                      float *probs, double *logits) {
    if (rows < 0 || d_r < 1 || E < 1 || k < 1 || k > E) return -1;
    route_key *key = malloc(sizeof(route_key) * (size_t)E);
    double *p = malloc(sizeof(double) * (size_t)E);
    if (!key || !p) { free(key); free(p); return -2; }
    for (int r = 0; r < rows; ++r) {
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int j = 0; j < d_r; ++j)
                acc += load_elem(x, (int64_t)r * d_r + j, dtype) *
                       load_elem(W_r, (int64_t)j * E + e, dtype);
            if (bias) acc += (double)bias[e];
            if (isnan(acc)) acc = -INFINITY;
            key[e].logit = acc;
            key[e].e = e;
            if (logits) logits[(int64_t)r * E + e] = acc;
        }
        double mx = -INFINITY;
        for (int e = 0; e < E; ++e) if (key[e].logit > mx) mx = key[e].logit;
        double den = 0.0;
        for (int e = 0; e < E; ++e) { p[e] = exp(key[e].logit - mx); den += p[e]; }
        for (int e = 0; e < E; ++e) {
            p[e] /= den;
            if (probs) probs[(int64_t)r * E + e] = (float)p[e];
        }
        qsort(key, (size_t)E, sizeof(route_key), route_cmp);
        double sel = 0.0;
        for (int j = 0; j < k; ++j) sel += p[key[j].e];
        for (int j = 0; j < k; ++j) {
            topk_idx[(int64_t)r * k + j] = key[j].e;
            gates[(int64_t)r * k + j] = (float)(p[key[j].e] / sel);
        }
    }
    free(key);
    free(p);
    return 0;
}

/* ----------------------------------------------------------------- attend */
/* One (sequence b, query head h): attention over the selected shards, then the
 * per-entry probabilities.  Row r of a shard's K for kv head hk is
 * K[hk*stride_h + r*stride_s + 0..w), w = D (dense) or rank (codes).                  */
static void entry_vector(const void *shard, int hk, int row, int64_t stride_h,
                         int64_t stride_s, int D, int rank, const void *U, const void *U_bias,
                         int dtype, double *out /*[D]*/) {
    int64_t base = (int64_t)hk * stride_h + (int64_t)row * stride_s;
    if (rank == 0) {
        for (int d = 0; d < D; ++d) out[d] = load_elem(shard, base + d, dtype);
        return;
    }
    /* Section 3.3: decoder D(.) of a rank-r code, x_d = sum_c code_c * U[hk][c][d]; with the
     * additive term b of Table 2's LoRA++ row (reconstruction W_d W_u K + b) when given.     */
    for (int d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int c = 0; c < rank; ++c)
            acc += load_elem(shard, base + c, dtype) *
                   load_elem(U, ((int64_t)hk * rank + c) * D + d, dtype);
        if (U_bias) acc += load_elem(U_bias, (int64_t)hk * D + d, dtype);
        out[d] = acc;
    }
}

int pikv_oracle_attend(int B, int Hq, int Hkv, int D, int E, int S, int rank, int dtype,
                       int64_t stride_h, int64_t stride_s, int route_rows_per_seq,
                       const void *q, const void *const *K_shards,
                       const void *const *V_shards, const void *U_K, const void *U_V,
                       const void *V_bias /*[Hkv,D] or NULL: LoRA++ decoder bias of the values*/,
                       const int32_t *n_valid, const int32_t *topk_idx, const float *gates,
                       int k, int combine, double scale, float *y, float *row_max,
                       float *row_norm, double *prob /*[B,Hq,k,S] or NULL*/, double decay,
                       float *utility /*[B,E,S] or NULL*/) {
    if (B < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || D < 1 || E < 1 || S < 1 || k < 1 || k > E)
        return -1;
    if (route_rows_per_seq != 1 && route_rows_per_seq != Hq) return -1;
    if (rank < 0 || (rank > 0 && (!U_K || !U_V))) return -1;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)D);
    const int G = Hq / Hkv;
    const int64_t per_head = (int64_t)k * S;
    double *pbuf = prob;
    if (!pbuf) {
        pbuf = malloc(sizeof(double) * (size_t)B * Hq * per_head);
        if (!pbuf) return -2;
    }
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            const int hk = h / G;
            const int row = b * route_rows_per_seq + (route_rows_per_seq == 1 ? 0 : h);
            const int32_t *sel = topk_idx + (int64_t)row * k;
            const float *gsel = gates ? gates + (int64_t)row * k : NULL;
            double *p = pbuf + ((int64_t)b * Hq + h) * per_head;
            double *kv = malloc(sizeof(double) * (size_t)D);
            double *o = malloc(sizeof(double) * (size_t)k * D);   /* o_e, per shard */
            double *m = malloc(sizeof(double) * (size_t)k);
            double *Z = malloc(sizeof(double) * (size_t)k);
            if (!kv || !o || !m || !Z) {
                fail = 1;
                free(kv); free(o); free(m); free(Z);
                continue;
            }
            for (int64_t i = 0; i < per_head; ++i) p[i] = 0.0;
            /* per-shard softmax attention: s_i, m_e, Z_e, o_e */
            for (int j = 0; j < k; ++j) {
                const int e = sel[j];
                const int n = n_valid[(int64_t)b * E + e];
                m[j] = -INFINITY;
                Z[j] = 0.0;
                for (int d = 0; d < D; ++d) o[(int64_t)j * D + d] = 0.0;
                if (n <= 0) continue;
                const void *Ks = K_shards[(int64_t)b * E + e];
                const void *Vs = V_shards[(int64_t)b * E + e];
                double *s = p + (int64_t)j * S;          /* scores, reused for e^{s-m} */
                for (int i = 0; i < n; ++i) {
                    entry_vector(Ks, hk, i, stride_h, stride_s, D, rank, U_K, NULL, dtype, kv);
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d)
                        dot += load_elem(q, ((int64_t)b * Hq + h) * D + d, dtype) * kv[d];
                    s[i] = scale * dot;
                    if (s[i] > m[j]) m[j] = s[i];
                }
                for (int i = 0; i < n; ++i) {
                    s[i] = exp(s[i] - m[j]);
                    Z[j] += s[i];
                }
                for (int i = 0; i < n; ++i) {
                    entry_vector(Vs, hk, i, stride_h, stride_s, D, rank, U_V, V_bias, dtype, kv);
                    for (int d = 0; d < D; ++d) o[(int64_t)j * D + d] += s[i] * kv[d];
                }
                for (int d = 0; d < D; ++d) o[(int64_t)j * D + d] /= Z[j];
            }
            /* combine the non-empty selected shards */
            float *yo = y + ((int64_t)b * Hq + h) * D;
            for (int d = 0; d < D; ++d) yo[d] = 0.0f;
            double M = -INFINITY;
            int any = 0;
            for (int j = 0; j < k; ++j)
                if (Z[j] > 0.0) { any = 1; if (m[j] > M) M = m[j]; }
            double norm = 0.0;
            if (any) {
                double *acc = kv;                         /* reuse as [D] accumulator  */
                for (int d = 0; d < D; ++d) acc[d] = 0.0;
                if (combine == ORACLE_COMBINE_LSE) {
                    /* joint softmax over the union of the shards, each entry weighted
                     * by its shard's gate: p_i = g_e e^{s_i-M} / Zn                    */
                    for (int j = 0; j < k; ++j)
                        if (Z[j] > 0.0) norm += (gsel ? (double)gsel[j] : 1.0) * Z[j] * exp(m[j] - M);
                    for (int j = 0; j < k; ++j) {
                        if (!(Z[j] > 0.0)) continue;
                        const double g = gsel ? (double)gsel[j] : 1.0;
                        const double w = g * Z[j] * exp(m[j] - M) / norm;
                        for (int d = 0; d < D; ++d) acc[d] += w * o[(int64_t)j * D + d];
                        const int n = n_valid[(int64_t)b * E + sel[j]];
                        double *pj = p + (int64_t)j * S;
                        for (int i = 0; i < n; ++i) pj[i] = g * pj[i] * exp(m[j] - M) / norm;
                    }
                } else {
                    /* per-shard softmax, outputs mixed by the renormalised gates      */
                    for (int j = 0; j < k; ++j)
                        if (Z[j] > 0.0) norm += gsel ? (double)gsel[j] : 1.0;
                    for (int j = 0; j < k; ++j) {
                        if (!(Z[j] > 0.0)) continue;
                        const double gh = (gsel ? (double)gsel[j] : 1.0) / norm;
                        for (int d = 0; d < D; ++d) acc[d] += gh * o[(int64_t)j * D + d];
                        const int n = n_valid[(int64_t)b * E + sel[j]];
                        double *pj = p + (int64_t)j * S;
                        for (int i = 0; i < n; ++i) pj[i] = gh * pj[i] / Z[j];
                    }
                }
                for (int d = 0; d < D; ++d) yo[d] = (float)acc[d];
            }
            if (row_max) row_max[(int64_t)b * Hq + h] = any ? (float)M : -INFINITY;
            if (row_norm) row_norm[(int64_t)b * Hq + h] = (float)norm;
            free(kv); free(o); free(m); free(Z);
        }
    }
    if (fail) { if (!prob) free(pbuf); return -2; }

    /* Section 3.4, Table 3 (H2O): u_i <- decay*u_i + a_i, a_i = sum over the query
     * heads that read entry i of its attention probability.  Only shards that some
     * head visited this step (and that hold entries) are touched.                      */
    if (utility) {
#pragma omp parallel for collapse(2) schedule(dynamic)
        for (int b = 0; b < B; ++b) {
            for (int e = 0; e < E; ++e) {
                const int n = n_valid[(int64_t)b * E + e];
                if (n <= 0) continue;
                int visited = 0;
                for (int h = 0; h < Hq && !visited; ++h) {
                    const int row = b * route_rows_per_seq + (route_rows_per_seq == 1 ? 0 : h);
                    for (int j = 0; j < k; ++j)
                        if (topk_idx[(int64_t)row * k + j] == e) visited = 1;
                }
                if (!visited) continue;
                float *u = utility + ((int64_t)b * E + e) * S;
                for (int i = 0; i < n; ++i) {
                    double a = 0.0;
                    for (int h = 0; h < Hq; ++h) {
                        const int row = b * route_rows_per_seq + (route_rows_per_seq == 1 ? 0 : h);
                        for (int j = 0; j < k; ++j)
                            if (topk_idx[(int64_t)row * k + j] == e)
                                a += pbuf[(((int64_t)b * Hq + h) * k + j) * S + i];
                    }
                    u[i] = (float)(decay * (double)u[i] + a);
                }
            }
        }
    }
    if (!prob) free(pbuf);
    return 0;
}

/* ------------------------------------------------------------------ evict */
/* Algorithm 1 scheduling step, Section 3.4: a shard holding n > capacity entries keeps
 * the `capacity` entries that come first when ordered by (utility descending, slot
 * ascending) - a full sort - and evicts the rest, reported in ascending slot order.
 * compact != 0 moves the kept rows (K, V, utility) down to slots 0..capacity-1 in
 * ascending original-slot order.  n becomes capacity.                                 */
typedef struct { float u; int slot; } evict_key;

static int evict_cmp(const void *a, const void *b) {
    const evict_key *x = a, *y = b;
    if (x->u > y->u) return -1;
    if (x->u < y->u) return 1;
    return (x->slot > y->slot) - (x->slot < y->slot);
}

static int int_cmp(const void *a, const void *b) {
    int x = *(const int *)a, y = *(const int *)b;
    return (x > y) - (x < y);
}

int pikv_oracle_evict(int B, int E, int S, int Hkv, int width, int dtype, int64_t stride_h,
                      int64_t stride_s, float *utility, int32_t *n_valid, int capacity,
                      const int32_t *shard_mask, int32_t *evicted_idx, int32_t *evicted_cnt,
                      int max_evict, int compact, void *const *K_shards,
                      void *const *V_shards) {
    if (capacity < 0 || max_evict < 0) return -1;
    evict_key *key = malloc(sizeof(evict_key) * (size_t)S);
    int *gone = malloc(sizeof(int) * (size_t)S);
    char *is_gone = malloc((size_t)S);
    if (!key || !gone || !is_gone) { free(key); free(gone); free(is_gone); return -2; }
    const size_t es = elem_size(dtype);
    int rc = 0;
    for (int b = 0; b < B && !rc; ++b) {
        for (int e = 0; e < E; ++e) {
            const int64_t be = (int64_t)b * E + e;
            evicted_cnt[be] = 0;
            if (shard_mask && !shard_mask[be]) continue;
            const int n = n_valid[be];
            if (n <= capacity) continue;
            const int ngone = n - capacity;
            if (ngone > max_evict) { rc = -3; break; }
            float *u = utility + be * S;
            for (int i = 0; i < n; ++i) { key[i].u = u[i]; key[i].slot = i; }
            qsort(key, (size_t)n, sizeof(evict_key), evict_cmp);
            for (int i = 0; i < ngone; ++i) gone[i] = key[capacity + i].slot;
            qsort(gone, (size_t)ngone, sizeof(int), int_cmp);
            for (int i = 0; i < ngone; ++i) evicted_idx[be * max_evict + i] = gone[i];
            evicted_cnt[be] = ngone;
            if (compact) {
                memset(is_gone, 0, (size_t)n);
                for (int i = 0; i < ngone; ++i) is_gone[gone[i]] = 1;
                int dst = 0;
                for (int src = 0; src < n; ++src) {
                    if (is_gone[src]) continue;
                    if (dst != src) {
                        u[dst] = u[src];
                        for (int hk = 0; hk < Hkv; ++hk) {
                            const int64_t so = ((int64_t)hk * stride_h + (int64_t)src * stride_s);
                            const int64_t dk = ((int64_t)hk * stride_h + (int64_t)dst * stride_s);
                            if (K_shards)
                                memmove((char *)K_shards[be] + dk * es,
                                        (char *)K_shards[be] + so * es, (size_t)width * es);
                            if (V_shards)
                                memmove((char *)V_shards[be] + dk * es,
                                        (char *)V_shards[be] + so * es, (size_t)width * es);
                        }
                    }
                    ++dst;
                }
            }
            n_valid[be] = capacity;
        }
    }
    free(key); free(gone); free(is_gone);
    return rc;
}

/* ----------------------------------------------------------------- append */
/* Algorithm 1 Insert / Section 3.1 storage invariants: each selected shard of sequence
 * b receives the new entry (one row per kv head) in O(1): into the slot an eviction
 * just freed (reuse_cnt > 0: first listed slot), otherwise at slot n.  The entry's
 * utility starts at 0 and the shard's entry count grows by one.                       */
int pikv_oracle_append(int B, int E, int S, int Hkv, int width, int dtype, int64_t stride_h,
                       int64_t stride_s, const void *K_new, const void *V_new,
                       const int32_t *topk_idx, int k, const int32_t *reuse_idx,
                       const int32_t *reuse_cnt, int max_evict, void *const *K_shards,
                       void *const *V_shards, float *utility, int32_t *n_valid) {
    const size_t es = elem_size(dtype);
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < k; ++j) {
            const int e = topk_idx[(int64_t)b * k + j];
            const int64_t be = (int64_t)b * E + e;
            int slot = n_valid[be];
            if (reuse_cnt && reuse_cnt[be] > 0) slot = reuse_idx[be * max_evict];
            if (slot < 0 || slot >= S || n_valid[be] >= S) return -3;
            for (int hk = 0; hk < Hkv; ++hk) {
                const int64_t dst = (int64_t)hk * stride_h + (int64_t)slot * stride_s;
                const int64_t src = ((int64_t)b * Hkv + hk) * width;
                memcpy((char *)K_shards[be] + dst * es, (const char *)K_new + src * es,
                       (size_t)width * es);
                memcpy((char *)V_shards[be] + dst * es, (const char *)V_new + src * es,
                       (size_t)width * es);
            }
            utility[be * S + slot] = 0.0f;
            n_valid[be] += 1;
        }
    }
    return 0;
}

/* --------------------------------------------------------- router penalties */
/* Section 3.2, Table 1, column "Penalty Term": the additive per-expert term of the
 * load-balanced router (row LB: -alpha * (mu_e - mean mu), mu_e = how often expert e has been
 * selected so far) and of the cache-aware router (row P: -lambda * log(1 + miss_e)).
 * `load` first absorbs this step's selections (rows x k expert ids), then the penalty is
 * formed from the updated counters.  mode 0 = LB, 1 = P (needs `miss`).                   */
int pikv_oracle_router_penalty(int mode, const int32_t *topk_idx, int rows, int k, int E,
                               int32_t *load, const int32_t *miss, double coef, float *bias) {
    if (E < 1 || rows < 0 || k < 0 || mode < 0 || mode > 2 || (mode == 1 && !miss)) return -1;
    for (int i = 0; i < rows * k; ++i) {
        if (topk_idx[i] < 0 || topk_idx[i] >= E) return -1;
        load[topk_idx[i]] += 1;
    }
    if (mode == 0) {
        double mean = 0.0;
        for (int e = 0; e < E; ++e) mean += (double)load[e];
        mean /= (double)E;
        for (int e = 0; e < E; ++e) bias[e] = (float)(-coef * ((double)load[e] - mean));
    } else if (mode == 1) {
        for (int e = 0; e < E; ++e) bias[e] = (float)(-coef * log(1.0 + (double)miss[e]));
    } else {
        /* Table 1 row E, -beta H(p_e): p_e is expert e's share of all selections so far and
         * H(p_e) = -p_e ln p_e its term of the entropy of that distribution (0 ln 0 = 0).  A
         * shift common to all experts does not change any routing decision; the term is
         * centred like the load-balance row's, so that it vanishes under uniform load.       */
        double total = 0.0, h_avg = 0.0;
        for (int e = 0; e < E; ++e) total += (double)load[e];
        for (int e = 0; e < E; ++e) {
            const double pe = total > 0.0 ? (double)load[e] / total : 0.0;
            h_avg += pe > 0.0 ? -pe * log(pe) : 0.0;
        }
        h_avg /= (double)E;
        for (int e = 0; e < E; ++e) {
            const double pe = total > 0.0 ? (double)load[e] / total : 0.0;
            const double he = pe > 0.0 ? -pe * log(pe) : 0.0;
            bias[e] = (float)(-coef * (he - h_avg));
        }
    }
    return 0;
}

/* ------------------------------------------------------- compress on insert */
/* Algorithm 1, (K^,V^) <- C_cmp(K_t,V_t) with the rank-r linear compressor of Section 3.3 /
 * Table 2 (LoRA rows: the width-d' code is a linear map of the width-d vector):
 * code[b][h'][c] = sum_d x[b][h'][d] * W_enc[h'][c][d], rounded once to the storage dtype
 * (bfloat16: round to nearest even).                                                      */
static uint16_t double_to_bf16(double v) {
    float f = (float)v;                 /* double -> float, then float -> bf16, both RNE   */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int pikv_oracle_compress(int B, int Hkv, int D, int rank, int dtype, const void *x,
                         const void *W_enc, void *codes) {
    if (B < 0 || Hkv < 1 || D < 1 || rank < 1) return -1;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h)
            for (int c = 0; c < rank; ++c) {
                double acc = 0.0;
                for (int d = 0; d < D; ++d)
                    acc += load_elem(x, ((int64_t)b * Hkv + h) * D + d, dtype) *
                           load_elem(W_enc, ((int64_t)h * rank + c) * D + d, dtype);
                const int64_t o = ((int64_t)b * Hkv + h) * rank + c;
                if (dtype == ORACLE_F32) ((float *)codes)[o] = (float)acc;
                else ((uint16_t *)codes)[o] = double_to_bf16(acc);
            }
    return 0;
}

/* ------------------------------------------------------- scheduling policies */
/* Section 3.4, Table 3: utilities built from integer bookkeeping per entry instead of the
 * attention mass: r_i = recency = steps since the entry was last accessed, f_i = how often
 * it has been accessed, and the step it was inserted at.  `now` is the caller's step
 * counter.  Rows of the table covered here:
 *   SL    u_i = 1 if the entry was inserted inside the last `window` steps, else 0
 *         (the indicator of the table with t_i read as the insertion step and the
 *         threshold tau = now - window);
 *   LRU   u_i = -r_i;
 *   LRU+  u_i = -r_i + lambda * f_i, rounded once to float (a fused multiply-add);
 *   H2O   u_i = the accumulated attention (copied through, so that one call serves all).
 * protect > 0 shields the entries younger than `protect` steps: their utility is +inf.  */

/* Insert bookkeeping (Algorithm 1 Insert): the entry that pikv_oracle_append is about to
 * write for each selected shard - into the first freed slot if an eviction freed one,
 * else at slot n; a full shard is an error, as it is for the append - starts with
 * birth = last access = now and frequency 0.  Call with n_valid as it is BEFORE the append. */
int pikv_oracle_policy_stamp(int B, int E, int S, int k, const int32_t *topk_idx,
                             const int32_t *reuse_idx, const int32_t *reuse_cnt, int max_evict,
                             const int32_t *n_valid, int now, int32_t *birth,
                             int32_t *last_access, int32_t *freq) {
    if (B < 0 || E < 1 || S < 1 || k < 1 || k > E) return -1;
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < k; ++j) {
            const int e = topk_idx[(int64_t)b * k + j];
            if (e < 0 || e >= E) return -1;
            const int64_t be = (int64_t)b * E + e;
            int slot = n_valid[be];
            if (reuse_cnt && reuse_cnt[be] > 0) slot = reuse_idx[be * max_evict];
            if (slot < 0 || slot >= S || n_valid[be] >= S) return -3;
            birth[be * S + slot] = now;
            last_access[be * S + slot] = now;
            freq[be * S + slot] = 0;
        }
    }
    return 0;
}

/* An entry counts as accessed in a step when the attention mass it received in that
 * step, a_i = sum over query heads of its probability, exceeds `threshold` (>= 0).      */
int pikv_oracle_policy_access(int B, int E, int S, const int32_t *n_valid, const float *mass,
                              float threshold, int now, int32_t *last_access, int32_t *freq) {
    if (B < 0 || E < 1 || S < 1 || !(threshold >= 0.0f)) return -1;
    for (int64_t be = 0; be < (int64_t)B * E; ++be) {
        for (int i = 0; i < n_valid[be]; ++i) {
            if (mass[be * S + i] > threshold) {
                last_access[be * S + i] = now;
                freq[be * S + i] += 1;
            }
        }
    }
    return 0;
}

int pikv_oracle_policy_utility(int policy, int B, int E, int S, const int32_t *n_valid, int now,
                               float lambda, int window, int protect, const int32_t *birth,
                               const int32_t *last_access, const int32_t *freq,
                               const float *h2o, float *out) {
    if (B < 0 || E < 1 || S < 1 || policy < 0 || policy > 3) return -1;
    if (policy == 0 && !h2o) return -1;
    for (int64_t be = 0; be < (int64_t)B * E; ++be) {
        for (int i = 0; i < n_valid[be]; ++i) {
            const int64_t x = be * S + i;
            float u;
            if (policy == 0) {
                u = h2o[x];
            } else if (policy == 1) {
                u = (now - birth[x] < window) ? 1.0f : 0.0f;
            } else {
                const float r = (float)(now - last_access[x]);
                u = (policy == 2) ? -r : fmaf(lambda, (float)freq[x], -r);
            }
            if (protect > 0 && now - birth[x] < protect) u = INFINITY;
            out[x] = u;
        }
    }
    return 0;
}

/* Compaction of the bookkeeping arrays after an eviction that compacted the shard
 * (pikv_oracle_evict with compact != 0): the kept entries' stamps and counts move down
 * with them, in ascending original-slot order.  evicted lists the removed slots
 * (ascending) per shard, n_valid is the entry count AFTER the eviction.                */
int pikv_oracle_policy_compact(int B, int E, int S, const int32_t *evicted_idx,
                               const int32_t *evicted_cnt, int max_evict, const int32_t *n_valid,
                               int32_t *birth, int32_t *last_access, int32_t *freq) {
    if (B < 0 || E < 1 || S < 1 || max_evict < 1) return -1;
    for (int64_t be = 0; be < (int64_t)B * E; ++be) {
        const int cnt = evicted_cnt[be];
        if (cnt <= 0) continue;
        const int n_old = n_valid[be] + cnt;
        if (n_old > S || cnt > max_evict) return -1;
        const int32_t *gone = evicted_idx + be * max_evict;
        int out = 0, g = 0;
        for (int i = 0; i < n_old; ++i) {
            if (g < cnt && gone[g] == i) { ++g; continue; }
            birth[be * S + out] = birth[be * S + i];
            last_access[be * S + out] = last_access[be * S + i];
            freq[be * S + out] = freq[be * S + i];
            ++out;
        }
        if (out != n_valid[be]) return -1;
    }
    return 0;
}

/* Section 3.2, Table 1 row B (base round-robin router, no scores): the k selections of
 * routed row r at step t are the experts ((t + r) * k + j) mod E, j = 0..k-1, each with
 * gate 1/k - consecutive (step, row) pairs take consecutive groups of k experts, so over
 * any E consecutive pairs every expert is chosen exactly k times.                        */
int pikv_oracle_route_round_robin(int rows, int E, int k, int64_t step, int32_t *topk_idx,
                                  float *gates) {
    if (rows < 0 || E < 1 || k < 1 || k > E || step < 0) return -1;
    for (int r = 0; r < rows; ++r) {
        for (int j = 0; j < k; ++j) {
            topk_idx[(int64_t)r * k + j] = (int32_t)(((step + r) * k + j) % E);
            gates[(int64_t)r * k + j] = (float)(1.0 / (double)k);
        }
    }
    return 0;
}

