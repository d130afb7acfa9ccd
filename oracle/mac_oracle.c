/*
 * CPU oracle for the MAC-Attention decode path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain C, fp64 throughout, no blocking, no fusion, no reordering beyond what
 * the paper's definitions state.  It shares no code with the HIP library and
 * is used only by the tests, by the smoke check and by the benchmark's
 * cpu_baseline leg.  Inputs are the same bf16 bit patterns the GPU path gets,
 * widened exactly to double.
 *
 * What follows the paper:
 *   - attention output and logits: Sec. 2 "Notation"
 *       l_t = Q^T K_t / sqrt(d);  o = S / Z,  S = sum_t e^{l_t} V_t,  Z = sum_t e^{l_t}
 *   - attention summary of an index set and merging of disjoint sets: Sec. 3.1
 *   - match: pre-RoPE L2 test of Eq. (accept) over the last W queries, Sec. 3.2.3, Sec. 3.5 step 1
 *   - amend + complete: Eq. (rect-recomp), Eq. (rect-merge), Sec. 3.5 steps 2-3
 *   - rectify-append (ring write-back): Fig. 1(c), Sec. 4.1, Sec. 4.2 "K3"
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - kv_len n counts the current token (the sum runs over t <= m);
 *   - hit iff d^2 < T^2, strict, on squared values; T = sqrt(2d)(1 - tau);
 *   - nearest candidate first (ties -> the most recent one), then the threshold;
 *   - candidates are ring entries created at lengths n_p in [n - W, n - 1];
 *   - an entry created at length n_p summarises keys [0, n_p - B) (0-based);
 *     on a hit the fresh part is [max(0, n_p - B), n);
 *   - the summary stored at a step is that step's (partly reused) total with
 *     the last-B band removed:  rect = prefix (+) fresh[s, n-B)  (add-only form
 *     of "total minus band"), so summaries chain across consecutive hits;
 *   - every step inserts, hit or miss; rings start empty.
 * Two variants beyond the per-head test (both off by default):
 *   - distance cap (appendix on prefill, "Recommendations" (i); App. B.3 "Common issues" (2)): the nearest
 *     candidate is accepted only if it also lies at most max_gap positions back, n - n_p <= max_gap;
 *   - one reuse point per KV group instead of per query head (the paper matches per query head, Sec. 4;
 *     this variant removes the skew inside a group of Sec. 5.8): the distance of a candidate is that of
 *     the group's concatenated pre-RoPE queries, D^2_j = sum over the group's heads of d^2_{h,j}; argmin
 *     and tie-break as above; hit iff D^2 < G T^2 (root-mean-square per-head distance below T); every
 *     head of the group takes the same reuse point.
 *
 * Summaries are carried in the numerically stable form (O, LSE): O = S/Z,
 * LSE = M + ln(sum e^{l - M}); the empty set is (0, -inf).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf16_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

typedef struct {
    int32_t batch, num_q_heads, num_kv_heads, head_dim, page_size;
    int32_t window, band;
    double threshold;      /* T */
    double sm_scale;       /* 1/sqrt(d) */
    int64_t stride_page, stride_kv, stride_head, stride_tok;   /* elements */
    int32_t block_table_stride;
    int32_t num_threads;   /* 0 = OpenMP default */
    int32_t max_gap;       /* distance cap: accept only n - n_p <= max_gap; 0 = no cap */
    int32_t group_match;   /* 0 = one reuse point per query head, 1 = per KV group */
} oracle_params;

typedef struct {
    uint64_t steps, head_steps, hits, misses, sum_gap, kv_tokens_read, kv_tokens_full;
    double sum_skip_frac;
} oracle_stats;

/* address of row t of K (kv=0) or V (kv=1) of kv head g for request b */
static inline const uint16_t *kv_row(const oracle_params *P, const uint16_t *kv_pages,
                                     const int32_t *block_table, int b, int kv, int g, int64_t t) {
    int64_t page = block_table[(int64_t)b * P->block_table_stride + t / P->page_size];
    int64_t within = t % P->page_size;
    return kv_pages + page * P->stride_page + kv * P->stride_kv + g * P->stride_head + within * P->stride_tok;
}

/* Attention summary of keys [lo, hi) under query q (bf16 bits), Sec. 2 / Sec. 3.1.
 * Two plain passes: logits and their max, then the shifted sums. */
static void summary(const oracle_params *P, const uint16_t *kv_pages, const int32_t *block_table,
                    int b, int g, const uint16_t *q, int64_t lo, int64_t hi, double *O, double *lse) {
    int d = P->head_dim;
    for (int i = 0; i < d; ++i) O[i] = 0.0;
    if (hi <= lo) { *lse = -INFINITY; return; }
    int64_t cnt = hi - lo;
    double *logit = (double *)malloc(sizeof(double) * (size_t)cnt);
    double M = -INFINITY;
    for (int64_t t = lo; t < hi; ++t) {
        const uint16_t *k = kv_row(P, kv_pages, block_table, b, 0, g, t);
        double dot = 0.0;
        for (int i = 0; i < d; ++i) dot += bf16_to_double(q[i]) * bf16_to_double(k[i]);
        double l = dot * P->sm_scale;
        logit[t - lo] = l;
        if (l > M) M = l;
    }
    double Z = 0.0;
    for (int64_t t = lo; t < hi; ++t) {
        double w = exp(logit[t - lo] - M);
        const uint16_t *v = kv_row(P, kv_pages, block_table, b, 1, g, t);
        Z += w;
        for (int i = 0; i < d; ++i) O[i] += w * bf16_to_double(v[i]);
    }
    for (int i = 0; i < d; ++i) O[i] /= Z;
    *lse = M + log(Z);
    free(logit);
}

/* Log-domain merge of two summaries over disjoint sets, Sec. 3.1 (sum of S and of Z):
 * with weights e^{LSE_a}, e^{LSE_b}:  O = (e^{LSE_a} O_a + e^{LSE_b} O_b) / (e^{LSE_a} + e^{LSE_b}). */
static void merge(int d, const double *Oa, double la, const double *Ob, double lb, double *O, double *l) {
    if (la == -INFINITY && lb == -INFINITY) {
        for (int i = 0; i < d; ++i) O[i] = 0.0;
        *l = -INFINITY;
        return;
    }
    double M = la > lb ? la : lb;
    double wa = exp(la - M), wb = exp(lb - M);
    double Z = wa + wb;
    for (int i = 0; i < d; ++i) O[i] = (wa * Oa[i] + wb * Ob[i]) / Z;
    *l = M + log(Z);
}

void oracle_merge(int32_t d, const double *Oa, double la, const double *Ob, double lb, double *O, double *l) {
    merge(d, Oa, la, Ob, lb, O, l);
}

/* summary of [lo, hi) for one (request, q head); exported for the tests */
void oracle_summary(const oracle_params *P, const uint16_t *q_rope, const uint16_t *kv_pages,
                    const int32_t *block_table, int32_t b, int32_t h, int64_t lo, int64_t hi,
                    double *O, double *lse) {
    int G = P->num_q_heads / P->num_kv_heads;
    const uint16_t *q = q_rope + ((int64_t)b * P->num_q_heads + h) * P->head_dim;
    summary(P, kv_pages, block_table, b, h / G, q, lo, hi, O, lse);
}

/* Full decode attention: out = summary of [0, n).O for every (request, head). Sec. 2. */
void oracle_full_decode(const oracle_params *P, const int32_t *kv_lens, const uint16_t *q_rope,
                        const uint16_t *kv_pages, const int32_t *block_table,
                        double *out /*[batch,Hq,d]*/, double *out_lse /*[batch,Hq]*/) {
    int Hq = P->num_q_heads, d = P->head_dim, G = Hq / P->num_kv_heads;
    int total = P->batch * Hq;
#ifdef _OPENMP
    if (P->num_threads > 0) omp_set_num_threads(P->num_threads);
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < total; ++bh) {
        int b = bh / Hq, h = bh % Hq;
        const uint16_t *q = q_rope + (int64_t)bh * d;
        summary(P, kv_pages, block_table, b, h / G, q, 0, kv_lens[b], out + (int64_t)bh * d, out_lse + bh);
    }
}

/* Squared L2 distance of two bf16 rows, Eq. (accept), accumulated in index order. */
static double sq_dist(const uint16_t *a, const uint16_t *b, int d) {
    double d2 = 0.0;
    for (int i = 0; i < d; ++i) {
        double diff = bf16_to_double(a[i]) - bf16_to_double(b[i]);
        d2 += diff * diff;
    }
    return d2;
}

/* Match, Sec. 3.5 step 1 / Eq. (accept): nearest ring entry among those created at lengths
 * n_p in [n - W, n - 1]; squared L2 distance of the pre-RoPE queries of heads [h0, h0 + nh) taken together
 * (nh = 1: the paper's per-head test; nh = G: one reuse point per KV group); ties -> larger n_p;
 * hit iff d^2 < nh T^2 and, with a distance cap, n - n_p <= max_gap.  Returns ring index j (or -1), writes
 * n_p (or -1) and the nearest d^2 (+inf when there is no candidate). */
static int match_one(const oracle_params *P, const uint16_t *q_pre /*[Hq,d] of this request*/,
                     const uint16_t *ring_q /*[W,Hq,d] of this slot*/,
                     const int32_t *ring_npos /*[W]*/, int h0, int nh, int64_t n, int32_t *n_p_out, double *d2_out) {
    int W = P->window, Hq = P->num_q_heads, d = P->head_dim;
    int best = -1;
    int32_t best_np = -1;
    double best_d2 = INFINITY;
    for (int j = 0; j < W; ++j) {
        int32_t np = ring_npos[j];
        if (np < n - W || np > n - 1 || np < 1) continue;      /* empty entries carry n_p = 0 */
        double d2 = 0.0;
        for (int h = h0; h < h0 + nh; ++h)
            d2 += sq_dist(q_pre + (int64_t)h * d, ring_q + ((int64_t)j * Hq + h) * d, d);
        if (best < 0 || d2 < best_d2 || (d2 == best_d2 && np > best_np)) {
            best = j; best_d2 = d2; best_np = np;
        }
    }
    *d2_out = best_d2;
    int ok = best >= 0 && best_d2 < P->threshold * P->threshold * (double)nh;
    if (ok && P->max_gap > 0 && n - best_np > P->max_gap) ok = 0;
    if (ok) { *n_p_out = best_np; return best; }
    *n_p_out = -1;
    return -1;
}

void oracle_match(const oracle_params *P, const int32_t *slot_ids, const int32_t *kv_lens, const uint16_t *q_pre,
                  const uint16_t *ring_q, const int32_t *ring_npos,
                  int32_t *match_pos /*[batch,Hq]*/, int32_t *match_idx /*[batch,Hq]*/, double *match_d2 /*[batch,Hq]*/) {
    int Hq = P->num_q_heads, d = P->head_dim, W = P->window;
    int G = Hq / P->num_kv_heads;
    int nh = P->group_match ? G : 1;
    for (int b = 0; b < P->batch; ++b)
        for (int h0 = 0; h0 < Hq; h0 += nh) {
            int64_t slot = slot_ids[b];
            int bh = b * Hq + h0;
            match_idx[bh] = match_one(P, q_pre + (int64_t)b * Hq * d, ring_q + slot * W * Hq * d,
                                      ring_npos + slot * W, h0, nh, kv_lens[b], &match_pos[bh], &match_d2[bh]);
            for (int k = 1; k < nh; ++k) {      /* the group's heads share the decision */
                match_idx[bh + k] = match_idx[bh]; match_pos[bh + k] = match_pos[bh]; match_d2[bh + k] = match_d2[bh];
            }
        }
}

/* One MAC decode step for the whole batch (Sec. 3.5; Fig. 1 a-c; Sec. 4.2 K1-K3).
 * Ring state (caller-owned, updated in place):
 *   ring_q    bf16 bits [slots, W, Hq, d]   pre-RoPE queries
 *   ring_O    f64       [slots, W, Hq, d]   rectified prefix summary, normalised row
 *   ring_lse  f64       [slots, W, Hq]      its ln-LSE scalar
 *   ring_npos i32       [slots, W]          length n_p at which the entry was created (0 = empty)
 */
void oracle_mac_step(const oracle_params *P, const int32_t *slot_ids, const int32_t *kv_lens,
                     const uint16_t *q_pre, const uint16_t *q_rope,
                     const uint16_t *kv_pages, const int32_t *block_table,
                     uint16_t *ring_q, double *ring_O, double *ring_lse, int32_t *ring_npos,
                     double *out /*[batch,Hq,d]*/, double *out_lse /*[batch,Hq]*/,
                     int32_t *match_pos /*[batch,Hq]*/, double *match_d2 /*[batch,Hq]*/,
                     double *rect_O /*[batch,Hq,d] or NULL*/, double *rect_lse /*[batch,Hq] or NULL*/,
                     oracle_stats *stats /* accumulated, may be NULL */) {
    int Hq = P->num_q_heads, Hkv = P->num_kv_heads, d = P->head_dim, W = P->window, B = P->band;
    int G = Hq / Hkv;
    int total = P->batch * Hq;
    int32_t *midx = (int32_t *)malloc(sizeof(int32_t) * (size_t)total);
    double *rO = (double *)malloc(sizeof(double) * (size_t)total * d);
    double *rL = (double *)malloc(sizeof(double) * (size_t)total);
#ifdef _OPENMP
    if (P->num_threads > 0) omp_set_num_threads(P->num_threads);
#endif

    /* 1. match, every head, against the ring as it stands before this step's insert */
    oracle_match(P, slot_ids, kv_lens, q_pre, ring_q, ring_npos, match_pos, midx, match_d2);

    /* 2. amend + complete */
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < total; ++bh) {
        int b = bh / Hq, h = bh % Hq, g = h / G;
        int64_t slot = slot_ids[b];
        int64_t n = kv_lens[b];
        const uint16_t *q = q_rope + (int64_t)bh * d;
        double prefix_O[1024], mid_O[1024], band_O[1024];
        double prefix_l, mid_l, band_l;
        int64_t s;
        if (midx[bh] >= 0) {                 /* hit: reuse the summary of keys [0, n_p - B) */
            int64_t np = match_pos[bh];
            s = np - B > 0 ? np - B : 0;
            const double *po = ring_O + ((slot * W + midx[bh]) * Hq + h) * d;
            for (int i = 0; i < d; ++i) prefix_O[i] = po[i];
            prefix_l = ring_lse[(slot * W + midx[bh]) * Hq + h];
        } else {                             /* miss: nothing reused */
            s = 0;
            for (int i = 0; i < d; ++i) prefix_O[i] = 0.0;
            prefix_l = -INFINITY;
        }
        int64_t nb = n - B > s ? n - B : s;  /* the band is the last B keys, [n - B, n) */
        summary(P, kv_pages, block_table, b, g, q, s, nb, mid_O, &mid_l);
        summary(P, kv_pages, block_table, b, g, q, nb, n, band_O, &band_l);
        merge(d, prefix_O, prefix_l, mid_O, mid_l, rO + (int64_t)bh * d, &rL[bh]);          /* rectified summary of [0, n-B) */
        merge(d, rO + (int64_t)bh * d, rL[bh], band_O, band_l, out + (int64_t)bh * d, &out_lse[bh]);
    }

    /* 3. rectify-append: after every head has matched and merged, insert into slot (n-1) mod W */
    for (int b = 0; b < P->batch; ++b) {
        int64_t slot = slot_ids[b];
        int64_t n = kv_lens[b];
        if (n < 1) continue;                 /* a request without tokens has no query position: entries are created at lengths n >= 1 */
        int64_t j = (n - 1) % W;
        for (int h = 0; h < Hq; ++h) {
            int bh = b * Hq + h;
            memcpy(ring_q + ((slot * W + j) * Hq + h) * d, q_pre + (int64_t)bh * d, sizeof(uint16_t) * (size_t)d);
            memcpy(ring_O + ((slot * W + j) * Hq + h) * d, rO + (int64_t)bh * d, sizeof(double) * (size_t)d);
            ring_lse[(slot * W + j) * Hq + h] = rL[bh];
        }
        ring_npos[slot * W + j] = (int32_t)n;
    }

    if (rect_O) memcpy(rect_O, rO, sizeof(double) * (size_t)total * d);
    if (rect_lse) memcpy(rect_lse, rL, sizeof(double) * (size_t)total);

    /* 4. statistics: acceptance, reuse gap, skipped-prefix fraction E[(p - r)_+ / m] with misses as 0
     * (Sec. 5.3 "Setup and metrics"), and KV tokens streamed when KV is read once per KV group
     * from the smallest start among the group's heads (Sec. 5.8). */
    if (stats) {
        stats->steps += 1;
        stats->head_steps += (uint64_t)total;
        for (int b = 0; b < P->batch; ++b) {
            int64_t n = kv_lens[b];
            for (int g = 0; g < Hkv; ++g) {
                int64_t gs = n;
                for (int h = g * G; h < (g + 1) * G; ++h) {
                    int bh = b * Hq + h;
                    int64_t s = 0;
                    if (match_pos[bh] >= 0) {
                        int64_t np = match_pos[bh];
                        s = np - B > 0 ? np - B : 0;
                        stats->hits += 1;
                        stats->sum_gap += (uint64_t)(n - np);
                        stats->sum_skip_frac += (double)s / (double)n;
                    } else {
                        stats->misses += 1;
                    }
                    if (s < gs) gs = s;
                }
                stats->kv_tokens_read += (uint64_t)(n - gs);
                stats->kv_tokens_full += (uint64_t)n;
            }
        }
    }
    free(midx); free(rO); free(rL);
}

int32_t oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
