/*
 * CPU oracle for the decode-step hybrid-head attention of LycheeDecode.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the GPU path
 * must compute, written out in fp64 on the exact bf16 input bits.  It shares no code
 * with the HIP library and is never part of the product path; only the tests, the
 * smoke check and the bench's cpu-baseline leg may call it.
 *
 * What it follows (paper sections / equations / algorithms):
 *   - Eq. 1 (Sec. 3.1): a retrieval head's attention map  A_h = softmax(q_h K_h^T / sqrt(d)).
 *   - Eq. 2 (Sec. 3.1): S_h = argsTopK(A_h, k).  Because softmax is strictly increasing
 *     in the logit, the k largest weights are at the k largest scaled logits; the
 *     oracle ranks the scaled logits.
 *   - Eq. 3 (Sec. 3.1): a sparse head's output = softmax over the inherited set only,
 *     times the V rows of that set; the set is handed on unchanged.
 *   - Alg. 1, retrieval branch / sparse branch (App. B): o_h = A_h V_h for a retrieval head.
 *   - App. F (implementation details): under grouped-query attention the query heads
 *     are average-pooled down to the KV heads, giving one token set per KV head.  By
 *     linearity the pooled query's logit is the mean of the pooled heads' logits.
 *
 * Readings where the paper is silent (all listed in the design notes of the repo):
 *   - pooling runs over the retrieval heads of the KV group (R_g); a group with no
 *     retrieval head passes its set on unchanged;
 *   - ties are broken towards the lower position; the returned set is ascending by
 *     position and padded with -1 when k exceeds the sequence length;
 *   - lengths count the current token; no sink / window positions are forced;
 *   - the Ratio rule of Sec. 4.4.1 keeps a budget proportional to the sequence length;
 *     App. E.2's sparsity table shows that its theta is the share of tokens dropped, so
 *     the share kept is 1 - theta.  The oracle takes the kept share in parts per million
 *     and rounds the budget up (the paper does not say how it rounds);
 *   - the block-granular variant: App. C's kernel takes *block* indices (Alg. 2, block size
 *     64 in Sec. 4.3.2) but the paper never says how a block is scored.  Here a block's score
 *     is the largest pooled token score inside it (so the block holding the best token is
 *     always kept), blocks are ranked like tokens (ties to the lower block), a set entry e
 *     names the positions [e*block, (e+1)*block) below the sequence length, and the budget
 *     counts blocks.  block = 1 is the token-granular method itself;
 *   - the Top-p and Threshold rules of Sec. 4.4.1 speak of attention probabilities.  Under
 *     grouped-query attention the set is scored by the pooled query (App. F), so the
 *     probabilities here are the softmax of the pooled logits over the whole sequence.
 *     Threshold keeps the tokens whose probability exceeds tau; Top-p keeps the shortest
 *     prefix of the descending order whose probabilities sum to at least p.  Both keep at
 *     least the best token and at most k (the capacity of a set) - the k best, if the rule
 *     would keep more - and both break ties like Eq. 2 does.
 *
 * Every function is a direct loop nest: no blocking, no fusion, no reordering.
 * OpenMP only spreads the independent (sequence, KV head) pairs over cores.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* bf16 is the upper half of an IEEE fp32: widening is exact. */
static double bf16_to_f64(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Eq. 1, the argument of the softmax:  s[t] = (sum_i q[i] * K[t][i]) / sqrt(d),  t < L.
 * K row t starts at K + t * stride_tok (elements). */
void lo_scores(const uint16_t *q, const uint16_t *K, int64_t stride_tok, int32_t L, int32_t d,
               double *s)
{
    const double inv = 1.0 / sqrt((double)d);
    for (int32_t t = 0; t < L; ++t) {
        double acc = 0.0;
        for (int32_t i = 0; i < d; ++i)
            acc += bf16_to_f64(q[i]) * bf16_to_f64(K[(int64_t)t * stride_tok + i]);
        s[t] = acc * inv;
    }
}

/* Eq. 3, the argument of the softmax on a subset: s[pos[j]] for the listed positions only
 * (the other entries of s are left untouched). */
void lo_scores_at(const uint16_t *q, const uint16_t *K, int64_t stride_tok, const int32_t *pos,
                  int32_t n, int32_t d, double *s)
{
    const double inv = 1.0 / sqrt((double)d);
    for (int32_t j = 0; j < n; ++j) {
        const int32_t t = pos[j];
        double acc = 0.0;
        for (int32_t i = 0; i < d; ++i)
            acc += bf16_to_f64(q[i]) * bf16_to_f64(K[(int64_t)t * stride_tok + i]);
        s[t] = acc * inv;
    }
}

/* Softmax weights of the scores at the listed positions (Eq. 1 when pos is every
 * position, Eq. 3 when pos is the inherited set):  w[j] = exp(s[pos[j]] - m) / Z. */
void lo_softmax_weights(const double *s, const int32_t *pos, int32_t n, double *w)
{
    double m = -INFINITY;
    for (int32_t j = 0; j < n; ++j)
        if (s[pos[j]] > m) m = s[pos[j]];
    double z = 0.0;
    for (int32_t j = 0; j < n; ++j) {
        w[j] = exp(s[pos[j]] - m);
        z += w[j];
    }
    for (int32_t j = 0; j < n; ++j) w[j] /= z;
}

/* o[i] = sum_j w[j] * V[pos[j]][i]   (Alg. 1: o_h = A_h V_h; Eq. 3 on a subset). */
void lo_weighted_values(const double *w, const int32_t *pos, int32_t n, const uint16_t *V,
                        int64_t stride_tok, int32_t d, double *o)
{
    for (int32_t i = 0; i < d; ++i) o[i] = 0.0;
    for (int32_t j = 0; j < n; ++j)
        for (int32_t i = 0; i < d; ++i)
            o[i] += w[j] * bf16_to_f64(V[(int64_t)pos[j] * stride_tok + i]);
}

typedef struct {
    double s;
    int32_t t;
} scored_pos;

static int by_score_desc_then_pos(const void *a, const void *b)
{
    const scored_pos *x = a, *y = b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->t > y->t) - (x->t < y->t);
}

static int by_int_asc(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* The Ratio rule's budget (Sec. 4.4.1: a budget proportional to the sequence length) for a
 * sequence of L rows: ceil(L * keep_ppm / 10^6) positions, at least 1, at most L and at most
 * the capacity k of a set.  keep_ppm = 0 switches the rule off: min(k, L), the Top-k rule. */
int32_t lo_ratio_budget(int32_t L, int32_t k, int32_t keep_ppm)
{
    int64_t n = k < L ? k : L;
    if (keep_ppm > 0) {
        int64_t r = ((int64_t)L * keep_ppm + 999999) / 1000000;
        if (r < 1) r = 1;
        if (r < n) n = r;
    }
    return (int32_t)n;
}

/* Eq. 2 by brute force: sort every position by (score descending, position ascending),
 * keep the first min(n, L), return them ascending by position, pad with -1 up to k >= n. */
void lo_topk_n(const double *sel, int32_t L, int32_t n, int32_t k, int32_t *idx_out)
{
    scored_pos *all = malloc((size_t)(L > 0 ? L : 1) * sizeof *all);
    for (int32_t t = 0; t < L; ++t) {
        all[t].s = sel[t];
        all[t].t = t;
    }
    qsort(all, (size_t)L, sizeof *all, by_score_desc_then_pos);
    if (n > L) n = L;
    for (int32_t j = 0; j < n; ++j) idx_out[j] = all[j].t;
    qsort(idx_out, (size_t)n, sizeof *idx_out, by_int_asc);
    for (int32_t j = n; j < k; ++j) idx_out[j] = -1;
    free(all);
}

/* How many positions the Threshold rule (rule 1: probability > param) or the Top-p rule (rule 2:
 * shortest descending prefix with probability mass >= param) keeps among L pooled logits, before
 * the clamp to [1, min(k, L)].  Probabilities are softmax(sel) over all L positions. */
int32_t lo_rule_count(const double *sel, int32_t L, int32_t rule, double param)
{
    double m = sel[0];
    for (int32_t t = 1; t < L; ++t)
        if (sel[t] > m) m = sel[t];
    double z = 0.0;
    for (int32_t t = 0; t < L; ++t) z += exp(sel[t] - m);
    if (rule == 1) {
        int32_t n = 0;
        for (int32_t t = 0; t < L; ++t)
            if (exp(sel[t] - m) / z > param) ++n;
        return n;
    }
    /* rule 2: walk down the sorted order */
    scored_pos *all = malloc((size_t)L * sizeof *all);
    for (int32_t t = 0; t < L; ++t) {
        all[t].s = sel[t];
        all[t].t = t;
    }
    qsort(all, (size_t)L, sizeof *all, by_score_desc_then_pos);
    double cum = 0.0;
    int32_t n = 0;
    while (n < L && cum < param) cum += exp(all[n++].s - m) / z;
    free(all);
    return n;
}

/* Eq. 2 with the fixed budget k. */
void lo_topk(const double *sel, int32_t L, int32_t k, int32_t *idx_out)
{
    lo_topk_n(sel, L, k, k, idx_out);
}

/*
 * One layer's attention for one decode step (Alg. 1, the per-head loop).
 *
 *   q          bf16 bits [B][Hq][d]
 *   K, V       bf16 bits, element (b, g, t, i) at  b*stride_b + g*stride_h + t*stride_t + i
 *   mask       [Hq]  1 = retrieval head (Eq. 1, 2), 0 = sparse head (Eq. 3)
 *   idx_in     [B][Hkv][k] inherited sets, valid entries first then -1; may be NULL when
 *              no head is sparse
 *   lengths    [B]
 *   out        fp64 [B][Hq][d]
 *   idx_out    [B][Hkv][k], may be NULL
 *   sel_out    fp64 [B][Hkv][max_len] pooled selection scores of groups that hold a
 *              retrieval head (other groups and t >= L_b: NaN); may be NULL
 *   keep_ppm   0: Eq. 2's fixed budget k.  > 0: the Ratio rule, lo_ratio_budget() entries
 *              per sequence, in sets of capacity k
 *   block      positions one set entry stands for (1: tokens; 64: the blocks of App. C).  The
 *              entries of idx_in / idx_out are then block numbers and k counts blocks.
 *   rule       0: the budget above.  1: Threshold, 2: Top-p (Sec. 4.4.1) with parameter
 *              rule_param (tau, p); token-granular only, without the Ratio rule
 * Returns 0, or -1 on an argument it cannot serve.
 */
int lo_decode_attn_block(int32_t B, int32_t Hq, int32_t Hkv, int32_t d, int32_t k, int32_t max_len,
                         const uint16_t *q, const uint16_t *K, const uint16_t *V, int64_t stride_b,
                         int64_t stride_h, int64_t stride_t, const uint8_t *mask,
                         const int32_t *idx_in, const int32_t *lengths, double *out,
                         int32_t *idx_out, double *sel_out, int32_t keep_ppm, int32_t block,
                         int32_t rule, double rule_param)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || d < 1 || k < 1 || block < 1) return -1;
    if (keep_ppm < 0 || keep_ppm > 1000000) return -1;
    if (rule < 0 || rule > 2 || (rule != 0 && (block != 1 || keep_ppm != 0))) return -1;
    if (rule != 0 && !(rule_param > 0.0 && rule_param <= 1.0)) return -1;
    const int32_t G = Hq / Hkv;
    int any_sparse = 0;
    for (int32_t h = 0; h < Hq; ++h)
        if (!mask[h]) any_sparse = 1;
    if (any_sparse && idx_in == NULL) return -1;
    for (int32_t b = 0; b < B; ++b)
        if (lengths[b] < 1 || lengths[b] > max_len) return -1;
    if (idx_in != NULL)
        for (int32_t b = 0; b < B; ++b)
            for (int64_t j = 0; j < (int64_t)Hkv * k; ++j)
                if ((int64_t)idx_in[(int64_t)b * Hkv * k + j] * block >= lengths[b]) return -1;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t g = 0; g < Hkv; ++g) {
            const int32_t L = lengths[b];
            const uint16_t *Kg = K + b * stride_b + g * stride_h;
            const uint16_t *Vg = V + b * stride_b + g * stride_h;
            const int32_t n_units = (L + block - 1) / block;  /* blocks of this sequence */
            double *s = malloc((size_t)L * sizeof *s);
            double *w = malloc((size_t)L * sizeof *w);
            double *sel = malloc((size_t)L * sizeof *sel);
            double *unit_score = malloc((size_t)n_units * sizeof *unit_score);
            int32_t *every = malloc((size_t)L * sizeof *every);
            int32_t *set = malloc((size_t)L * sizeof *set);
            for (int32_t t = 0; t < L; ++t) {
                every[t] = t;
                sel[t] = 0.0;
            }
            /* the inherited set of this KV head: the positions below L that the valid
             * entries of idx_in stand for (entries are distinct, so no position repeats) */
            int32_t n_set = 0;
            if (idx_in != NULL)
                for (int32_t j = 0; j < k; ++j) {
                    int32_t e = idx_in[((int64_t)b * Hkv + g) * k + j];
                    if (e < 0) continue;
                    for (int32_t t = e * block; t < (e + 1) * block && t < L && n_set < L; ++t)
                        set[n_set++] = t;
                }
            int32_t n_retrieval = 0;
            for (int32_t h = g * G; h < (g + 1) * G; ++h) {
                const uint16_t *qh = q + ((int64_t)b * Hq + h) * d;
                double *oh = out + ((int64_t)b * Hq + h) * d;
                if (mask[h]) {
                    /* retrieval head: full attention, and its logits join the pool */
                    lo_scores(qh, Kg, stride_t, L, d, s);
                    lo_softmax_weights(s, every, L, w);
                    lo_weighted_values(w, every, L, Vg, stride_t, d, oh);
                    for (int32_t t = 0; t < L; ++t) sel[t] += s[t];
                    ++n_retrieval;
                } else {
                    /* sparse head: attention restricted to the inherited set */
                    lo_scores_at(qh, Kg, stride_t, set, n_set, d, s);
                    lo_softmax_weights(s, set, n_set, w);
                    lo_weighted_values(w, set, n_set, Vg, stride_t, d, oh);
                }
            }
            if (n_retrieval > 0)
                for (int32_t t = 0; t < L; ++t) sel[t] /= (double)n_retrieval;
            if (idx_out != NULL) {
                int32_t *dst = idx_out + ((int64_t)b * Hkv + g) * k;
                if (n_retrieval > 0) {
                    /* a block is as good as its best token */
                    for (int32_t u = 0; u < n_units; ++u) {
                        double best = sel[u * block];
                        for (int32_t t = u * block + 1; t < (u + 1) * block && t < L; ++t)
                            if (sel[t] > best) best = sel[t];
                        unit_score[u] = best;
                    }
                    int32_t n_keep = lo_ratio_budget(n_units, k, keep_ppm);
                    if (rule != 0) {
                        int32_t want = lo_rule_count(sel, L, rule, rule_param);
                        if (want < 1) want = 1;
                        if (want < n_keep) n_keep = want;
                    }
                    lo_topk_n(unit_score, n_units, n_keep, k, dst);
                }
                else
                    memcpy(dst, idx_in + ((int64_t)b * Hkv + g) * k, (size_t)k * sizeof *dst);
            }
            if (sel_out != NULL) {
                double *dst = sel_out + ((int64_t)b * Hkv + g) * max_len;
                for (int32_t t = 0; t < max_len; ++t)
                    dst[t] = (n_retrieval > 0 && t < L) ? sel[t] : NAN;
            }
            free(s);
            free(w);
            free(sel);
            free(unit_score);
            free(every);
            free(set);
        }
    }
    return 0;
}

/* Token-granular sets (the method as Sec. 3.1 states it), either rule. */
int lo_decode_attn_rule(int32_t B, int32_t Hq, int32_t Hkv, int32_t d, int32_t k, int32_t max_len,
                        const uint16_t *q, const uint16_t *K, const uint16_t *V, int64_t stride_b,
                        int64_t stride_h, int64_t stride_t, const uint8_t *mask,
                        const int32_t *idx_in, const int32_t *lengths, double *out,
                        int32_t *idx_out, double *sel_out, int32_t keep_ppm)
{
    return lo_decode_attn_block(B, Hq, Hkv, d, k, max_len, q, K, V, stride_b, stride_h, stride_t, mask,
                                idx_in, lengths, out, idx_out, sel_out, keep_ppm, 1, 0, 0.0);
}

/* The same with Eq. 2's fixed budget. */
int lo_decode_attn(int32_t B, int32_t Hq, int32_t Hkv, int32_t d, int32_t k, int32_t max_len,
                   const uint16_t *q, const uint16_t *K, const uint16_t *V, int64_t stride_b,
                   int64_t stride_h, int64_t stride_t, const uint8_t *mask,
                   const int32_t *idx_in, const int32_t *lengths, double *out,
                   int32_t *idx_out, double *sel_out)
{
    return lo_decode_attn_rule(B, Hq, Hkv, d, k, max_len, q, K, V, stride_b, stride_h, stride_t, mask,
                               idx_in, lengths, out, idx_out, sel_out, 0);
}

/* Alg. 1, "C.append(k, v)": the new token's key and value rows ([B][Hkv][d] each) become row
 * lengths[b] - 1 of every KV head's cache (lengths count the token being decoded). */
int lo_append_kv(int32_t B, int32_t Hkv, int32_t d, const uint16_t *k_new, const uint16_t *v_new,
                 uint16_t *K, uint16_t *V, int64_t stride_b, int64_t stride_h, int64_t stride_t,
                 const int32_t *lengths)
{
    for (int32_t b = 0; b < B; ++b) {
        if (lengths[b] < 1) return -1;
        for (int32_t g = 0; g < Hkv; ++g) {
            const int64_t at = b * stride_b + g * stride_h + (int64_t)(lengths[b] - 1) * stride_t;
            for (int32_t i = 0; i < d; ++i) {
                K[at + i] = k_new[((int64_t)b * Hkv + g) * d + i];
                V[at + i] = v_new[((int64_t)b * Hkv + g) * d + i];
            }
        }
    }
    return 0;
}

/* Number of threads the (sequence, KV head) loop above spreads over. */
int32_t lo_num_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}
