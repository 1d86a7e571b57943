/*
 * CPU oracle for the judge-augmented verification step of lossy speculative
 * decoding (AutoJudge, Section 3.3 "Inference"; base algorithm: Section 2,
 * "Speculative Decoding" and its footnote on greedy verification).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64,
 * scalar statement of what the GPU library must compute.  It shares no code
 * with the HIP path and must never be called from it; only the tests, the
 * smoke check and the benchmark's CPU-baseline leg may use it.
 *
 * The method is exact given its inputs, so each function below is the plain
 * definition written out:
 *
 *   step 1  logit[r][v] = sum_k hidden_t[r][k] * W_lm[v][k]        (LM head)
 *   step 2  t*[r]       = lowest v that attains max_v logit[r][v]   (greedy token)
 *   step 3  slot j of a window mismatches when t*[j] != draft_tok[j]; at a
 *           mismatch the judge computes z = clf_w . [h_t ; h_d] + clf_b on
 *           the hidden states that ENCODE the draft token of slot j, i.e.
 *           verify row j+1 (Section 3.2, design choice 1, and Appendix B
 *           "draft token embeddings"); P(important) = sigmoid(z); the
 *           mismatch is overridden (accepted) when P(important) < tau
 *           (Section 3.3: call the classifier where the base algorithm
 *           would reject, accept if deemed unimportant, keep verifying)
 *   step 4  the first slot that mismatches and is not overridden ends the
 *           window: out_len = its index (K when there is none), out_tok =
 *           t*[out_len], the target's correction token or, for out_len == K,
 *           the bonus token predicted from the last hidden state.
 *
 * Inputs are the very bytes the GPU receives (fp32, or bfloat16 bits in
 * uint16), widened exactly to fp64; all sums are fp64 in index order (the
 * compiler may split the k-sum over SIMD lanes: rounding order only).
 *
 * Readings where the paper is silent (each is restated in the design notes):
 *   - the threshold test is taken in logit space, z < log(tau/(1-tau)), with
 *     -inf / +inf at tau = 0 / 1, so that tau = 1 accepts every finite z and
 *     tau = 0 none; equal to sigmoid(z) < tau in real arithmetic;
 *   - feat_offset selects the feature row j + feat_offset (1 = encoded draft
 *     token, the paper's choice; 0 = the state that predicted the token);
 *   - clf_w holds the target part first, then the draft part;
 *   - ties of the maximum go to the lowest index, compared as IEEE values.
 *
 * Parity pins (tests/test_oracle_pins.py): every function here is pinned; see
 * that file for the list.  The top-K baseline of Section 4 (ajo_rank_rows,
 * ajo_walk_topk, ajo_verify_topk, at the end of this file) is pinned in
 * tests/test_oracle_topk_pins.py, the sampling mode of Appendix A (ajo_gumbel,
 * ajo_sampled_rows, ajo_verify_sampled) in tests/test_oracle_sampling_pins.py, draft trees
 * (ajo_walk_tree, ajo_verify_tree) in tests/test_oracle_tree_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { AJO_F32 = 0, AJO_BF16 = 1 };

#define AJO_NEAR_TIE_REL 1e-3   /* top-2 gap below this times |max| flags the row */
#define AJO_NEAR_THR_REL 1e-4   /* |z - logit(tau)| below this times max(1,|z|) flags the slot */
#define AJO_RANK_BAND_REL 1e-4  /* logits closer than this times |max| to a draft token's may count either way */

static inline double widen_at(const void *p, size_t i, int dtype)
{
    if (dtype == AJO_F32)
        return (double)((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;   /* bf16 = top half of an fp32 */
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static inline size_t elem_size(int dtype) { return dtype == AJO_F32 ? 4 : 2; }

int ajo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ step 1 */

/* dot of an fp64 vector with a stored (fp32 / bf16) vector */
static double dot_f64(const double *a, const void *b, size_t b_off, int dtype, int n)
{
    double acc = 0.0;
    if (dtype == AJO_F32) {
        const float *w = (const float *)b + b_off;
#pragma omp simd reduction(+ : acc)
        for (int k = 0; k < n; ++k)
            acc += a[k] * (double)w[k];
    } else {
        const uint16_t *w = (const uint16_t *)b + b_off;
#pragma omp simd reduction(+ : acc)
        for (int k = 0; k < n; ++k) {
            uint32_t u = (uint32_t)w[k] << 16;
            float f;
            memcpy(&f, &u, 4);
            acc += a[k] * (double)f;
        }
    }
    return acc;
}

/* LM head for ONE verify row: out[v] = sum_k h_row[k] * W_lm[v][k], v in [0,V). */
int ajo_logits_row(int dtype, const void *h_row, const void *W_lm, int V, int d_t, double *out)
{
    if (!h_row || !W_lm || !out || V <= 0 || d_t <= 0)
        return -1;
    double *h = (double *)malloc(sizeof(double) * (size_t)d_t);
    if (!h)
        return -2;
    for (int k = 0; k < d_t; ++k)
        h[k] = widen_at(h_row, (size_t)k, dtype);
    for (int v = 0; v < V; ++v)
        out[v] = dot_f64(h, W_lm, (size_t)v * (size_t)d_t, dtype, d_t);
    free(h);
    return 0;
}

/* ------------------------------------------------------------------ steps 1-2 */

/*
 * Greedy target token of each of M verify rows.
 *   t_star[r] = lowest v with logit[r][v] == max_v logit[r][v]
 *   max1[r]   = that maximum; max2[r] = largest logit over v != t_star[r]
 *               (-inf when V == 1); either may be NULL.
 * Rows are independent; threads split rows only.
 */
int ajo_greedy_rows(int dtype, const void *hidden_t, int M, const void *W_lm, int V, int d_t,
                    int32_t *t_star, double *max1, double *max2)
{
    if (!hidden_t || !W_lm || !t_star || M < 0 || V <= 0 || d_t <= 0)
        return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)d_t);
        if (!h) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < M; ++r) {
            if (!h)
                continue;
            for (int k = 0; k < d_t; ++k)
                h[k] = widen_at(hidden_t, (size_t)r * (size_t)d_t + (size_t)k, dtype);
            double best = -INFINITY, second = -INFINITY;
            int32_t arg = 0;
            for (int v = 0; v < V; ++v) {
                double l = dot_f64(h, W_lm, (size_t)v * (size_t)d_t, dtype, d_t);
                if (v == 0) {
                    best = l;
                    arg = 0;
                } else if (l > best) {      /* strict: an equal later value never wins */
                    second = best;
                    best = l;
                    arg = v;
                } else if (l > second) {
                    second = l;
                }
            }
            t_star[r] = arg;
            if (max1)
                max1[r] = best;
            if (max2)
                max2[r] = second;
        }
        free(h);
    }
    return fail ? -2 : 0;
}

/* ------------------------------------------------------------------ step 3 */

/* Judge logit z = clf_w[0:d_t] . ht_row + clf_w[d_t:d_t+d_d] . hd_row + clf_b. */
double ajo_judge_logit(int dtype, const void *ht_row, const void *hd_row, const void *clf_w,
                       int d_t, int d_d, double clf_b)
{
    double z = 0.0;
    for (int i = 0; i < d_t; ++i)
        z += widen_at(clf_w, (size_t)i, dtype) * widen_at(ht_row, (size_t)i, dtype);
    for (int i = 0; i < d_d; ++i)
        z += widen_at(clf_w, (size_t)d_t + (size_t)i, dtype) * widen_at(hd_row, (size_t)i, dtype);
    return z + clf_b;
}

/* log(tau / (1 - tau)); -inf at tau <= 0, +inf at tau >= 1. */
double ajo_threshold_logit(double tau)
{
    if (tau <= 0.0)
        return -INFINITY;
    if (tau >= 1.0)
        return INFINITY;
    return log(tau / (1.0 - tau));
}

/* ------------------------------------------------------------------ steps 3-4 */

/*
 * Walk every window given the greedy tokens t_star[B][K+1].
 * Outputs  out_len[B] in [0,K], out_tok[B].
 * Optional per-slot diagnostics [B][K] (NULL to skip), filled for EVERY slot,
 * also those after the first rejection:
 *   mismatch (0/1), z and p (NaN at matching slots), near_thr (0/1).
 */
int ajo_walk(int B, int K, int d_t, int d_d, int dtype, int feat_offset,
             const void *hidden_t, const void *hidden_d, const int32_t *t_star,
             const int32_t *draft_tok, const void *clf_w, float clf_b, float tau,
             int32_t *out_len, int32_t *out_tok,
             uint8_t *mismatch, double *z_out, double *p_out, uint8_t *near_thr)
{
    if (B < 0 || K < 1 || d_t <= 0 || d_d < 0 || (feat_offset != 0 && feat_offset != 1))
        return -1;
    if (!hidden_t || (d_d > 0 && !hidden_d) || !t_star || !draft_tok || !clf_w || !out_len || !out_tok)
        return -1;
    if (!(tau >= 0.0f && tau <= 1.0f))
        return -1;
    const double zthr = ajo_threshold_logit((double)tau);
    const size_t es = elem_size(dtype);
    for (int b = 0; b < B; ++b) {
        const int32_t *t = t_star + (size_t)b * (size_t)(K + 1);
        int n = K;
        int open = 1;                               /* still inside the accepted prefix */
        for (int j = 0; j < K; ++j) {
            size_t s = (size_t)b * (size_t)K + (size_t)j;
            int mis = (t[j] != draft_tok[s]);
            double z = NAN, p = NAN;
            int accept = 1, nthr = 0;
            if (mis) {
                size_t row = (size_t)b * (size_t)(K + 1) + (size_t)(j + feat_offset);
                const char *ht = (const char *)hidden_t + row * (size_t)d_t * es;
                const char *hd = d_d > 0 ? (const char *)hidden_d + row * (size_t)d_d * es : NULL;
                z = ajo_judge_logit(dtype, ht, hd, clf_w, d_t, d_d, (double)clf_b);
                p = 1.0 / (1.0 + exp(-z));
                accept = (z < zthr);
                if (isfinite(zthr))
                    nthr = fabs(z - zthr) < AJO_NEAR_THR_REL * fmax(1.0, fabs(z));
            }
            if (open && !accept) {                  /* first real rejection */
                n = j;
                open = 0;
            }
            if (mismatch) mismatch[s] = (uint8_t)mis;
            if (z_out) z_out[s] = z;
            if (p_out) p_out[s] = p;
            if (near_thr) near_thr[s] = (uint8_t)nthr;
        }
        out_len[b] = n;
        out_tok[b] = t[n];
    }
    return 0;
}

/* ------------------------------------------------------------------ the whole step */

/*
 * Steps 1-4 for B windows.  hidden_t [B][K+1][d_t], hidden_d [B][K+1][d_d],
 * W_lm [V][d_t], draft_tok [B][K], clf_w [d_t+d_d]; all row-major host arrays.
 * Optional per-row diagnostics [B*(K+1)]: t_star, max1, max2, near_tie; and the
 * per-slot diagnostics of ajo_walk.
 */
int ajo_verify(int B, int K, int d_t, int d_d, int V, int dtype, int feat_offset,
               const void *hidden_t, const void *hidden_d, const void *W_lm,
               const int32_t *draft_tok, const void *clf_w, float clf_b, float tau,
               int32_t *out_len, int32_t *out_tok,
               int32_t *t_star_out, double *max1_out, double *max2_out, uint8_t *near_tie,
               uint8_t *mismatch, double *z_out, double *p_out, uint8_t *near_thr)
{
    if (B < 0 || K < 1 || V <= 0)
        return -1;
    int M = B * (K + 1);
    int32_t *t = (int32_t *)calloc((size_t)(M > 0 ? M : 1), sizeof(int32_t));
    double *m1 = (double *)calloc((size_t)(M > 0 ? M : 1), sizeof(double));
    double *m2 = (double *)calloc((size_t)(M > 0 ? M : 1), sizeof(double));
    int rc = -2;
    if (t && m1 && m2) {
        rc = M > 0 ? ajo_greedy_rows(dtype, hidden_t, M, W_lm, V, d_t, t, m1, m2) : 0;
        if (rc == 0)
            rc = ajo_walk(B, K, d_t, d_d, dtype, feat_offset, hidden_t, hidden_d, t, draft_tok,
                          clf_w, clf_b, tau, out_len, out_tok, mismatch, z_out, p_out, near_thr);
        if (rc == 0) {
            for (int r = 0; r < M; ++r) {
                if (t_star_out) t_star_out[r] = t[r];
                if (max1_out) max1_out[r] = m1[r];
                if (max2_out) max2_out[r] = m2[r];
                if (near_tie) near_tie[r] = (uint8_t)((m1[r] - m2[r]) < AJO_NEAR_TIE_REL * fabs(m1[r]));
            }
        }
    }
    free(t);
    free(m1);
    free(m2);
    return rc;
}

/* ------------------------------------------------------------------ top-K baseline (Section 4) */

/*
 * The simpler lossy baseline of Section 4 ("Our baselines ..."): a mismatching draft token
 * is accepted when it is among the top_k most likely tokens of the target model.  With the
 * greedy tie rule extended to an order (larger logit first, lower index first among equals):
 *
 *   rank[r] = #{ v : logit[r][v] > logit[r][tok[r]] } + #{ v < tok[r] : logit[r][v] == logit[r][tok[r]] }
 *
 * so rank 0 is the greedy token and "within the top_k" is rank < top_k (top_k = 1 is plain
 * greedy verification, top_k = V accepts every token of the vocabulary).  A token outside
 * [0,V) is in no top-k: rank = V.
 *
 * tok[r] < 0 marks a row without a draft token (the bonus row): rank[r] = 0, nothing counted.
 * rank_lo / rank_hi (either may be NULL) bracket what an fp32-accumulating LM head may
 * count: entries that beat the token by more than band = AJO_RANK_BAND_REL * |max logit| count in
 * both, entries within the band of it only in rank_hi.  (The band is ~50 x the fp32
 * accumulation error seen at these sizes, 2e-6 |max logit|; the 1e-3 of the greedy near-tie
 * rule would span a dozen vocabulary entries for a token in the bulk of the distribution.)
 */
int ajo_rank_rows(int dtype, const void *hidden_t, int M, const void *W_lm, int V, int d_t,
                  const int32_t *tok, int32_t *t_star, double *max1, int32_t *rank,
                  int32_t *rank_lo, int32_t *rank_hi, double *tok_logit)
{
    if (!hidden_t || !W_lm || !tok || !rank || M < 0 || V <= 0 || d_t <= 0)
        return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)d_t);
        double *L = (double *)malloc(sizeof(double) * (size_t)V);
        if (!h || !L) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < M; ++r) {
            if (!h || !L)
                continue;
            for (int k = 0; k < d_t; ++k)
                h[k] = widen_at(hidden_t, (size_t)r * (size_t)d_t + (size_t)k, dtype);
            double best = -INFINITY;
            int32_t arg = 0;
            for (int v = 0; v < V; ++v) {
                L[v] = dot_f64(h, W_lm, (size_t)v * (size_t)d_t, dtype, d_t);
                if (v == 0 || L[v] > best) {
                    best = L[v];
                    arg = v;
                }
            }
            if (t_star) t_star[r] = arg;
            if (max1) max1[r] = best;
            const int32_t t = tok[r];
            int32_t rk = 0, lo = 0, hi = 0;
            double lt = NAN;
            if (t >= V) {
                rk = lo = hi = V;
            } else if (t >= 0) {
                lt = L[t];
                const double band = AJO_RANK_BAND_REL * fabs(best);
                for (int v = 0; v < V; ++v) {
                    if (v == t)
                        continue;
                    if (L[v] > lt || (L[v] == lt && v < t)) ++rk;
                    if (L[v] > lt + band) ++lo;
                    if (L[v] >= lt - band) ++hi;
                }
            }
            rank[r] = rk;
            if (rank_lo) rank_lo[r] = lo;
            if (rank_hi) rank_hi[r] = hi;
            if (tok_logit) tok_logit[r] = lt;
        }
        free(h);
        free(L);
    }
    return fail ? -2 : 0;
}

/*
 * First-reject walk of the top-K baseline given rank[B][K+1] (of the draft token of each
 * slot; the entry of row K is ignored) and the greedy tokens t_star[B][K+1]:
 * slot j is accepted when rank < top_k; out_len = first rejected slot (K if none),
 * out_tok = t_star[out_len] as in the judge-augmented walk.
 */
int ajo_walk_topk(int B, int K, int top_k, const int32_t *rank, const int32_t *t_star,
                  int32_t *out_len, int32_t *out_tok)
{
    if (B < 0 || K < 1 || top_k < 1 || !rank || !t_star || !out_len || !out_tok)
        return -1;
    for (int b = 0; b < B; ++b) {
        const int32_t *rk = rank + (size_t)b * (size_t)(K + 1);
        int n = K;
        for (int j = 0; j < K; ++j) {
            if (!(rk[j] < top_k)) {
                n = j;
                break;
            }
        }
        out_len[b] = n;
        out_tok[b] = t_star[(size_t)b * (size_t)(K + 1) + (size_t)n];
    }
    return 0;
}

/* The whole baseline step: LM head, ranks of the draft tokens, walk.  Per-row diagnostics
 * [B*(K+1)] are optional (NULL to skip). */
int ajo_verify_topk(int B, int K, int d_t, int V, int dtype, int top_k,
                    const void *hidden_t, const void *W_lm, const int32_t *draft_tok,
                    int32_t *out_len, int32_t *out_tok,
                    int32_t *t_star_out, double *max1_out, int32_t *rank_out,
                    int32_t *rank_lo_out, int32_t *rank_hi_out)
{
    if (B < 0 || K < 1 || V <= 0 || top_k < 1)
        return -1;
    const int M = B * (K + 1);
    const size_t n = (size_t)(M > 0 ? M : 1);
    int32_t *tok = (int32_t *)calloc(n, sizeof(int32_t));
    int32_t *t = (int32_t *)calloc(n, sizeof(int32_t));
    int32_t *rk = (int32_t *)calloc(n, sizeof(int32_t));
    int32_t *lo = (int32_t *)calloc(n, sizeof(int32_t));
    int32_t *hi = (int32_t *)calloc(n, sizeof(int32_t));
    double *m1 = (double *)calloc(n, sizeof(double));
    int rc = -2;
    if (tok && t && rk && lo && hi && m1) {
        for (int b = 0; b < B; ++b)
            for (int j = 0; j <= K; ++j)
                tok[(size_t)b * (K + 1) + j] = j < K ? draft_tok[(size_t)b * K + j] : -1;
        for (int r = 0; r < M; ++r)      /* a negative draft token is invalid, not "no token" */
            if (r % (K + 1) < K && tok[r] < 0) tok[r] = V;
        rc = M > 0 ? ajo_rank_rows(dtype, hidden_t, M, W_lm, V, d_t, tok, t, m1, rk, lo, hi, NULL) : 0;
        if (rc == 0)
            rc = ajo_walk_topk(B, K, top_k, rk, t, out_len, out_tok);
        if (rc == 0)
            for (int r = 0; r < M; ++r) {
                if (t_star_out) t_star_out[r] = t[r];
                if (max1_out) max1_out[r] = m1[r];
                if (rank_out) rank_out[r] = rk[r];
                if (rank_lo_out) rank_lo_out[r] = lo[r];
                if (rank_hi_out) rank_hi_out[r] = hi[r];
            }
    }
    free(tok);
    free(t);
    free(rk);
    free(lo);
    free(hi);
    free(m1);
    return rc;
}

/* ------------------------------------------------------------------ sampling mode (Appendix A) */

/*
 * Stochastic decoding as a deterministic function of a random state (Appendix A, "Generalization
 * to sampling"): the target's token of a verify row is
 *
 *     y[r] = argmax_v ( logit[r][v] / T + G(key[r], v) ),     G = standard Gumbel noise,
 *
 * which is distributed as softmax(logit[r] / T) (Gumbel-max trick) and reproducible given the
 * key - in the paper the key stands for the random state joined with the row's context; here
 * the caller supplies one 64-bit key per verify row.  Everything after the token (mismatch test,
 * judge, first-reject walk) is the greedy pipeline with y in place of the greedy token.
 *
 * The paper names no generator.  This one is counter-based so that every (row, v) can be
 * evaluated independently, and is specified by this text, which the GPU library implements
 * on its own:
 *     h = v * 0x9E3779 + lo32(key);  h ^= h >> 16;  h *= 0x85EBCA6B;  h ^= hi32(key);
 *     h ^= h >> 13;  h *= 0xC2B2AE35;  h ^= h >> 16;  h *= 0x27D4EB2F;  h ^= h >> 15;   (all mod 2^32)
 *     u = ((h >> 9) + 0.5) * 2^-23   in (0,1);      G = -log(-log(u))
 * 23 bits, so that u (an odd multiple of 2^-24 below 1) is exact in fp32 as well as in fp64; the
 * oracle takes the logarithms in fp64.
 */
static inline uint32_t ajo_noise_bits(uint64_t key, uint32_t v)
{
    uint32_t h = v * 0x9E3779u + (uint32_t)(key & 0xffffffffu);
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= (uint32_t)(key >> 32);
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    h *= 0x27D4EB2Fu;
    h ^= h >> 15;
    return h;
}

double ajo_gumbel(uint64_t key, int32_t v)
{
    const double u = ((double)(ajo_noise_bits(key, (uint32_t)v) >> 9) + 0.5) * (1.0 / 8388608.0);
    return -log(-log(u));
}

/*
 * Sampled token of each of M verify rows: y[r] = lowest v attaining the maximum of the perturbed
 * scores; max1 / max2 = largest and second-largest perturbed score (as in ajo_greedy_rows).
 */
int ajo_sampled_rows(int dtype, const void *hidden_t, int M, const void *W_lm, int V, int d_t,
                     double inv_temperature, const uint64_t *row_key,
                     int32_t *y, double *max1, double *max2)
{
    if (!hidden_t || !W_lm || !y || !row_key || M < 0 || V <= 0 || d_t <= 0 || !(inv_temperature >= 0.0))
        return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)d_t);
        if (!h) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < M; ++r) {
            if (!h)
                continue;
            for (int k = 0; k < d_t; ++k)
                h[k] = widen_at(hidden_t, (size_t)r * (size_t)d_t + (size_t)k, dtype);
            double best = -INFINITY, second = -INFINITY;
            int32_t arg = 0;
            for (int v = 0; v < V; ++v) {
                const double s = dot_f64(h, W_lm, (size_t)v * (size_t)d_t, dtype, d_t) * inv_temperature
                                 + ajo_gumbel(row_key[r], v);
                if (v == 0) {
                    best = s;
                    arg = 0;
                } else if (s > best) {
                    second = best;
                    best = s;
                    arg = v;
                } else if (s > second) {
                    second = s;
                }
            }
            y[r] = arg;
            if (max1) max1[r] = best;
            if (max2) max2[r] = second;
        }
        free(h);
    }
    return fail ? -2 : 0;
}

/* The whole step in sampling mode; arguments as ajo_verify plus the temperature and the keys. */
int ajo_verify_sampled(int B, int K, int d_t, int d_d, int V, int dtype, int feat_offset,
                       const void *hidden_t, const void *hidden_d, const void *W_lm,
                       const int32_t *draft_tok, const void *clf_w, float clf_b, float tau,
                       float inv_temperature, const uint64_t *row_key,
                       int32_t *out_len, int32_t *out_tok,
                       int32_t *y_out, double *max1_out, double *max2_out, uint8_t *near_tie,
                       uint8_t *mismatch, double *z_out, double *p_out, uint8_t *near_thr)
{
    if (B < 0 || K < 1 || V <= 0)
        return -1;
    int M = B * (K + 1);
    int32_t *t = (int32_t *)calloc((size_t)(M > 0 ? M : 1), sizeof(int32_t));
    double *m1 = (double *)calloc((size_t)(M > 0 ? M : 1), sizeof(double));
    double *m2 = (double *)calloc((size_t)(M > 0 ? M : 1), sizeof(double));
    int rc = -2;
    if (t && m1 && m2) {
        rc = M > 0 ? ajo_sampled_rows(dtype, hidden_t, M, W_lm, V, d_t, (double)inv_temperature, row_key, t, m1, m2) : 0;
        if (rc == 0)
            rc = ajo_walk(B, K, d_t, d_d, dtype, feat_offset, hidden_t, hidden_d, t, draft_tok,
                          clf_w, clf_b, tau, out_len, out_tok, mismatch, z_out, p_out, near_thr);
        if (rc == 0) {
            for (int r = 0; r < M; ++r) {
                if (y_out) y_out[r] = t[r];
                if (max1_out) max1_out[r] = m1[r];
                if (max2_out) max2_out[r] = m2[r];
                if (near_tie) near_tie[r] = (uint8_t)((m1[r] - m2[r]) < AJO_NEAR_TIE_REL * fabs(m1[r]));
            }
        }
    }
    free(t);
    free(m1);
    free(m2);
    return rc;
}

/* ------------------------------------------------------------------ tree drafts (Section 3.3, "Generality") */

/*
 * Section 3.3 ("Generality") states that the judge applies to any speculative decoding
 * algorithm with a verification stage, tree-based ones included, and gives no further detail;
 * the rule below is that section's rule (call the classifier where the base algorithm would
 * reject, accept if unimportant, keep verifying) applied edge by edge to a draft tree.
 *
 * A window is a tree of K draft nodes.  parent[j] in [-1, j) is node j's parent (-1 = the root,
 * i.e. the context; parents come before children).  Verify row 0 is the root's state and row
 * j+1 the state that has consumed node j's token, so the target's prediction that node j is
 * checked against is t_star[row(parent[j])] with row(-1) = 0, row(p) = p + 1, and the state
 * that ENCODES node j's token (the judge's features, feat_offset = 1) is row j + 1; with
 * feat_offset = 0 the features are the state that predicted the token, row(parent[j]).
 *
 *   edge_ok[j]  = (draft_tok[j] == t_star[row(parent[j])])  or  judge logit z_j < logit(tau)
 *   accepted[j] = edge_ok[j] and (parent[j] == -1 or accepted[parent[j]])
 *   out_node    = the accepted node of greatest depth, lowest index among equals (-1: none)
 *   out_len     = its depth (number of tokens on the accepted path), out_tok = t_star[row(out_node)]
 *
 * With parent[j] = j - 1 (a chain) this is ajo_walk; with tau = 0 it is plain greedy tree
 * verification.  Diagnostics as in ajo_walk, per node.  Returns -1 for a parent outside [-1, j).
 */
int ajo_walk_tree(int B, int K, int d_t, int d_d, int dtype, int feat_offset,
                  const void *hidden_t, const void *hidden_d, const int32_t *t_star,
                  const int32_t *draft_tok, const int32_t *parent, const void *clf_w, float clf_b, float tau,
                  int32_t *out_len, int32_t *out_tok, int32_t *out_node,
                  uint8_t *mismatch, double *z_out, double *p_out, uint8_t *near_thr)
{
    if (B < 0 || K < 1 || d_t <= 0 || d_d < 0 || (feat_offset != 0 && feat_offset != 1))
        return -1;
    if (!hidden_t || (d_d > 0 && !hidden_d) || !t_star || !draft_tok || !parent || !clf_w || !out_len ||
        !out_tok || !out_node)
        return -1;
    if (!(tau >= 0.0f && tau <= 1.0f))
        return -1;
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < K; ++j) {
            int32_t p = parent[(size_t)b * (size_t)K + (size_t)j];
            if (p < -1 || p >= j)
                return -1;
        }
    const double zthr = ajo_threshold_logit((double)tau);
    const size_t es = elem_size(dtype);
    int32_t *depth = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);   /* 0 = not accepted */
    if (!depth)
        return -2;
    for (int b = 0; b < B; ++b) {
        const int32_t *t = t_star + (size_t)b * (size_t)(K + 1);
        int best = -1, best_depth = 0;
        for (int j = 0; j < K; ++j) {
            size_t s = (size_t)b * (size_t)K + (size_t)j;
            int p = parent[s];
            int prow = p + 1;                                      /* row(-1) = 0, row(p) = p + 1 */
            int mis = (t[prow] != draft_tok[s]);
            double z = NAN, pr = NAN;
            int ok = 1, nthr = 0;
            if (mis) {
                size_t row = (size_t)b * (size_t)(K + 1) + (size_t)(feat_offset ? j + 1 : prow);
                const char *ht = (const char *)hidden_t + row * (size_t)d_t * es;
                const char *hd = d_d > 0 ? (const char *)hidden_d + row * (size_t)d_d * es : NULL;
                z = ajo_judge_logit(dtype, ht, hd, clf_w, d_t, d_d, (double)clf_b);
                pr = 1.0 / (1.0 + exp(-z));
                ok = (z < zthr);
                if (isfinite(zthr))
                    nthr = fabs(z - zthr) < AJO_NEAR_THR_REL * fmax(1.0, fabs(z));
            }
            int pd = p < 0 ? 0 : depth[p];                         /* depth of the parent, 0 if not accepted */
            depth[j] = (ok && (p < 0 || pd > 0)) ? pd + 1 : 0;
            if (depth[j] > best_depth) {                           /* strict: lowest index among equal depths */
                best_depth = depth[j];
                best = j;
            }
            if (mismatch) mismatch[s] = (uint8_t)mis;
            if (z_out) z_out[s] = z;
            if (p_out) p_out[s] = pr;
            if (near_thr) near_thr[s] = (uint8_t)nthr;
        }
        out_node[b] = best;
        out_len[b] = best_depth;
        out_tok[b] = t[best + 1];
    }
    free(depth);
    return 0;
}

/* The whole step on draft trees: LM head and greedy tokens of all B*(K+1) rows, then ajo_walk_tree. */
int ajo_verify_tree(int B, int K, int d_t, int d_d, int V, int dtype, int feat_offset,
                    const void *hidden_t, const void *hidden_d, const void *W_lm,
                    const int32_t *draft_tok, const int32_t *parent, const void *clf_w, float clf_b, float tau,
                    int32_t *out_len, int32_t *out_tok, int32_t *out_node,
                    int32_t *t_star_out, double *max1_out, double *max2_out,
                    uint8_t *mismatch, double *z_out, double *p_out, uint8_t *near_thr)
{
    if (B < 0 || K < 1 || V <= 0)
        return -1;
    int M = B * (K + 1);
    int32_t *t = (int32_t *)calloc((size_t)(M > 0 ? M : 1), sizeof(int32_t));
    double *m1 = (double *)calloc((size_t)(M > 0 ? M : 1), sizeof(double));
    double *m2 = (double *)calloc((size_t)(M > 0 ? M : 1), sizeof(double));
    int rc = -2;
    if (t && m1 && m2) {
        rc = M > 0 ? ajo_greedy_rows(dtype, hidden_t, M, W_lm, V, d_t, t, m1, m2) : 0;
        if (rc == 0)
            rc = ajo_walk_tree(B, K, d_t, d_d, dtype, feat_offset, hidden_t, hidden_d, t, draft_tok, parent,
                               clf_w, clf_b, tau, out_len, out_tok, out_node, mismatch, z_out, p_out, near_thr);
        if (rc == 0)
            for (int r = 0; r < M; ++r) {
                if (t_star_out) t_star_out[r] = t[r];
                if (max1_out) max1_out[r] = m1[r];
                if (max2_out) max2_out[r] = m2[r];
            }
    }
    free(t);
    free(m1);
    free(m2);
    return rc;
}
