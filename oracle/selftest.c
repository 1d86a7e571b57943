/*
 * Sanitizer self-test of the CPU oracle (test infrastructure, like the oracle itself): a standalone
 * program that drives every oracle entry point on small inputs, edge cases included, so that it can be
 * built with -fsanitize=address,undefined and run without an interpreter in between.  It checks no
 * values (the pins in tests/ do); it exists to let the sanitizers see every code path.
 * Built and run by tests/test_oracle_sanitizers.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int ajo_num_threads(void);
int ajo_logits_row(int, const void *, const void *, int, int, double *);
int ajo_greedy_rows(int, const void *, int, const void *, int, int, int32_t *, double *, double *);
double ajo_judge_logit(int, const void *, const void *, const void *, int, int, double);
double ajo_threshold_logit(double);
int ajo_walk(int, int, int, int, int, int, const void *, const void *, const int32_t *, const int32_t *, const void *,
             float, float, int32_t *, int32_t *, uint8_t *, double *, double *, uint8_t *);
int ajo_verify(int, int, int, int, int, int, int, const void *, const void *, const void *, const int32_t *,
               const void *, float, float, int32_t *, int32_t *, int32_t *, double *, double *, uint8_t *, uint8_t *,
               double *, double *, uint8_t *);
int ajo_rank_rows(int, const void *, int, const void *, int, int, const int32_t *, int32_t *, double *, int32_t *,
                  int32_t *, int32_t *, double *);
int ajo_walk_topk(int, int, int, const int32_t *, const int32_t *, int32_t *, int32_t *);
int ajo_verify_topk(int, int, int, int, int, int, const void *, const void *, const int32_t *, int32_t *, int32_t *,
                    int32_t *, double *, int32_t *, int32_t *, int32_t *);
double ajo_gumbel(uint64_t, int32_t);
int ajo_sampled_rows(int, const void *, int, const void *, int, int, double, const uint64_t *, int32_t *, double *,
                     double *);
int ajo_verify_sampled(int, int, int, int, int, int, int, const void *, const void *, const void *, const int32_t *,
                       const void *, float, float, float, const uint64_t *, int32_t *, int32_t *, int32_t *, double *,
                       double *, uint8_t *, uint8_t *, double *, double *, uint8_t *);
int ajo_walk_tree(int, int, int, int, int, int, const void *, const void *, const int32_t *, const int32_t *,
                  const int32_t *, const void *, float, float, int32_t *, int32_t *, int32_t *, uint8_t *, double *,
                  double *, uint8_t *);
int ajo_verify_tree(int, int, int, int, int, int, int, const void *, const void *, const void *, const int32_t *,
                    const int32_t *, const void *, float, float, int32_t *, int32_t *, int32_t *, int32_t *, double *,
                    double *, uint8_t *, double *, double *, uint8_t *);

static uint32_t state = 12345u;
static float rnd(void)                       /* small LCG, uniform in [-1, 1) */
{
    state = state * 1664525u + 1013904223u;
    return (float)(state >> 8) / 8388608.0f - 1.0f;
}

static void *tensor(size_t n, int dtype)     /* exactly n elements: one more read is a heap overflow */
{
    if (dtype == 0) {
        float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
        for (size_t i = 0; i < n; ++i) p[i] = rnd();
        return p;
    }
    uint16_t *p = (uint16_t *)malloc(sizeof(uint16_t) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) {
        float f = rnd();
        uint32_t u;
        __builtin_memcpy(&u, &f, 4);
        p[i] = (uint16_t)(u >> 16);
    }
    return p;
}

static int run(int B, int K, int d_t, int d_d, int V, int dtype)
{
    const int M = B * (K + 1), n = M > 0 ? M : 1, s = B * K > 0 ? B * K : 1;
    void *ht = tensor((size_t)M * d_t, dtype), *hd = tensor((size_t)M * d_d, dtype);
    void *W = tensor((size_t)V * d_t, dtype), *cw = tensor((size_t)d_t + d_d, dtype);
    int32_t *draft = (int32_t *)malloc(sizeof(int32_t) * s), *parent = (int32_t *)malloc(sizeof(int32_t) * s);
    uint64_t *key = (uint64_t *)malloc(sizeof(uint64_t) * n);
    for (int i = 0; i < B * K; ++i) {
        draft[i] = (int32_t)((rnd() + 1.0f) * 0.5f * (float)(V + 2)) - 1;      /* includes -1 and V */
        int j = i % K;
        parent[i] = j == 0 ? -1 : (int32_t)((rnd() + 1.0f) * 0.5f * (float)(j + 1)) - 1;
        if (parent[i] >= j) parent[i] = j - 1;
    }
    for (int i = 0; i < M; ++i) key[i] = ((uint64_t)state << 32) ^ (uint64_t)i * 0x9E3779B97F4A7C15ull;
    int32_t *ol = (int32_t *)malloc(sizeof(int32_t) * (B ? B : 1)), *ot = (int32_t *)malloc(sizeof(int32_t) * (B ? B : 1));
    int32_t *on = (int32_t *)malloc(sizeof(int32_t) * (B ? B : 1));
    int32_t *t = (int32_t *)malloc(sizeof(int32_t) * n), *rk = (int32_t *)malloc(sizeof(int32_t) * n);
    int32_t *lo = (int32_t *)malloc(sizeof(int32_t) * n), *hi = (int32_t *)malloc(sizeof(int32_t) * n);
    double *m1 = (double *)malloc(sizeof(double) * n), *m2 = (double *)malloc(sizeof(double) * n);
    uint8_t *nt = (uint8_t *)malloc(n), *mis = (uint8_t *)malloc(s), *nthr = (uint8_t *)malloc(s);
    double *z = (double *)malloc(sizeof(double) * s), *p = (double *)malloc(sizeof(double) * s);
    double *lg = (double *)malloc(sizeof(double) * V);
    int bad = 0;
    for (int fo = 0; fo <= 1; ++fo)
        for (int ti = 0; ti < 3; ++ti) {
            const float tau = ti == 0 ? 0.f : ti == 1 ? 0.4f : 1.f;
            bad |= ajo_verify(B, K, d_t, d_d, V, dtype, fo, ht, hd, W, draft, cw, 0.1f, tau, ol, ot, t, m1, m2, nt, mis, z, p, nthr);
            bad |= ajo_verify(B, K, d_t, d_d, V, dtype, fo, ht, hd, W, draft, cw, 0.1f, tau, ol, ot, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL);
            bad |= ajo_verify_sampled(B, K, d_t, d_d, V, dtype, fo, ht, hd, W, draft, cw, 0.f, tau, 1.5f, key, ol, ot, t, m1, m2, nt, mis, z, p, nthr);
            bad |= ajo_verify_tree(B, K, d_t, d_d, V, dtype, fo, ht, hd, W, draft, parent, cw, 0.f, tau, ol, ot, on, t, m1, m2, mis, z, p, nthr);
        }
    for (int top_k = 1; top_k <= V + 1; top_k += (V > 3 ? V / 3 : 1))
        bad |= ajo_verify_topk(B, K, d_t, V, dtype, top_k, ht, W, draft, ol, ot, t, m1, rk, lo, hi);
    if (M > 0) {
        bad |= ajo_logits_row(dtype, ht, W, V, d_t, lg);
        bad |= ajo_greedy_rows(dtype, ht, M, W, V, d_t, t, NULL, NULL);
        (void)ajo_judge_logit(dtype, ht, d_d > 0 ? hd : NULL, cw, d_t, d_d, 0.5);
    }
    /* refusals must come back as codes, without touching memory */
    if (B > 0 && K > 1) {
        parent[1] = 1;
        if (ajo_walk_tree(B, K, d_t, d_d, dtype, 1, ht, hd, t, draft, parent, cw, 0.f, 0.5f, ol, ot, on, NULL, NULL, NULL, NULL) != -1) bad |= 64;
    }
    if (ajo_verify(B, K, d_t, d_d, V, dtype, 1, ht, hd, W, draft, cw, 0.f, 1.5f, ol, ot, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == 0 && M > 0) bad |= 128;
    if (ajo_verify_topk(B, K, d_t, V, dtype, 0, ht, W, draft, ol, ot, NULL, NULL, NULL, NULL, NULL) != -1) bad |= 256;
    free(ht); free(hd); free(W); free(cw); free(draft); free(parent); free(key); free(ol); free(ot); free(on);
    free(t); free(rk); free(lo); free(hi); free(m1); free(m2); free(nt); free(mis); free(nthr); free(z); free(p); free(lg);
    return bad;
}

int main(void)
{
    int bad = 0;
    (void)ajo_num_threads();
    (void)ajo_threshold_logit(0.0);
    (void)ajo_threshold_logit(1.0);
    (void)ajo_gumbel(0xffffffffffffffffull, 2147483647);
    for (int dtype = 0; dtype <= 1; ++dtype) {
        bad |= run(3, 5, 24, 8, 37, dtype);
        bad |= run(1, 1, 8, 0, 1, dtype);        /* one token, one slot, no draft features */
        bad |= run(0, 4, 8, 8, 5, dtype);        /* empty batch */
        bad |= run(2, 9, 40, 16, 300, dtype);
    }
    if (bad) {
        printf("selftest: unexpected return code mask %d\n", bad);
        return 1;
    }
    printf("selftest ok\n");
    return 0;
}
