/*
 * Runs every routine of the float64 oracle on small deterministic inputs, edge cases and rejected
 * arguments included.  Built with -fsanitize=address,undefined by tests/test_sanitizers_cpu.py: any
 * out-of-bounds access, use after free, leak, misaligned access or integer overflow aborts the run.
 * It checks a few invariants (counts, ascending indices) but is not a parity test.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int ckvo_num_threads(void);
int ckvo_window_attention(int, int, int, int, int, int, double, int, int, const float *, const float *, double *);
int ckvo_maxpool1d(int, int, int, const double *, double *);
int ckvo_projected_value_norm(int, int, int, int, int, int, int, const float *, const float *, double *);
int ckvo_group_keys(int, int, int, int, double, const double *, const double *, double *, double *);
int ckvo_select_head(int, const double *, const double *, int, double, int, int *, unsigned char *, double *);
int ckvo_select(int, int, const double *, const double *, const int *, double, int, int, int *, int *, double *,
                unsigned char *);
int ckvo_allocate(int, int, int, const double *, int, double, int *);
int ckvo_diagnostics(int, int, int, int, int, int, int, const double *, const float *, const float *, int, const int *,
                     const int *, const unsigned char *, double *);
int ckvo_compact(int, int, int, int, const float *, const int *, const int *, float *);

static unsigned long long state = 88172645463325252ull;
static float rnd(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (float)((double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

static int run(int b, int H, int Hkv, int dh, int dm, int n, int W, int pool, int causal, int protect, int norm)
{
    const size_t nq = (size_t)b * H * W * dh, nk = (size_t)b * Hkv * n * dh, nw = (size_t)H * dh * dm;
    float *q = malloc(nq * sizeof(float)), *k = malloc(nk * sizeof(float)), *v = malloc(nk * sizeof(float));
    float *w = malloc(nw * sizeof(float));
    double *a = malloc((size_t)b * H * n * sizeof(double)), *ab = malloc((size_t)b * H * n * sizeof(double));
    double *N = malloc((size_t)b * H * n * sizeof(double));
    double *attn = malloc((size_t)b * Hkv * n * sizeof(double)), *crit = malloc((size_t)b * Hkv * n * sizeof(double));
    for (size_t i = 0; i < nq; ++i) q[i] = rnd();
    for (size_t i = 0; i < nk; ++i) { k[i] = rnd(); v[i] = 3.0f * rnd(); }
    for (size_t i = 0; i < nw; ++i) w[i] = 0.1f * rnd();
    CHECK(ckvo_window_attention(b, H, Hkv, dh, n, W, 1.0 / sqrt((double)dh), 0, causal, q, k, a) == 0);
    CHECK(ckvo_maxpool1d(b * H, n, pool, a, ab) == 0);
    CHECK(ckvo_projected_value_norm(b, H, Hkv, dh, dm, n, norm, v, w, N) == 0);
    CHECK(ckvo_group_keys(b, H, Hkv, n, 1e-4, ab, N, attn, crit) == 0);
    const int heads = b * Hkv;
    const int budgets[] = {0, 1, n / 3, n - 1 > 0 ? n - 1 : 0, n};
    const double alphas[] = {0.0, 0.3, 0.5, 1.0};
    for (unsigned bi = 0; bi < sizeof(budgets) / sizeof(budgets[0]); ++bi)
        for (unsigned ai = 0; ai < sizeof(alphas) / sizeof(alphas[0]); ++ai) {
            const int B = budgets[bi], mb = B > 0 ? B : 1;
            int *budget = malloc(heads * sizeof(int)), *idx = malloc((size_t)heads * mb * sizeof(int));
            int *count = malloc(heads * sizeof(int));
            double *tau = malloc(2 * heads * sizeof(double));
            unsigned char *st1 = malloc((size_t)heads * mb);
            for (int h = 0; h < heads; ++h) budget[h] = B;
            CHECK(ckvo_select(heads, n, attn, crit, budget, alphas[ai], protect ? W : 0, mb, idx, count, tau, st1) == 0);
            for (int h = 0; h < heads; ++h) {
                CHECK(count[h] == B);
                for (int j = 0; j < B; ++j) {
                    CHECK(idx[(size_t)h * mb + j] >= 0 && idx[(size_t)h * mb + j] < n);
                    CHECK(j == 0 || idx[(size_t)h * mb + j] > idx[(size_t)h * mb + j - 1]);
                }
            }
            float *ko = calloc((size_t)heads * mb * dh, sizeof(float));
            CHECK(ckvo_compact(heads, n, dh, mb, k, idx, count, ko) == 0);
            double *dg = malloc((size_t)b * H * 8 * sizeof(double));
            CHECK(ckvo_diagnostics(b, H, Hkv, dh, dm, n, norm, a, v, w, mb, idx, count, st1, dg) == 0);
            free(budget); free(idx); free(count); free(tau); free(st1); free(ko); free(dg);
        }
    int *alloc = malloc(heads * sizeof(int));
    CHECK(ckvo_allocate(b, Hkv, n, attn, Hkv * n / 2, 0.25, alloc) == 0);
    CHECK(ckvo_allocate(b, Hkv, n, attn, 0, 1.0, alloc) == 0);
    CHECK(ckvo_allocate(b, Hkv, n, attn, Hkv * n, 0.0, alloc) == 0);
    free(alloc);
    free(q); free(k); free(v); free(w); free(a); free(ab); free(N); free(attn); free(crit);
    return 0;
}

int main(void)
{
    CHECK(ckvo_num_threads() >= 1);
    /* b, H, Hkv, dh, dm, n, W, pool, causal, protect, norm */
    CHECK(run(1, 4, 4, 8, 16, 37, 5, 5, 0, 0, 1) == 0);   /* small multi-head layer               */
    CHECK(run(2, 6, 2, 4, 8, 23, 4, 3, 1, 1, 2) == 0);    /* grouped heads, causal tail, kept window, L2 */
    CHECK(run(1, 2, 1, 4, 4, 1, 1, 1, 0, 0, 1) == 0);     /* a single entry                       */
    CHECK(run(1, 2, 2, 4, 4, 6, 6, 7, 1, 1, 1) == 0);     /* window = context, pool wider than n  */
    /* rejected arguments: no access may happen before the check */
    double one[4] = {1, 1, 1, 1};
    int idx[8];
    CHECK(ckvo_select_head(4, one, one, 5, 0.5, 0, idx, NULL, NULL) != 0);   /* B > n */
    CHECK(ckvo_select_head(4, one, one, 2, 1.5, 0, idx, NULL, NULL) != 0);   /* alpha out of range */
    CHECK(ckvo_select_head(4, one, one, 2, 0.5, 5, idx, NULL, NULL) != 0);   /* window > n */
    CHECK(ckvo_select_head(4, one, one, 2, 0.5, -1, idx, NULL, NULL) != 0);
    CHECK(ckvo_maxpool1d(1, 4, 4, one, one) != 0);                           /* even width */
    CHECK(ckvo_window_attention(1, 3, 2, 4, 4, 1, 1.0, 0, 0, NULL, NULL, NULL) != 0);  /* H % Hkv */
    CHECK(ckvo_window_attention(1, 2, 2, 4, 4, 5, 1.0, 0, 0, NULL, NULL, NULL) != 0);  /* W > n */
    CHECK(ckvo_projected_value_norm(1, 2, 2, 4, 4, 4, 3, NULL, NULL, NULL) != 0);      /* unknown norm */
    CHECK(ckvo_allocate(1, 2, 4, one, 9, 0.5, idx) != 0);                             /* total > Hkv * n */
    CHECK(ckvo_allocate(1, 2, 4, one, 4, 1.5, idx) != 0);
    puts("oracle sanitizer run: OK");
    return 0;
}
