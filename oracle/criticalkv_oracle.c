/*
 * CPU oracle for the per-layer KV-cache selection pass (test infrastructure).
 *
 * This file is NOT part of the product path.  It is a plain, slow, float64
 * implementation of what the paper defines, used only by the tests, by the
 * smoke check and by the benchmark's "cpu_baseline" leg.  It shares no code,
 * headers, tables or helpers with the HIP kernels.
 *
 * Every function takes float32 inputs (which hold the exact bf16 / fp32 values
 * the GPU consumes), up-casts them exactly and computes in double.  There is
 * no blocking, fusion or reordering beyond the loop nests the definitions give;
 * OpenMP only distributes independent (batch, head, token) iterations.
 *
 * Paper passages followed (section / equation / algorithm):
 *   - attention weights A = softmax(q K^T / sqrt(d)) ............ Section 3.1, eq. (2)
 *   - observation window: last n' queries, softmax per query row,
 *     mean over the window, 1-D max pooling ..................... Algorithm 2, lines 2-4
 *   - projected values  V W^O  and the L1 norm of each row ...... Theorem 3.3, Algorithm 1 lines 2-3
 *   - criticality  (A + eps) * ||(V W^O)_i||_1, eps = 1e-4 ...... Algorithm 1 line 3, footnote in Section 3.4
 *   - budget split b' = b*alpha, b'' = b - b', two Top-k stages .. Algorithm 1 lines 4-9
 *   - the selected entries form the compacted cache ............. Algorithm 1 line 10, Definition 3.1
 *
 * Readings taken where the paper is silent (grouped-query heads, rounding of
 * b*alpha, ties, pooling borders) are stated at each function.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define CKVO_OK 0
#define CKVO_BAD_ARG -1
#define CKVO_NO_MEM -2

int ckvo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Observation-window attention (Algorithm 2, lines 2-3; eq. (2)).
 *
 * For every batch item bi, query head h (reading keys of kv head g = h / G,
 * G = H / Hkv) and window row w:
 *     s_{w,i} = scale * sum_t q[bi,h,w,t] * k[bi,g,i,t]          i = 0..n-1
 *     p_{w,.} = softmax_i(s_{w,.})                               (all n keys, no mask)
 *     a[bi,h,i] = (1/W) sum_w p_{w,i}      or   sum_w p_{w,i}  when window_sum != 0
 *
 * causal_tail != 0 (chunked-prefill reading): the window queries are the last W tokens of the prompt,
 * window row w sits at position n - W + w and attends to keys i <= n - W + w only (the usual causal mask,
 * which only bites inside the last W keys); masked weights are exactly 0.
 *
 * q_win [b,H,W,d_h], k [b,Hkv,n,d_h], a [b,H,n]; row-major, contiguous.
 */
int ckvo_window_attention(int b, int H, int Hkv, int d_h, int n, int W,
                          double scale, int window_sum, int causal_tail,
                          const float *q_win, const float *k, double *a)
{
    if (b < 1 || H < 1 || Hkv < 1 || H % Hkv || d_h < 1 || n < 1 || W < 1 || W > n) return CKVO_BAD_ARG;
    const int G = H / Hkv;
    int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int bi = 0; bi < b; ++bi) {
        for (int h = 0; h < H; ++h) {
            const int g = h / G;
            const float *kk = k + ((size_t)bi * Hkv + g) * (size_t)n * d_h;
            double *out = a + ((size_t)bi * H + h) * (size_t)n;
            double *s = (double *)malloc(sizeof(double) * (size_t)n);
            if (!s) {
#pragma omp atomic write
                err = 1;
                continue;
            }
            for (int i = 0; i < n; ++i) out[i] = 0.0;
            for (int w = 0; w < W; ++w) {
                const float *qq = q_win + (((size_t)bi * H + h) * W + w) * (size_t)d_h;
                const int visible = causal_tail ? n - W + w + 1 : n; /* keys 0 .. visible-1 */
                double smax = -INFINITY;
                for (int i = 0; i < visible; ++i) {
                    double dot = 0.0;
                    for (int t = 0; t < d_h; ++t) dot += (double)qq[t] * (double)kk[(size_t)i * d_h + t];
                    s[i] = scale * dot;
                    if (s[i] > smax) smax = s[i];
                }
                double z = 0.0;
                for (int i = 0; i < visible; ++i) { s[i] = exp(s[i] - smax); z += s[i]; }
                for (int i = 0; i < visible; ++i) out[i] += s[i] / z;
            }
            if (!window_sum)
                for (int i = 0; i < n; ++i) out[i] /= (double)W;
            free(s);
        }
    }
    return err ? CKVO_NO_MEM : CKVO_OK;
}

/*
 * 1-D max pooling (Algorithm 2, line 4): stride 1, same length, odd kernel k,
 * window clipped at both ends:  out_i = max{ in_j : |j - i| <= k/2, 0 <= j < n }.
 * `rows` independent rows of length n.
 */
int ckvo_maxpool1d(int rows, int n, int kernel, const double *in, double *out)
{
    if (rows < 0 || n < 1 || kernel < 1 || (kernel % 2) == 0) return CKVO_BAD_ARG;
    const int r = kernel / 2;
#pragma omp parallel for schedule(static)
    for (int row = 0; row < rows; ++row) {
        const double *x = in + (size_t)row * n;
        double *y = out + (size_t)row * n;
        for (int i = 0; i < n; ++i) {
            int lo = i - r < 0 ? 0 : i - r;
            int hi = i + r > n - 1 ? n - 1 : i + r;
            double m = x[lo];
            for (int j = lo + 1; j <= hi; ++j)
                if (x[j] > m) m = x[j];
            y[i] = m;
        }
    }
    return CKVO_OK;
}

/*
 * Per-entry magnitude of the projected value (Theorem 3.3; Algorithm 1, lines 2-3).
 *
 * For query head h with kv head g = h / G, the head's slice of the output
 * projection is rows [h*d_h, (h+1)*d_h) of w_o [H*d_h, d_model]:
 *     P_{i,c}      = sum_t v[bi,g,i,t] * w_o[h*d_h + t, c]
 *     N[bi,h,i]    = sum_c |P_{i,c}|                (norm == 1, the paper's L1)
 *                  = sqrt(sum_c P_{i,c}^2)          (norm == 2)
 * Each P_{i,c} is accumulated over t in ascending order; the loop nest below
 * keeps a row of d_model accumulators so that w_o is walked along its
 * contiguous dimension, which changes no sum's order.
 */
int ckvo_projected_value_norm(int b, int H, int Hkv, int d_h, int d_model, int n, int norm,
                              const float *v, const float *w_o, double *N)
{
    if (b < 1 || H < 1 || Hkv < 1 || H % Hkv || d_h < 1 || d_model < 1 || n < 1) return CKVO_BAD_ARG;
    if (norm != 1 && norm != 2) return CKVO_BAD_ARG;
    const int G = H / Hkv;
    int err = 0;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)d_model);
        if (!p) {
#pragma omp atomic write
            err = 1;
        }
#pragma omp for collapse(3) schedule(static)
        for (int bi = 0; bi < b; ++bi) {
            for (int h = 0; h < H; ++h) {
                for (int i = 0; i < n; ++i) {
                    if (!p) continue;
                    const int g = h / G;
                    const float *vv = v + (((size_t)bi * Hkv + g) * (size_t)n + i) * d_h;
                    for (int c = 0; c < d_model; ++c) p[c] = 0.0;
                    for (int t = 0; t < d_h; ++t) {
                        const double vt = (double)vv[t];
                        const float *wrow = w_o + ((size_t)h * d_h + t) * (size_t)d_model;
                        for (int c = 0; c < d_model; ++c) p[c] += vt * (double)wrow[c];
                    }
                    double acc = 0.0;
                    if (norm == 1) {
                        for (int c = 0; c < d_model; ++c) acc += fabs(p[c]);
                    } else {
                        for (int c = 0; c < d_model; ++c) acc += p[c] * p[c];
                        acc = sqrt(acc);
                    }
                    N[((size_t)bi * H + h) * (size_t)n + i] = acc;
                }
            }
        }
        free(p);
    }
    return err ? CKVO_NO_MEM : CKVO_OK;
}

/*
 * Selection keys per kv head (Algorithm 1, line 3, applied to the pooled
 * window score that Algorithm 2 hands over).
 *
 * The paper analyses one attention head.  Reading for grouped-query heads:
 * score and magnitude are computed per query head, and the two keys a kv
 * head's entries are ranked by are the group means
 *     attn[bi,g,i] = (1/G) sum_{h in g} abar[bi,h,i]
 *     crit[bi,g,i] = (1/G) sum_{h in g} (abar[bi,h,i] + eps) * N[bi,h,i]
 * With G == 1 this is exactly the paper's A and (A + eps) * ||V W^O||_1.
 *
 */
int ckvo_group_keys(int b, int H, int Hkv, int n, double eps,
                    const double *abar, const double *N, double *attn, double *crit)
{
    if (b < 1 || H < 1 || Hkv < 1 || H % Hkv || n < 1) return CKVO_BAD_ARG;
    const int G = H / Hkv;
#pragma omp parallel for collapse(2) schedule(static)
    for (int bi = 0; bi < b; ++bi) {
        for (int g = 0; g < Hkv; ++g) {
            for (int i = 0; i < n; ++i) {
                double sa = 0.0, sc = 0.0;
                for (int j = 0; j < G; ++j) {
                    const size_t o = ((size_t)bi * H + (size_t)g * G + j) * (size_t)n + i;
                    sa += abar[o];
                    sc += (abar[o] + eps) * N[o];
                }
                attn[((size_t)bi * Hkv + g) * (size_t)n + i] = sa / (double)G;
                crit[((size_t)bi * Hkv + g) * (size_t)n + i] = sc / (double)G;
            }
        }
    }
    return CKVO_OK;
}

typedef struct { double key; int idx; } ckvo_pair;

/* descending key; equal keys: lower index first */
static int ckvo_cmp_desc(const void *pa, const void *pb)
{
    const ckvo_pair *x = (const ckvo_pair *)pa, *y = (const ckvo_pair *)pb;
    if (x->key > y->key) return -1;
    if (x->key < y->key) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

/*
 * Two-stage perturbation-constrained selection for one head (Algorithm 1, lines 4-9).
 *
 *   b'  = floor(alpha * B)      b'' = B - b'
 *   stage 1: the b' entries with the largest attn        -> taken, removed
 *   stage 2: the b'' entries with the largest crit among the remaining ones
 * Ties (the paper does not order equal keys): the lower index wins.
 *
 * protect_last = W > 0 is the workflow of the observation-window methods the paper builds on (Algorithm 2 is
 * their template): the window's own tokens, the last W entries, are kept as they are and the algorithm picks
 * the rest of the budget among the n - W entries before them.  Written as sets:
 *     P = the last min(W, B) entries                       (kept whatever their scores)
 *     R = Algorithm 1 on entries 0 .. n-W-1 alone, with budget B - |P|   (so b' = floor(alpha * (B - |P|)))
 *     S = R u P
 * The window entries never compete in either stage and use up no part of the split.
 *
 * idx[0..B) receives S in ascending index order; fixed_flag[j] (may be NULL) is 1 where idx[j] was fixed
 * before stage 2 ran, i.e. taken in stage 1 or a member of P.  tau[0], tau[1] (may be NULL) receive the
 * smallest key taken in each stage (NaN for an empty stage).
 */
int ckvo_select_head(int n, const double *attn, const double *crit, int B, double alpha, int protect_last,
                     int *idx, unsigned char *fixed_flag, double *tau)
{
    if (n < 1 || B < 0 || B > n || !(alpha >= 0.0) || !(alpha <= 1.0)) return CKVO_BAD_ARG;
    if (protect_last < 0 || protect_last > n) return CKVO_BAD_ARG;
    const int n_kept_window = protect_last < B ? protect_last : B; /* |P| */
    const int m = n - protect_last;                                 /* entries 0 .. m-1 compete */
    const int Br = B - n_kept_window;                               /* budget of Algorithm 1 */
    const int b1 = (int)floor(alpha * (double)Br);
    const int b2 = Br - b1;
    ckvo_pair *p = (ckvo_pair *)malloc(sizeof(ckvo_pair) * (size_t)n);
    unsigned char *taken = (unsigned char *)calloc((size_t)n, 1);
    if (!p || !taken) { free(p); free(taken); return CKVO_NO_MEM; }
    double t1 = NAN, t2 = NAN;

    for (int i = 0; i < m; ++i) { p[i].key = attn[i]; p[i].idx = i; }
    qsort(p, (size_t)m, sizeof(ckvo_pair), ckvo_cmp_desc);
    for (int j = 0; j < b1; ++j) taken[p[j].idx] = 1;
    if (b1 > 0) t1 = p[b1 - 1].key;

    int r = 0;
    for (int i = 0; i < m; ++i)
        if (!taken[i]) { p[r].key = crit[i]; p[r].idx = i; ++r; }
    qsort(p, (size_t)r, sizeof(ckvo_pair), ckvo_cmp_desc);
    for (int j = 0; j < b2; ++j) taken[p[j].idx] = 2;
    if (b2 > 0) t2 = p[b2 - 1].key;

    for (int i = n - n_kept_window; i < n; ++i) taken[i] = 3; /* P */

    int c = 0;
    for (int i = 0; i < n; ++i)
        if (taken[i]) {
            idx[c] = i;
            if (fixed_flag) fixed_flag[c] = (taken[i] != 2);
            ++c;
        }
    if (tau) { tau[0] = t1; tau[1] = t2; }
    free(p);
    free(taken);
    return c == B ? CKVO_OK : CKVO_BAD_ARG;
}

/*
 * Selection for all (batch, kv head) pairs.  attn, crit [b*Hkv, n]; budget [b*Hkv];
 * idx [b*Hkv, max_budget] (unused tail = -1); count [b*Hkv]; tau [b*Hkv, 2] or NULL;
 * stage1 [b*Hkv, max_budget] or NULL: 1 where idx[j] was fixed before stage 2 (stage 1 or the kept window).
 * protect_last: see ckvo_select_head.
 */
int ckvo_select(int heads, int n, const double *attn, const double *crit, const int *budget,
                double alpha, int protect_last, int max_budget, int *idx, int *count, double *tau,
                unsigned char *stage1)
{
    int err = 0;
#pragma omp parallel for schedule(dynamic)
    for (int hd = 0; hd < heads; ++hd) {
        int B = budget[hd];
        int *out = idx + (size_t)hd * max_budget;
        for (int j = 0; j < max_budget; ++j) out[j] = -1;
        if (B > max_budget) {
#pragma omp atomic write
            err = 1;
            continue;
        }
        if (stage1) memset(stage1 + (size_t)hd * max_budget, 0, (size_t)max_budget);
        int rc = ckvo_select_head(n, attn + (size_t)hd * n, crit + (size_t)hd * n, B, alpha, protect_last, out,
                                  stage1 ? stage1 + (size_t)hd * max_budget : NULL,
                                  tau ? tau + 2 * (size_t)hd : NULL);
        if (rc != CKVO_OK) {
#pragma omp atomic write
            err = 1;
        }
        count[hd] = B;
    }
    return err ? CKVO_BAD_ARG : CKVO_OK;
}

/*
 * Budget allocation across the kv heads of one batch item (Algorithm 2, line 1).
 *
 * The paper only names this step (it cites adaptive allocation methods without defining them), so this is
 * a definition written for this build, in the spirit of the adaptive scheme it cites: every head gets a
 * floor f = floor(floor_frac * total / Hkv); the remaining P = total - Hkv * f slots go to the P entries
 * with the largest pooled score `attn` among ALL Hkv * n entries of the batch item (equal scores: lower
 * head, then lower token first), and a head's budget is f plus the number of those entries it owns,
 * capped at n.  floor_frac = 1 gives the uniform split.
 */
int ckvo_allocate(int b, int Hkv, int n, const double *attn, int total, double floor_frac, int *budget)
{
    if (b < 1 || Hkv < 1 || n < 1 || total < 0 || (long long)total > (long long)Hkv * n) return CKVO_BAD_ARG;
    if (!(floor_frac >= 0.0) || !(floor_frac <= 1.0)) return CKVO_BAD_ARG;
    const int f = (int)floor(floor_frac * (double)total / (double)Hkv);
    const int P = total - Hkv * f;
    const size_t m = (size_t)Hkv * n;
    ckvo_pair *p = (ckvo_pair *)malloc(sizeof(ckvo_pair) * m);
    if (!p) return CKVO_NO_MEM;
    for (int bi = 0; bi < b; ++bi) {
        for (size_t e = 0; e < m; ++e) { p[e].key = attn[(size_t)bi * m + e]; p[e].idx = (int)e; }
        qsort(p, m, sizeof(ckvo_pair), ckvo_cmp_desc);
        for (int g = 0; g < Hkv; ++g) budget[bi * Hkv + g] = f;
        for (int j = 0; j < P; ++j) budget[bi * Hkv + p[j].idx / n] += 1;
        for (int g = 0; g < Hkv; ++g)
            if (budget[bi * Hkv + g] > n) budget[bi * Hkv + g] = n;
    }
    free(p);
    return CKVO_OK;
}

/*
 * Perturbation quantities of a given selection, per (batch item, query head)
 * (Definition 3.1; Theorems 3.2, 3.3, 3.5, 3.6; Assumption 3.4).
 *
 * For query head h (kv head g = h / G) let A = a[bi,h,:] be the head's attention distribution over the n
 * entries (here the window mean of the softmax rows, before pooling; it sums to 1), P_i = v[bi,g,i,:] W_O^h
 * the projected value of entry i, N_i = ||P_i|| (L1, or L2 with norm == 2), S the selected set
 * idx[bi,g,0..count) and S1 its stage-1 part.  Written out from the definitions, nothing shortened:
 *   sigma  = sum_{S1} A_i                     s = sum_{S} A_i
 *   C      = sum_i A_i N_i                    M = min_i N_i
 *   theta  = C - (2 - 1/s) sum_{S} A_i N_i                                     (Theorem 3.3)
 *   C'     = C - (2 - 1/sigma) sum_{S1} A_i N_i
 *   theta_hat   = C' - (2 - 1/sigma) sum_{S \ S1} A_i N_i                      (Theorem 3.5)
 *   theta_relax = C' - M (2 - 1/sigma) sum_{S \ S1} A_i                        (Theorem 3.6)
 *   L      = || sum_i (A_i - A'_i) P_i ||,   A'_i = A_i / s on S, 0 elsewhere   (Definition 3.1, Theorem 3.2)
 * Empty sets: with S empty the pruned output is zero, so L = ||sum_i A_i P_i|| and theta = C; with S1
 * empty (sigma = 0) the two stage-2 bounds say nothing and are reported as +infinity.
 * out[bi,h,:] = { sigma, s, C, theta, theta_hat, theta_relax, L, M }.
 */
int ckvo_diagnostics(int b, int H, int Hkv, int d_h, int d_model, int n, int norm, const double *a,
                     const float *v, const float *w_o, int max_budget, const int *idx, const int *count,
                     const unsigned char *stage1, double *out)
{
    if (b < 1 || H < 1 || Hkv < 1 || H % Hkv || d_h < 1 || d_model < 1 || n < 1 || max_budget < 0) return CKVO_BAD_ARG;
    if (norm != 1 && norm != 2) return CKVO_BAD_ARG;
    const int G = H / Hkv;
    int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int bi = 0; bi < b; ++bi) {
        for (int h = 0; h < H; ++h) {
            const int g = h / G;
            const size_t hd = (size_t)bi * Hkv + g;
            const double *A = a + ((size_t)bi * H + h) * (size_t)n;
            const int cnt = count[hd];
            /* masks N' (stage 1) and N'' (stage 2) of the theorems */
            unsigned char *in1 = (unsigned char *)calloc((size_t)n, 1), *in2 = (unsigned char *)calloc((size_t)n, 1);
            double *p = (double *)malloc(sizeof(double) * (size_t)d_model);
            double *o = (double *)calloc((size_t)d_model, sizeof(double));
            double *o_hat = (double *)calloc((size_t)d_model, sizeof(double));
            int bad = !in1 || !in2 || !p || !o || !o_hat || cnt < 0 || cnt > max_budget;
            for (int j = 0; !bad && j < cnt; ++j) {
                const int i = idx[hd * max_budget + j];
                if (i < 0 || i >= n) { bad = 1; break; }
                if (stage1[hd * max_budget + j]) in1[i] = 1; else in2[i] = 1;
            }
            if (bad) {
#pragma omp atomic write
                err = 1;
            } else {
                double sigma = 0.0, s2 = 0.0;
                for (int i = 0; i < n; ++i) { if (in1[i]) sigma += A[i]; if (in2[i]) s2 += A[i]; }
                const double s = sigma + s2;
                double C = 0.0, D1 = 0.0, D2 = 0.0, M = INFINITY;
                for (int i = 0; i < n; ++i) {
                    const float *vv = v + (hd * (size_t)n + i) * d_h;
                    for (int c = 0; c < d_model; ++c) p[c] = 0.0;
                    for (int t = 0; t < d_h; ++t) {
                        const double vt = (double)vv[t];
                        const float *wrow = w_o + ((size_t)h * d_h + t) * (size_t)d_model;
                        for (int c = 0; c < d_model; ++c) p[c] += vt * (double)wrow[c];
                    }
                    double N = 0.0;
                    if (norm == 1) { for (int c = 0; c < d_model; ++c) N += fabs(p[c]); }
                    else { for (int c = 0; c < d_model; ++c) N += p[c] * p[c]; N = sqrt(N); }
                    C += A[i] * N;
                    if (in1[i]) D1 += A[i] * N;
                    if (in2[i]) D2 += A[i] * N;
                    if (N < M) M = N;
                    const double A_hat = (in1[i] || in2[i]) ? A[i] / s : 0.0;
                    for (int c = 0; c < d_model; ++c) { o[c] += A[i] * p[c]; o_hat[c] += A_hat * p[c]; }
                }
                double L = 0.0;
                if (norm == 1) { for (int c = 0; c < d_model; ++c) L += fabs(o[c] - o_hat[c]); }
                else { for (int c = 0; c < d_model; ++c) L += (o[c] - o_hat[c]) * (o[c] - o_hat[c]); L = sqrt(L); }
                double *r = out + ((size_t)bi * H + h) * 8;
                r[0] = sigma; r[1] = s; r[2] = C; r[7] = M;
                r[3] = s > 0.0 ? C - (2.0 - 1.0 / s) * (D1 + D2) : C;
                if (sigma > 0.0) {
                    const double C1 = C - (2.0 - 1.0 / sigma) * D1;
                    r[4] = C1 - (2.0 - 1.0 / sigma) * D2;
                    r[5] = C1 - M * (2.0 - 1.0 / sigma) * s2;
                } else {
                    r[4] = r[5] = INFINITY;
                }
                r[6] = L;
            }
            free(in1); free(in2); free(p); free(o); free(o_hat);
        }
    }
    return err ? CKVO_BAD_ARG : CKVO_OK;
}

/*
 * Compacted cache (Algorithm 1, line 10): out[hd, j, :] = src[hd, idx[hd, j], :] for
 * j < count[hd]; later rows are left untouched.  src [heads, n, d_h] float32.
 */
int ckvo_compact(int heads, int n, int d_h, int max_budget, const float *src,
                 const int *idx, const int *count, float *out)
{
    for (int hd = 0; hd < heads; ++hd) {
        for (int j = 0; j < count[hd]; ++j) {
            const int i = idx[(size_t)hd * max_budget + j];
            if (i < 0 || i >= n) return CKVO_BAD_ARG;
            memcpy(out + ((size_t)hd * max_budget + j) * d_h, src + ((size_t)hd * n + i) * d_h,
                   sizeof(float) * (size_t)d_h);
        }
    }
    return CKVO_OK;
}
