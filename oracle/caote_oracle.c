/*
 * CAOTE oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, scalar fp64 CPU implementation of what the score / select /
 * compact path computes, written from the paper's definitions (CAOTE,
 * arXiv 2504.14051).  It exists only so that the tests, the smoke check and the
 * benchmark's cpu_baseline leg can compare the HIP kernels against something
 * that can be checked against the paper by eye.  It shares no code with the HIP
 * path, and nothing in the product path may call it.
 *
 * One call handles ONE (sequence, KV head) instance.  All arrays are row-major
 * fp64 (the callers widen the exact bf16 / fp32 input values to double).
 *
 * Notation (paper Sec. 2-3):
 *   N  tokens in the cache,  d  head dimension,  G  query heads that share this
 *   KV head,  W  window length (m in the paper's block-wise prefill),
 *   R = G*W query rows, row r = g*W + i  (g = query head in group, i = window
 *   position),  A  attention weights (R x N),  a  column sums of A,  h  base
 *   retention score,  w = h / sum(h)  (h^norm),  o = V w^T,  c  CAOTE score.
 *
 * Every function is pinned by tests/test_oracle_*.py against brute force,
 * closed forms and invariants; none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_BASE_NONE   0
#define ORACLE_BASE_H2O    1
#define ORACLE_BASE_SNAPKV 2

/* ------------------------------------------------------------------------- *
 * Attention of the window queries over the cache: Sec. 2, block-wise prefill
 * (the equation for Softmax(Q_{t+1:t+m}[K_{:t}, K_{t+1:t+m}]^T)); generation is
 * the case W = 1.  The paper omits the 1/sqrt(d) factor; `scale` multiplies
 * every logit.  If window_in_cache != 0 the last W cache rows are the window's
 * own keys and attention inside the window is causal: window position i sees
 * cache row j iff  j < N-W  or  j-(N-W) <= i.  Masked entries are exactly 0.
 *   q [G*W][d], k [N][d]  ->  A [G*W][N]
 * Returns 0, or -1 if some row has no visible key.
 * ------------------------------------------------------------------------- */
int oracle_window_attention(const double *q, const double *k, int G, int W,
                            int N, int d, double scale, int window_in_cache,
                            double *A)
{
    int R = G * W;
    int P = window_in_cache ? N - W : N; /* keys [0,P) are visible to all rows */
    if (window_in_cache && N < W) return -1;
    if (N < 1) return -1;
    for (int r = 0; r < R; ++r) {
        int i = r % W;
        int n_vis = window_in_cache ? P + i + 1 : N;
        if (n_vis < 1) return -1;
        double *Ar = A + (size_t)r * N;
        double mx = -INFINITY;
        for (int j = 0; j < n_vis; ++j) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += q[(size_t)r * d + c] * k[(size_t)j * d + c];
            s *= scale;
            Ar[j] = s;
            if (s > mx) mx = s;
        }
        double den = 0.0;
        for (int j = 0; j < n_vis; ++j) {
            Ar[j] = exp(Ar[j] - mx);
            den += Ar[j];
        }
        for (int j = 0; j < n_vis; ++j) Ar[j] /= den;
        for (int j = n_vis; j < N; ++j) Ar[j] = 0.0;
    }
    return 0;
}

/* ------------------------------------------------------------------------- *
 * The same attention slice when the caller hands over the softmax normalisers
 * of its own attention pass (App. C counts only the value-side work of the score:
 * the attention weights are taken to exist already).  row_lse[r] is the natural
 * logarithm of sum_j exp(scale * q_r.k_j) over the keys visible to row r, so
 *   A_rj = exp(scale * q_r.k_j - row_lse[r]).
 * Nothing is renormalised here: with an exact row_lse the rows sum to 1, with a
 * shifted one they do not, and that is the caller's statement, not ours.
 *   q [G*W][d], k [N][d], row_lse [G*W]  ->  A [G*W][N]
 * ------------------------------------------------------------------------- */
int oracle_window_attention_given_lse(const double *q, const double *k, int G, int W,
                                      int N, int d, double scale, int window_in_cache,
                                      const double *row_lse, double *A)
{
    int R = G * W;
    int P = window_in_cache ? N - W : N;
    if (window_in_cache && N < W) return -1;
    if (N < 1) return -1;
    for (int r = 0; r < R; ++r) {
        int i = r % W;
        int n_vis = window_in_cache ? P + i + 1 : N;
        if (n_vis < 1) return -1;
        double *Ar = A + (size_t)r * N;
        for (int j = 0; j < n_vis; ++j) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += q[(size_t)r * d + c] * k[(size_t)j * d + c];
            Ar[j] = exp(s * scale - row_lse[r]);
        }
        for (int j = n_vis; j < N; ++j) Ar[j] = 0.0;
    }
    return 0;
}

/* What such a caller would hand over: row_lse[r] = log sum_j exp(scale * q_r.k_j)
 * over the visible keys, by the definition (maximum taken out for range only).   */
int oracle_row_lse(const double *q, const double *k, int G, int W, int N, int d,
                   double scale, int window_in_cache, double *row_lse)
{
    int R = G * W;
    int P = window_in_cache ? N - W : N;
    if (window_in_cache && N < W) return -1;
    if (N < 1) return -1;
    double *s = (double *)malloc((size_t)N * sizeof(double));
    if (!s) return -2;
    for (int r = 0; r < R; ++r) {
        int i = r % W;
        int n_vis = window_in_cache ? P + i + 1 : N;
        if (n_vis < 1) { free(s); return -1; }
        double mx = -INFINITY;
        for (int j = 0; j < n_vis; ++j) {
            double t = 0.0;
            for (int c = 0; c < d; ++c) t += q[(size_t)r * d + c] * k[(size_t)j * d + c];
            s[j] = t * scale;
            if (s[j] > mx) mx = s[j];
        }
        double den = 0.0;
        for (int j = 0; j < n_vis; ++j) den += exp(s[j] - mx);
        row_lse[r] = mx + log(den);
    }
    free(s);
    return 0;
}

/* Column sums of the attention slice: the H2O score function of Sec. 2,
 * f_score,j = sum_i A_{i,j}, summed here over every query row of the group
 * (all G heads, all W positions).   A [R][N] -> a [N]                        */
void oracle_column_sums(const double *A, int R, int N, double *a)
{
    for (int j = 0; j < N; ++j) {
        double s = 0.0;
        for (int r = 0; r < R; ++r) s += A[(size_t)r * N + j];
        a[j] = s;
    }
}

/* ------------------------------------------------------------------------- *
 * Base retention score h from the column sums a (Sec. 3.2).
 *   NONE    h = a  (with W = 1, G = 1 this is TOVA's last-row score, Sec. 2)
 *   H2O     h = h_in + a : the sum of previous attention scores (Sec. 3.2,
 *           "CAOTE for H2O"; App. "H2O scores"); h is the updated accumulator.
 *           h_in may be NULL (= zeros).
 *   SNAPKV  the paper names SnapKV without defining it; the reading used here
 *           is: column sums over the window, then 1-D max pooling of odd width
 *           pool_kernel, stride 1, over the scored range [lo,hi) only, the
 *           pooling window clipped at lo and hi.  Rows outside [lo,hi) keep
 *           h = a (they are protected and never enter a score).
 * ------------------------------------------------------------------------- */
void oracle_base_score(const double *a, const double *h_in, int N, int base,
                       int pool_kernel, int lo, int hi, double *h)
{
    if (base == ORACLE_BASE_H2O) {
        for (int j = 0; j < N; ++j) h[j] = (h_in ? h_in[j] : 0.0) + a[j];
    } else if (base == ORACLE_BASE_SNAPKV) {
        int half = pool_kernel / 2;
        for (int j = 0; j < N; ++j) {
            if (j < lo || j >= hi) { h[j] = a[j]; continue; }
            int t0 = j - half < lo ? lo : j - half;
            int t1 = j + half > hi - 1 ? hi - 1 : j + half;
            double m = a[t0];
            for (int t = t0 + 1; t <= t1; ++t) if (a[t] > m) m = a[t];
            h[j] = m;
        }
    } else {
        for (int j = 0; j < N; ++j) h[j] = a[j];
    }
}

/* ------------------------------------------------------------------------- *
 * CAOTE score with a general base score: Sec. 3.2, c_j = h^norm_j /
 * (1 - h^norm_j) * || V (H^norm)^T - v_j ||_2, with h^norm = h / sum(h)
 * (the normalisation equation of "CAOTE for H2O").  The scored set is
 * [lo,hi); rows outside are protected and get +INFINITY.
 *   fast != 0 : FastCAOTE (Sec. 3.3): V (H^norm)^T is replaced by the plain
 *               mean of the scored values.
 * Conventions where the paper is silent: one scored token -> +INFINITY (the
 * only token is never evicted); sum(h) == 0 -> all weights 0 -> all scores 0.
 *   h [N], v [N][d] -> c [N]; w_out [N] and o_out [d] optional (may be NULL).
 * ------------------------------------------------------------------------- */
void oracle_caote_scores(const double *h, const double *v, int N, int d, int lo,
                         int hi, int fast, double *c, double *w_out,
                         double *o_out)
{
    double *w = (double *)calloc((size_t)(N > 0 ? N : 1), sizeof(double));
    double *o = (double *)calloc((size_t)d, sizeof(double));
    double Z = 0.0;
    int n_scored = hi - lo;
    for (int j = lo; j < hi; ++j) Z += h[j];
    for (int j = lo; j < hi; ++j) w[j] = Z > 0.0 ? h[j] / Z : 0.0;
    if (fast) {
        for (int j = lo; j < hi; ++j)
            for (int x = 0; x < d; ++x) o[x] += v[(size_t)j * d + x] / (double)n_scored;
    } else {
        for (int j = lo; j < hi; ++j)
            for (int x = 0; x < d; ++x) o[x] += w[j] * v[(size_t)j * d + x];
    }
    for (int j = 0; j < N; ++j) {
        if (j < lo || j >= hi || n_scored == 1) { c[j] = INFINITY; continue; }
        double dist2 = 0.0;
        for (int x = 0; x < d; ++x) {
            double t = o[x] - v[(size_t)j * d + x];
            dist2 += t * t;
        }
        c[j] = w[j] / (1.0 - w[j]) * sqrt(dist2);
    }
    if (w_out) memcpy(w_out, w, (size_t)N * sizeof(double));
    if (o_out) memcpy(o_out, o, (size_t)d * sizeof(double));
    free(w);
    free(o);
}

/* ------------------------------------------------------------------------- *
 * The whole scoring step for one (sequence, KV head): attention slice ->
 * column sums -> base score -> CAOTE score, in that order (Sec. 2 flow of
 * token eviction + Sec. 3.2).  h_inout: H2O accumulator in, updated h out
 * (for the other bases it only receives h; may be NULL).  a_out optional.
 * Returns 0, -1 on a row with no visible key, -2 on allocation failure.
 * ------------------------------------------------------------------------- */
int oracle_score_given_lse(const double *q, const double *k, const double *v,
                           double *h_inout, int G, int W, int N, int d, double scale,
                           int window_in_cache, int base, int pool_kernel,
                           int n_protect_head, int n_protect_tail, int fast,
                           const double *row_lse, double *c, double *a_out);

int oracle_score(const double *q, const double *k, const double *v,
                 double *h_inout, int G, int W, int N, int d, double scale,
                 int window_in_cache, int base, int pool_kernel,
                 int n_protect_head, int n_protect_tail, int fast, double *c,
                 double *a_out)
{
    return oracle_score_given_lse(q, k, v, h_inout, G, W, N, d, scale, window_in_cache, base,
                                  pool_kernel, n_protect_head, n_protect_tail, fast, NULL, c,
                                  a_out);
}

/* The same with the caller's row normalisers (row_lse != NULL), see
 * oracle_window_attention_given_lse; row_lse == NULL is oracle_score.               */
int oracle_score_given_lse(const double *q, const double *k, const double *v,
                           double *h_inout, int G, int W, int N, int d, double scale,
                           int window_in_cache, int base, int pool_kernel,
                           int n_protect_head, int n_protect_tail, int fast,
                           const double *row_lse, double *c, double *a_out)
{
    int R = G * W;
    int lo = n_protect_head, hi = N - n_protect_tail;
    if (lo > N) lo = N;
    if (hi < lo) hi = lo;
    double *A = (double *)malloc((size_t)R * N * sizeof(double));
    double *a = (double *)malloc((size_t)N * sizeof(double));
    double *h = (double *)malloc((size_t)N * sizeof(double));
    if (!A || !a || !h) { free(A); free(a); free(h); return -2; }
    int rc = row_lse ? oracle_window_attention_given_lse(q, k, G, W, N, d, scale,
                                                         window_in_cache, row_lse, A)
                     : oracle_window_attention(q, k, G, W, N, d, scale, window_in_cache, A);
    if (rc == 0) {
        oracle_column_sums(A, R, N, a);
        oracle_base_score(a, base == ORACLE_BASE_H2O ? h_inout : NULL, N, base,
                          pool_kernel, lo, hi, h);
        oracle_caote_scores(h, v, N, d, lo, hi, fast, c, NULL, NULL);
        if (h_inout) memcpy(h_inout, h, (size_t)N * sizeof(double));
        if (a_out) memcpy(a_out, a, (size_t)N * sizeof(double));
    }
    free(A); free(a); free(h);
    return rc;
}

/* ------------------------------------------------------------------------- *
 * Selection: keep the `budget` highest-scoring tokens (Sec. 2, argmax_b of
 * the score).  Ties are not treated by the paper: the lower index is kept.
 * Protected tokens carry +INFINITY and so are always kept while budget
 * allows.  Output: kept indices in ascending order.  If budget >= N all N
 * tokens are kept and idx[N..budget) = -1.  A library sort is the primitive.
 * ------------------------------------------------------------------------- */
typedef struct { double c; int j; } oracle_pair;

static int oracle_pair_cmp(const void *x, const void *y)
{
    const oracle_pair *p = (const oracle_pair *)x, *r = (const oracle_pair *)y;
    if (p->c > r->c) return -1;
    if (p->c < r->c) return 1;
    return (p->j > r->j) - (p->j < r->j);
}

static int oracle_int_cmp(const void *x, const void *y)
{
    int a = *(const int *)x, b = *(const int *)y;
    return (a > b) - (a < b);
}

void oracle_select(const double *c, int N, int budget, int32_t *idx)
{
    int n_keep = budget < N ? budget : N;
    oracle_pair *p = (oracle_pair *)malloc((size_t)(N > 0 ? N : 1) * sizeof(oracle_pair));
    for (int j = 0; j < N; ++j) { p[j].c = c[j]; p[j].j = j; }
    qsort(p, (size_t)N, sizeof(oracle_pair), oracle_pair_cmp);
    for (int i = 0; i < n_keep; ++i) idx[i] = p[i].j;
    qsort(idx, (size_t)n_keep, sizeof(int32_t), oracle_int_cmp);
    for (int i = n_keep; i < budget; ++i) idx[i] = -1;
    free(p);
}

/* ------------------------------------------------------------------------- *
 * Cache update (Sec. 2: after eviction attention uses only rows i_1..i_b).
 * Rows are opaque byte strings of row_bytes each, so K, V and the H2O
 * accumulator all go through the same routine.
 *   stable    : out row i = in row idx[i], i < n_keep  (ascending order kept)
 *   swap_last : exactly one token is evicted (n_keep = N-1); the evicted
 *               position receives the last row, everything else stays put.
 * All work in place on `rows` ([N][row_bytes]); rows beyond the new length
 * are left untouched.  Return the new length.
 * ------------------------------------------------------------------------- */
int oracle_compact_stable(unsigned char *rows, int N, size_t row_bytes,
                          const int32_t *idx, int budget)
{
    int n_keep = 0;
    while (n_keep < budget && idx[n_keep] >= 0) ++n_keep;
    unsigned char *tmp = (unsigned char *)malloc((size_t)(n_keep > 0 ? n_keep : 1) * row_bytes);
    for (int i = 0; i < n_keep; ++i)
        memcpy(tmp + (size_t)i * row_bytes, rows + (size_t)idx[i] * row_bytes, row_bytes);
    memcpy(rows, tmp, (size_t)n_keep * row_bytes);
    free(tmp);
    (void)N;
    return n_keep;
}

int oracle_compact_swap_last(unsigned char *rows, int N, size_t row_bytes,
                             const int32_t *idx, int budget)
{
    int n_keep = 0;
    while (n_keep < budget && idx[n_keep] >= 0) ++n_keep;
    if (n_keep >= N) return N;            /* nothing evicted */
    if (n_keep != N - 1) return -1;       /* not an evict-one call */
    int jstar = N - 1;                    /* the index missing from idx */
    for (int i = 0; i < n_keep; ++i) if (idx[i] != i) { jstar = i; break; }
    if (jstar != N - 1)
        memcpy(rows + (size_t)jstar * row_bytes, rows + (size_t)(N - 1) * row_bytes, row_bytes);
    return N - 1;
}

/* fill : the kept rows that already lie below the new length n_keep stay where
 * they are; the kept rows from at or beyond n_keep move, in ascending order,
 * into the positions below n_keep that evicted rows leave free, taken in
 * ascending order as well (there are as many of the one as of the other).  The
 * kept SET is what Sec. 2 fixes; the order of the rows is the caller's choice,
 * and this one moves the fewest rows.  With one evicted token it is swap_last. */
int oracle_compact_fill(unsigned char *rows, int N, size_t row_bytes,
                        const int32_t *idx, int budget)
{
    int n_keep = 0;
    while (n_keep < budget && idx[n_keep] >= 0) ++n_keep;
    if (n_keep >= N) return N;            /* nothing evicted */
    unsigned char *is_kept = (unsigned char *)calloc((size_t)N, 1);
    for (int i = 0; i < n_keep; ++i) is_kept[idx[i]] = 1;
    int src = n_keep;                     /* next kept row at or beyond n_keep */
    for (int x = 0; x < n_keep; ++x) {
        if (is_kept[x]) continue;         /* stays where it is */
        while (!is_kept[src]) ++src;
        memcpy(rows + (size_t)x * row_bytes, rows + (size_t)src * row_bytes, row_bytes);
        ++src;
    }
    free(is_kept);
    return n_keep;
}

/* ------------------------------------------------------------------------- *
 * The DEFINITION the closed form is proved equal to (Sec. 3.1, eviction
 * error): really remove token j, renormalise the remaining weights so they
 * sum to 1, recompute the weighted value sum, and measure the L2 distance to
 * the output before eviction.  w [N] must sum to 1.   -> e [N]
 * ------------------------------------------------------------------------- */
void oracle_bruteforce_eviction_error(const double *w, const double *v, int N,
                                      int d, double *e)
{
    double *o = (double *)calloc((size_t)d, sizeof(double));
    double *o2 = (double *)malloc((size_t)d * sizeof(double));
    for (int i = 0; i < N; ++i)
        for (int x = 0; x < d; ++x) o[x] += w[i] * v[(size_t)i * d + x];
    for (int j = 0; j < N; ++j) {
        double rest = 0.0;
        for (int i = 0; i < N; ++i) if (i != j) rest += w[i];
        for (int x = 0; x < d; ++x) o2[x] = 0.0;
        for (int i = 0; i < N; ++i) {
            if (i == j) continue;
            double wi = w[i] / rest;
            for (int x = 0; x < d; ++x) o2[x] += wi * v[(size_t)i * d + x];
        }
        double dist2 = 0.0;
        for (int x = 0; x < d; ++x) dist2 += (o[x] - o2[x]) * (o[x] - o2[x]);
        e[j] = sqrt(dist2);
    }
    free(o); free(o2);
}

/* The same definition taken literally for one query (generation, Sec. 3.1):
 * delete key j and value j from the cache, recompute the softmax from the
 * logits of the remaining keys, recompute the attention output, measure the
 * change.   q [d], k [N][d], v [N][d] -> e [N]                               */
void oracle_bruteforce_delete_token(const double *q, const double *k,
                                    const double *v, int N, int d, double scale,
                                    double *e)
{
    double *s = (double *)malloc((size_t)N * sizeof(double));
    double *o = (double *)malloc((size_t)d * sizeof(double));
    double *o2 = (double *)malloc((size_t)d * sizeof(double));
    for (int j = 0; j < N; ++j) {
        s[j] = 0.0;
        for (int x = 0; x < d; ++x) s[j] += q[x] * k[(size_t)j * d + x];
        s[j] *= scale;
    }
    for (int pass = -1; pass < N; ++pass) { /* pass -1: nothing deleted */
        double mx = -INFINITY, den = 0.0;
        double *dst = pass < 0 ? o : o2;
        for (int i = 0; i < N; ++i) if (i != pass && s[i] > mx) mx = s[i];
        for (int i = 0; i < N; ++i) if (i != pass) den += exp(s[i] - mx);
        for (int x = 0; x < d; ++x) dst[x] = 0.0;
        for (int i = 0; i < N; ++i) {
            if (i == pass) continue;
            double al = exp(s[i] - mx) / den;
            for (int x = 0; x < d; ++x) dst[x] += al * v[(size_t)i * d + x];
        }
        if (pass >= 0) {
            double dist2 = 0.0;
            for (int x = 0; x < d; ++x) dist2 += (o[x] - o2[x]) * (o[x] - o2[x]);
            e[pass] = sqrt(dist2);
        }
    }
    free(s); free(o); free(o2);
}

/* Joint eviction error of a token set (App. "Extending CAOTE to Multi-token
 * Eviction"): || sum_{i in S} w_i (o - v_i) ||_2 / (1 - sum_{i in S} w_i).
 * set [m] holds the token indices.  Used to pin the single-token formula
 * (m = 1 must reduce to it).                                                 */
double oracle_joint_eviction_error(const double *w, const double *v, int N,
                                   int d, const int32_t *set, int m)
{
    double *o = (double *)calloc((size_t)d, sizeof(double));
    double *acc = (double *)calloc((size_t)d, sizeof(double));
    double wsum = 0.0, n2 = 0.0;
    for (int i = 0; i < N; ++i)
        for (int x = 0; x < d; ++x) o[x] += w[i] * v[(size_t)i * d + x];
    for (int t = 0; t < m; ++t) {
        int i = set[t];
        wsum += w[i];
        for (int x = 0; x < d; ++x) acc[x] += w[i] * (o[x] - v[(size_t)i * d + x]);
    }
    for (int x = 0; x < d; ++x) n2 += acc[x] * acc[x];
    free(o); free(acc);
    return sqrt(n2) / (1.0 - wsum);
}

/* ------------------------------------------------------------------------- *
 * One step of multi-token eviction (App. "Extending CAOTE to Multi-token
 * Eviction"): with the set S = set[0..m) already evicted, the joint error of
 * evicting scored token j as well, by the appendix's m-token formula applied to
 * S + j:
 *     c_{S+j} = || sum_{i in S+j} w_i (o - v_i) ||_2 / (1 - sum_{i in S+j} w_i),
 * o = sum_i w_i v_i being the output BEFORE any eviction.  A candidate that
 * would leave no weight behind (denominator <= 0) has error +INF.
 *   w [N] sums to 1 over the scored rows [lo,hi) (entries outside are ignored),
 *   v [N][d]  ->  c [N]; NaN for rows that are not candidates (in S, or outside
 *   [lo,hi)).
 * ------------------------------------------------------------------------- */
void oracle_joint_candidates(const double *w, const double *v, int N, int d,
                             int lo, int hi, const int32_t *set, int m, double *c)
{
    double *o = (double *)calloc((size_t)d, sizeof(double));
    double *u = (double *)calloc((size_t)d, sizeof(double));
    double a = 0.0;
    for (int i = lo; i < hi; ++i)
        for (int x = 0; x < d; ++x) o[x] += w[i] * v[(size_t)i * d + x];
    for (int j = 0; j < N; ++j) c[j] = (j >= lo && j < hi) ? 0.0 : NAN;
    for (int t = 0; t < m; ++t) {
        int i = set[t];
        a += w[i];
        for (int x = 0; x < d; ++x) u[x] += w[i] * (o[x] - v[(size_t)i * d + x]);
        c[i] = NAN;
    }
    for (int j = lo; j < hi; ++j) {
        if (isnan(c[j])) continue;
        double rest = 1.0 - a - w[j], n2 = 0.0;
        for (int x = 0; x < d; ++x) {
            double y = u[x] + w[j] * (o[x] - v[(size_t)j * d + x]);
            n2 += y * y;
        }
        c[j] = rest > 0.0 ? sqrt(n2) / rest : INFINITY;
    }
    free(o); free(u);
}

/* Greedy multi-token eviction under the joint error (the appendix notes that
 * the exact choice among all token sets is combinatorial and leaves greedy
 * strategies as the way out).  Tokens leave one at a time: each step evicts the
 * candidate with the smallest joint error given what is already gone; equal
 * errors evict the higher index (the lower one is kept, as in oracle_select).
 *   m <= hi - lo evictions -> order [m]: the evicted token of each step;
 *   err [m]: the joint error of everything evicted up to and including it.
 * Returns 0, or -1 on bad arguments.                                         */
int oracle_greedy_joint_evict(const double *w, const double *v, int N, int d,
                              int lo, int hi, int m, int32_t *order, double *err)
{
    if (lo < 0 || hi > N || lo > hi || m < 0 || m > hi - lo) return -1;
    double *c = (double *)malloc((size_t)(N > 0 ? N : 1) * sizeof(double));
    for (int t = 0; t < m; ++t) {
        int best = -1;
        oracle_joint_candidates(w, v, N, d, lo, hi, order, t, c);
        for (int j = lo; j < hi; ++j) {
            if (isnan(c[j])) continue;
            if (best < 0 || c[j] < c[best] || (c[j] == c[best] && j > best)) best = j;
        }
        order[t] = best;
        err[t] = c[best];
    }
    free(c);
    return 0;
}
