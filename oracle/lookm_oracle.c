/*
 * LOOK-M prefill-time KV-cache compression: plain CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
 * what the compression path computes.  It shares no code with the HIP library and
 * must never be linked, imported or called by it; only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may use it.
 *
 * Everything follows the paper's Section 3.2 (text-prior eviction, Eq. 4-8) and
 * Section 3.3 (nearest-neighbour matching Eq. 9, averaged / pivotal / weighted
 * merging Eq. 10-12), one head at a time (the paper drops head and layer indices;
 * heads are independent).  Inputs are float32 arrays holding the exact values of
 * the caller's bf16 or fp32 tensors; every arithmetic step is IEEE binary64 in the
 * order written here (no blocking, no reassociation; build with -ffp-contract=off).
 *
 * Readings taken where the paper is silent or garbled (all listed in the design notes):
 *  - Attn(.) in Eq. 4 is the causal row softmax of Q K^T / sqrt(d), d = head_dim
 *    (the scale is the one printed in Eq. 3; row i sees columns j <= i).
 *  - the sum in Eq. 4 runs over the L prompt rows 0..L-1.
 *  - Eq. 5 is applied literally (T_p = max over all of A_s is added to text entries);
 *    Eq. 8 then takes the N = B - M highest entries of the boosted A_s[0 : L-M]
 *    with ties going to the lower position, and Eq. 6-7 append the last M rows.
 *    B is the total size S = N + M of the compressed cache.  A budget too small to
 *    hold every text token plus the recent window is rejected (return -4).
 *  - kept rows are emitted in ascending original position.
 *  - Eq. 9 uses the original, un-merged keys; every kept row (text, recent, image)
 *    is a candidate; ties go to the lower position; a zero-norm key has cosine 0.
 *  - L_sim in Eq. 10-12 is the number n of evicted tokens matched to the kept token;
 *    the sums have n terms; k^closest in Eq. 11 is the original kept key; Eq. 12 is
 *    taken literally (divisor n + 1, weights = the matching cosines).
 *  - values reuse the keys' matching and weights.
 *
 * Pins for every function live in tests/test_oracle_*.py (closed forms, brute force,
 * library softmax, invariants, the prose example of Section 3.3).
 * Parity with the authors' own (unpublished here) implementation is unpinned: the
 * paper prints no numeric worked example for this path.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_BUDGET_RANGE (-3)
#define ORACLE_ERR_BUDGET_BELOW_PROTECTED (-4)

/* ---- Eq. 4: accumulated attention scores of one head -------------------------------- */
/* q, k: [L, d] float32;  scores: [L] double, A_s[j] = sum_i A_p[i, j], the sum running over the query rows
 * i = first_row .. L-1.  Eq. 4 sums all rows (first_row = 0); an observation window of w rows - the scoring of
 * the pooling baseline the paper compares with (Section 4.2), offered as a variant - is first_row = L - w.     */
static void scores_from_row(const float *q, const float *k, int L, int d, int first_row, double *scores)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    const double root_d = sqrt((double)d);
    for (int j = 0; j < L; ++j) scores[j] = 0.0;
    for (int i = first_row; i < L; ++i) {
        /* row i of Q K^T / sqrt(d), causal: columns 0..i */
        double m = -INFINITY;
        for (int j = 0; j <= i; ++j) {
            double dot = 0.0;
            for (int c = 0; c < d; ++c)
                dot += (double)q[(size_t)i * d + c] * (double)k[(size_t)j * d + c];
            s[j] = dot / root_d;
            if (s[j] > m) m = s[j];
        }
        /* softmax over the row */
        double z = 0.0;
        for (int j = 0; j <= i; ++j) {
            s[j] = exp(s[j] - m);
            z += s[j];
        }
        /* column accumulation: A_s += A_p[i, :] */
        for (int j = 0; j <= i; ++j) scores[j] += s[j] / z;
    }
    free(s);
}

void oracle_scores_head(const float *q, const float *k, int L, int d, double *scores)
{
    scores_from_row(q, k, L, d, 0, scores);
}

/* scores of the last `window` query rows only (1 <= window <= L) */
void oracle_scores_window_head(const float *q, const float *k, int L, int d, int window, double *scores)
{
    scores_from_row(q, k, L, d, L - window, scores);
}

/* Natural-log log-sum-exp of every row of the causal scaled logits, lse[i] = log sum_{j<=i} exp(q_i.k_j/sqrt(d)):
 * the normaliser of A_p in Eq. 4 (A_p[i, j] = exp(s_ij - lse[i])), which a prefill attention kernel already holds. */
void oracle_row_lse_head(const float *q, const float *k, int L, int d, double *lse)
{
    double *t = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    const double inv_root_d = 1.0 / sqrt((double)d);
    for (int i = 0; i < L; ++i) {
        const float *qi = q + (size_t)i * d;
        double top = -INFINITY;
        for (int j = 0; j <= i; ++j) {           /* causal: keys 0..i */
            const float *kj = k + (size_t)j * d;
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += (double)qi[c] * (double)kj[c];
            t[j] = acc * inv_root_d;
            if (t[j] > top) top = t[j];
        }
        double z = 0.0;
        for (int j = 0; j <= i; ++j) z += exp(t[j] - top);
        lse[i] = top + log(z);
    }
    free(t);
}

/* ---- Eq. 5-8: text-prior selection of one head ---------------------------------------- */
typedef struct { double key; int32_t pos; } cand_t;

static int cand_cmp(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->key > y->key) return -1;   /* higher score first */
    if (x->key < y->key) return 1;
    return (x->pos > y->pos) - (x->pos < y->pos); /* tie: lower position first */
}

static int int_cmp(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* |T u R|: text positions (mask 0) united with the last M positions. */
int oracle_protected_count(const uint8_t *mask, int L, int M)
{
    int n = 0;
    for (int j = 0; j < L; ++j)
        if (mask[j] == 0 || j >= L - M) ++n;
    return n;
}

/* scores: [L] raw A_s; mask: [L], 1 = image token, 0 = text token.
 * kept: [B] ascending positions; evicted: [L - B] ascending positions.
 * rule 0: every text token must be conserved - a budget below |T u R| is refused (the reading under which
 *         "I is the union of T and the Top-N tokens" and Eq. 8 say the same thing);
 * rule 1: Eq. 5 and Eq. 8 exactly as printed, for any M <= B <= L: when the N = B - M places do not hold all
 *         text tokens, the boosted text tokens compete among themselves by score and no image token is conserved. */
int oracle_select_rule_head(const double *scores, const uint8_t *mask, int L, int B, int M, int rule,
                            int32_t *kept, int32_t *evicted)
{
    if (L <= 0 || M < 0 || rule < 0 || rule > 1) return ORACLE_ERR_ARG;
    if (M > L || B > L || B < M) return ORACLE_ERR_BUDGET_RANGE;
    if (rule == 0 && B < oracle_protected_count(mask, L, M)) return ORACLE_ERR_BUDGET_BELOW_PROTECTED;

    /* Eq. 5: A_s[T] += T_p, T_p = Max(A_s) */
    double t_p = -INFINITY;
    for (int j = 0; j < L; ++j)
        if (scores[j] > t_p) t_p = scores[j];
    const int head = L - M;             /* A_s[:-M] */
    const int N = B - M;                /* important tokens, S = N + M */
    cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)(head > 0 ? head : 1));
    for (int j = 0; j < head; ++j) {
        c[j].key = (mask[j] == 0) ? scores[j] + t_p : scores[j];
        c[j].pos = j;
    }
    /* Eq. 8: I = Top_N(A_s[:-M], N) */
    qsort(c, (size_t)head, sizeof(cand_t), cand_cmp);
    for (int r = 0; r < N; ++r) kept[r] = c[r].pos;
    /* Eq. 6-7: conserved rows = [I, last M rows]; emitted in ascending position */
    for (int r = 0; r < M; ++r) kept[N + r] = head + r;
    qsort(kept, (size_t)B, sizeof(int32_t), int_cmp);
    /* eviction set K_e = K - K_c */
    for (int r = N; r < head; ++r) evicted[r - N] = c[r].pos;
    qsort(evicted, (size_t)(L - B), sizeof(int32_t), int_cmp);
    free(c);
    return ORACLE_OK;
}

int oracle_select_head(const double *scores, const uint8_t *mask, int L, int B, int M,
                       int32_t *kept, int32_t *evicted)
{
    return oracle_select_rule_head(scores, mask, L, B, M, 0, kept, evicted);
}

/* Section 4 "Implementation Details": recent window M = alpha_1 * L, important tokens N = alpha_2 * L
 * (rounded to nearest), cache size S = N + M (Eq. 8 and the sentence after it).  Returns S, or a negative
 * code when the ratios are outside [0, 1] or their sum exceeds the prompt. */
int oracle_budget_from_ratios(int L, double alpha_recent, double alpha_important, int *M_out, int *N_out)
{
    if (L <= 0 || !(alpha_recent >= 0.0 && alpha_recent <= 1.0) || !(alpha_important >= 0.0 && alpha_important <= 1.0))
        return ORACLE_ERR_ARG;
    const int M = (int)floor(alpha_recent * (double)L + 0.5);
    const int N = (int)floor(alpha_important * (double)L + 0.5);
    if (M + N > L) return ORACLE_ERR_BUDGET_RANGE;
    *M_out = M;
    *N_out = N;
    return M + N;
}

/* ---- Eq. 9: cosine nearest kept key for every evicted key ------------------------------ */
static double dot_seq(const float *a, const float *b, int d)
{
    double acc = 0.0;
    for (int c = 0; c < d; ++c) acc += (double)a[c] * (double)b[c];
    return acc;
}

/* cosine of two rows; 0 when either norm vanishes */
static double cosine(const float *a, const float *b, int d)
{
    double na = dot_seq(a, a, d), nb = dot_seq(b, b, d);
    if (na == 0.0 || nb == 0.0) return 0.0;
    return dot_seq(a, b, d) / (sqrt(na) * sqrt(nb));
}

/* k: [L, d]; assign[e] = slot r in 0..B-1 of the closest kept row; sim[e] = that cosine. */
void oracle_nearest_head(const float *k, int d, const int32_t *kept, int B,
                         const int32_t *evicted, int Le, int32_t *assign, double *sim)
{
    for (int e = 0; e < Le; ++e) {
        const float *ki = k + (size_t)evicted[e] * d;
        int best = -1;
        double best_s = 0.0;
        for (int r = 0; r < B; ++r) {          /* kept[] ascending => first maximum = lowest position */
            double s = cosine(ki, k + (size_t)kept[r] * d, d);
            if (best < 0 || s > best_s) { best = r; best_s = s; }
        }
        assign[e] = best;
        sim[e] = best_s;
    }
}

/* ---- Eq. 10-12: merging, applied to one [L, d] tensor (K or V alike) ------------------- */
/* mode: 0 none, 1 averaged (Eq. 10), 2 pivotal (Eq. 11), 3 weighted (Eq. 12).
 * out: [B, d] double, row r = merged row of position kept[r].                            */
int oracle_merge_head(const float *x, int d, const int32_t *kept, int B,
                      const int32_t *evicted, int Le, const int32_t *assign,
                      const double *sim, int mode, double *out)
{
    if (mode < 0 || mode > 3) return ORACLE_ERR_ARG;
    for (int r = 0; r < B; ++r) {
        const float *xc = x + (size_t)kept[r] * d;
        double *o = out + (size_t)r * d;
        int n = 0;                               /* L_sim: size of this row's similarity set */
        for (int c = 0; c < d; ++c) o[c] = 0.0;  /* running sum over the set */
        if (mode != 0) {
            for (int e = 0; e < Le; ++e) {       /* evicted[] ascending */
                if (assign[e] != r) continue;
                const float *xe = x + (size_t)evicted[e] * d;
                ++n;
                for (int c = 0; c < d; ++c) {
                    if (mode == 1) o[c] += (double)xe[c];
                    else if (mode == 2) o[c] += ((double)xe[c] + (double)xc[c]);
                    else o[c] += (double)xe[c] * sim[e];
                }
            }
        }
        for (int c = 0; c < d; ++c) {
            if (n == 0) o[c] = (double)xc[c];
            else if (mode == 2) o[c] = ((double)xc[c] + 0.5 * o[c]) / (double)(n + 1);
            else o[c] = ((double)xc[c] + o[c]) / (double)(n + 1);
        }
    }
    return ORACLE_OK;
}

/* ---- whole path over H heads ------------------------------------------------------------ */
/* q, k, v: [H, L, d] float32; mask: [L]; outputs: scores [H, L], kept [H, B], evicted [H, L-B],
 * assign [H, L-B], sim [H, L-B], k_out / v_out [H, B, d] double.  Heads run in parallel
 * (OpenMP) when compiled with -fopenmp; each head's arithmetic is unchanged by that.      */
int oracle_compress_rule(const float *q, const float *k, const float *v, const uint8_t *mask,
                         int H, int L, int d, int B, int M, int mode, int rule,
                         double *scores, int32_t *kept, int32_t *evicted, int32_t *assign,
                         double *sim, double *k_out, double *v_out)
{
    if (H <= 0 || L <= 0 || d <= 0 || M < 0 || mode < 0 || mode > 3 || rule < 0 || rule > 1) return ORACLE_ERR_ARG;
    if (M > L || B > L || B < M) return ORACLE_ERR_BUDGET_RANGE;
    if (B < oracle_protected_count(mask, L, M) && rule == 0) return ORACLE_ERR_BUDGET_BELOW_PROTECTED;
    const int Le = L - B;
    int rc = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        const float *qh = q + (size_t)h * L * d, *kh = k + (size_t)h * L * d, *vh = v + (size_t)h * L * d;
        double *sc = scores + (size_t)h * L;
        int32_t *kp = kept + (size_t)h * B, *ev = evicted + (size_t)h * Le, *as = assign + (size_t)h * Le;
        double *sm = sim + (size_t)h * Le;
        oracle_scores_head(qh, kh, L, d, sc);
        int r = oracle_select_rule_head(sc, mask, L, B, M, rule, kp, ev);
        if (r == ORACLE_OK) {
            oracle_nearest_head(kh, d, kp, B, ev, Le, as, sm);
            r = oracle_merge_head(kh, d, kp, B, ev, Le, as, sm, mode, k_out + (size_t)h * B * d);
            if (r == ORACLE_OK)
                r = oracle_merge_head(vh, d, kp, B, ev, Le, as, sm, mode, v_out + (size_t)h * B * d);
        }
        if (r != ORACLE_OK) {
#pragma omp critical
            rc = r;
        }
    }
    return rc;
}

int oracle_compress(const float *q, const float *k, const float *v, const uint8_t *mask,
                    int H, int L, int d, int B, int M, int mode,
                    double *scores, int32_t *kept, int32_t *evicted, int32_t *assign,
                    double *sim, double *k_out, double *v_out)
{
    return oracle_compress_rule(q, k, v, mask, H, L, d, B, M, mode, 0, scores, kept, evicted, assign, sim, k_out, v_out);
}

/* scores only, all heads (used by tests that need just Eq. 4 at larger sizes) */
void oracle_scores(const float *q, const float *k, int H, int L, int d, double *scores)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h)
        oracle_scores_head(q + (size_t)h * L * d, k + (size_t)h * L * d, L, d, scores + (size_t)h * L);
}

/* Grouped-query attention: H query heads share kv_heads key heads, query head h reading key head h / (H / kv_heads).
 * The paper omits head indices (Section 3.1) and evaluates multi-head models; with grouped heads one cache row serves a
 * whole group, so its score is read as the SUM of Eq. 4 over the group's query heads.
 * q: [H, L, d]; k: [kv_heads, L, d]; scores: [kv_heads, L].  Returns a negative code if kv_heads does not divide H. */
int oracle_scores_grouped(const float *q, const float *k, int H, int kv_heads, int L, int d, double *scores)
{
    if (H <= 0 || kv_heads <= 0 || H % kv_heads != 0) return ORACLE_ERR_ARG;
    const int group = H / kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int kh = 0; kh < kv_heads; ++kh) {
        double *one = (double *)malloc(sizeof(double) * (size_t)L);
        double *acc = scores + (size_t)kh * L;
        for (int j = 0; j < L; ++j) acc[j] = 0.0;
        for (int m = 0; m < group; ++m) {          /* query heads kh*group .. kh*group + group - 1, in order */
            scores_from_row(q + ((size_t)kh * group + m) * L * d, k + (size_t)kh * L * d, L, d, 0, one);
            for (int j = 0; j < L; ++j) acc[j] += one[j];
        }
        free(one);
    }
    return ORACLE_OK;
}

void oracle_scores_window(const float *q, const float *k, int H, int L, int d, int window, double *scores)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h)
        oracle_scores_window_head(q + (size_t)h * L * d, k + (size_t)h * L * d, L, d, window, scores + (size_t)h * L);
}

void oracle_row_lse(const float *q, const float *k, int H, int L, int d, double *lse)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h)
        oracle_row_lse_head(q + (size_t)h * L * d, k + (size_t)h * L * d, L, d, lse + (size_t)h * L);
}

/* ---- Eq. 3: attention of one new token over a (compressed or full) cache ------------------------------ */
/* q: [d]; k, v: [S, d] float32 (the first S rows of the cache, the new token's own key and value included by the
 * caller, Eq. 2); out: [d] double = Softmax(q K^T / sqrt(d)) V.                                              */
void oracle_decode_head(const float *q, const float *k, const float *v, int S, int d, double *out)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)(S > 0 ? S : 1));
    const double root_dim = sqrt((double)d);
    double peak = -INFINITY;
    for (int r = 0; r < S; ++r) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += (double)q[c] * (double)k[(size_t)r * d + c];
        p[r] = dot / root_dim;
        if (p[r] > peak) peak = p[r];
    }
    double total = 0.0;
    for (int r = 0; r < S; ++r) {
        p[r] = exp(p[r] - peak);
        total += p[r];
    }
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    for (int r = 0; r < S; ++r)
        for (int c = 0; c < d; ++c) out[c] += (p[r] / total) * (double)v[(size_t)r * d + c];
    free(p);
}

/* q: [H, d]; k, v: [H, rows, d] of which the first S rows are attended; out: [H, d] */
void oracle_decode(const float *q, const float *k, const float *v, int H, int rows, int S, int d, double *out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h)
        oracle_decode_head(q + (size_t)h * d, k + (size_t)h * rows * d, v + (size_t)h * rows * d, S, d,
                           out + (size_t)h * d);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
