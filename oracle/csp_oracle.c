/*
 * CPU oracle for Cross-Self Pruning (CSP, arXiv 2412.04652).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, double-precision
 * implementation of what the pruning pass and the n-softmax decode step
 * compute, written from the paper's definitions so that it can be checked
 * against the paper by eye.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the product (the HIP library)
 * shares no code with it.
 *
 * Every function works on ONE sequence and ONE query head (or one selection
 * group) with dense row-major double arrays; the Python wrapper slices the
 * batch.  No blocking, no fusion: each step is the formula written out.
 *
 * Readings of the paper taken here (each is a switch or a stated choice):
 *  - Eq. "M = M^s AND M^c" is read as a union of the two top-K sets (the text
 *    of "Cross-self pruning" and of "Influence of the hyper-parameters" says
 *    the two selections are made independently and concatenated); the literal
 *    intersection is available as combine=1.
 *  - Budget: kept = selected + recent (the cache-construction equation), so
 *    K_sel = T - R; K^c = floor(cross_ratio * K_sel), K^s = K_sel - K^c
 *    (appendix table "Cross Ratio"); a side that has fewer candidates than its
 *    share hands the excess to the other side.
 *  - The observation window is the last O queries, the last R keys are always
 *    kept and are not ranked (A[-O:, :-R]); the softmax denominator still runs
 *    over every visible key, the trim happens after the softmax.
 *  - Top-K runs over the keys that the region actually covers (a key whose
 *    modality no window query shares has no intra-modality entry at all).
 *  - Ties: the lower index wins.
 *
 * Parity pins (tests/test_oracle_*.py): numpy brute force with the four
 * explicit blocks A^st, A^sv, A^ct, A^cv; softmax rows sum to 1; the n-softmax
 * closed forms (virtual zero key, shift law, the special n that undoes the
 * sharpness shift); Q = 0 closed form; planted keys; count, nesting and
 * identity invariants.  No function here is "parity unpinned" with respect to
 * the formulas; which of the readings above the authors' own code takes is
 * unpinned (their code is not available).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------
 * Attention weights of the observation window and their per-key sums.
 * Softmax / n-softmax: Eq. "A = softmax(O), O = QK^T/sqrt(d)" and Eq.
 * "n-softmax"; cross/self split: Eq. "cross-self"; window and recent trim:
 * "A[-O:, :-R]" in "Cross-self pruning"; Algorithm 1, steps "A <- n-Softmax(O)"
 * to "A^s, A^c <- ...".
 *
 *   q        [O][D]  queries of positions L-O .. L-1
 *   k        [L][D]  all cached keys
 *   mod      [L]     0 = text, 1 = visual
 *   a_self, a_cross [L]  ACCUMULATED INTO (+=): entry j < L-R receives the
 *            sum over window rows i of A_ij, split by whether query i and
 *            key j have the same modality (self) or not (cross).  Entries
 *            j >= L-R are left untouched.  Calling this once per head of a
 *            selection group with the same outputs sums over the group.
 *   row_sum  [O] or NULL: sum_j A_ij over all visible keys (for the pins).
 * ---------------------------------------------------------------------- */
void csp_oracle_head_scores(const double* q, const double* k, const uint8_t* mod,
                            int L, int O, int R, int D, double n_score, int causal,
                            double* a_self, double* a_cross, double* row_sum)
{
    double* s = (double*)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    for (int i = 0; i < O; ++i) {
        const int p = L - O + i;                 /* absolute position of query i */
        const int n_vis = causal ? p + 1 : L;    /* keys j <= p are visible */
        double m = -INFINITY;
        for (int j = 0; j < n_vis; ++j) {
            double dot = 0.0;
            for (int d = 0; d < D; ++d) dot += q[(size_t)i * D + d] * k[(size_t)j * D + d];
            s[j] = dot * inv_sqrt_d;
            if (s[j] > m) m = s[j];
        }
        /* e^{s_j} / (n + sum e^{s_j'}) evaluated with both sides scaled by e^{-m} */
        double denom = n_score * exp(-m);
        for (int j = 0; j < n_vis; ++j) denom += exp(s[j] - m);
        double rs = 0.0;
        for (int j = 0; j < n_vis; ++j) {
            const double a = exp(s[j] - m) / denom;
            rs += a;
            if (j < L - R) {
                if (mod[j] == mod[p]) a_self[j] += a;
                else                  a_cross[j] += a;
            }
        }
        if (row_sum) row_sum[i] = rs;
    }
    free(s);
}

/* ------------------------------------------------------------------------
 * Budget rule.  T is the maximum cache length ("Preliminary"); the cache is
 * the selected keys followed by the last R ("K = (K.M) (+) K[-R:]").
 * n_s, n_c: number of candidate keys of the self / cross region.
 * Returns 0, or -1 if T < R.
 * ---------------------------------------------------------------------- */
int csp_oracle_budget(int T, int R, double cross_ratio, int n_s, int n_c, int* K_s, int* K_c)
{
    if (T < R) return -1;
    const int K_sel = T - R;
    int kc = (int)floor(cross_ratio * (double)K_sel);
    if (kc > K_sel) kc = K_sel;
    if (kc < 0) kc = 0;
    int ks = K_sel - kc;
    if (ks > n_s) { kc += ks - n_s; ks = n_s; }
    if (kc > n_c) { ks += kc - n_c; kc = n_c; }
    if (ks > n_s) ks = n_s;
    *K_s = ks;
    *K_c = kc;
    return 0;
}

typedef struct { double score; int idx; } csp_oracle_item;

static int cmp_desc_score_then_idx(const void* a, const void* b)
{
    const csp_oracle_item* x = (const csp_oracle_item*)a;
    const csp_oracle_item* y = (const csp_oracle_item*)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

/* mark[j] = 1 for the K candidates with the largest score (ties: lower index) */
static void topk_mark(const double* score, const uint8_t* cand, int n, int K, uint8_t* mark)
{
    csp_oracle_item* it = (csp_oracle_item*)malloc(sizeof(csp_oracle_item) * (size_t)(n > 0 ? n : 1));
    int c = 0;
    for (int j = 0; j < n; ++j)
        if (cand[j]) { it[c].score = score[j]; it[c].idx = j; ++c; }
    qsort(it, (size_t)c, sizeof(csp_oracle_item), cmp_desc_score_then_idx);
    memset(mark, 0, (size_t)n);
    for (int t = 0; t < K && t < c; ++t) mark[it[t].idx] = 1;
    free(it);
}

/* ------------------------------------------------------------------------
 * Selection: Eq. "top-K" masks per region, their combination, and the recent
 * keys (Algorithm 1, steps "M^s <- Topk(A^s), M^c <- Topk(A^c)" to the
 * concatenation with K[-R:]).  Early-out of Algorithm 1: a cache that already
 * fits the budget is returned unchanged.
 *
 *   a_self, a_cross [L]  scores (entries >= L-R ignored)
 *   mod [L]
 *   combine: 0 = union (default reading), 1 = literal intersection
 *   idx_out [min(T,L)]   kept positions, ascending
 *   counts  [4]          {kept, K^s, K^c, number of keys in both masks}
 * Returns the number of kept keys, or -1 on invalid arguments.
 * ---------------------------------------------------------------------- */
int csp_oracle_select(const double* a_self, const double* a_cross, const uint8_t* mod,
                      int L, int O, int R, int T, double cross_ratio, int combine,
                      int32_t* idx_out, int32_t* counts)
{
    if (O > L || R > L || O < 0 || R < 0 || T < 0) return -1;
    if (L <= T) {                               /* identity */
        for (int j = 0; j < L; ++j) idx_out[j] = j;
        if (counts) { counts[0] = L; counts[1] = 0; counts[2] = 0; counts[3] = 0; }
        return L;
    }
    if (T < R) return -1;
    const int P = L - R;                        /* prefix = rankable keys */
    int has_q[2] = {0, 0};
    for (int i = L - O; i < L; ++i) has_q[mod[i] ? 1 : 0] = 1;
    uint8_t* cand_s = (uint8_t*)calloc((size_t)P + 1, 1);
    uint8_t* cand_c = (uint8_t*)calloc((size_t)P + 1, 1);
    uint8_t* m_s = (uint8_t*)calloc((size_t)P + 1, 1);
    uint8_t* m_c = (uint8_t*)calloc((size_t)P + 1, 1);
    int n_s = 0, n_c = 0;
    for (int j = 0; j < P; ++j) {
        const int mj = mod[j] ? 1 : 0;
        cand_s[j] = (uint8_t)has_q[mj];         /* some window query shares j's modality */
        cand_c[j] = (uint8_t)has_q[1 - mj];     /* some window query has the other one */
        n_s += cand_s[j];
        n_c += cand_c[j];
    }
    int K_s = 0, K_c = 0;
    csp_oracle_budget(T, R, cross_ratio, n_s, n_c, &K_s, &K_c);
    topk_mark(a_self, cand_s, P, K_s, m_s);
    topk_mark(a_cross, cand_c, P, K_c, m_c);
    int kept = 0, both = 0;
    for (int j = 0; j < P; ++j) {
        const int in = combine == 0 ? (m_s[j] | m_c[j]) : (m_s[j] & m_c[j]);
        both += (m_s[j] & m_c[j]);
        if (in) idx_out[kept++] = j;
    }
    for (int j = P; j < L; ++j) idx_out[kept++] = j;
    if (counts) { counts[0] = kept; counts[1] = K_s; counts[2] = K_c; counts[3] = both; }
    free(cand_s); free(cand_c); free(m_s); free(m_c);
    return kept;
}

/* ------------------------------------------------------------------------
 * Cache construction, Eq. "K = (K.M) (+) K[-R:]": a bit copy of the kept rows.
 * ---------------------------------------------------------------------- */
void csp_oracle_gather(const void* src, size_t row_bytes, const int32_t* idx, int n, void* dst)
{
    for (int t = 0; t < n; ++t)
        memcpy((char*)dst + (size_t)t * row_bytes, (const char*)src + (size_t)idx[t] * row_bytes, row_bytes);
}

/* ------------------------------------------------------------------------
 * One decode step over a cache of T keys with the n-softmax of Eq.
 * "n-softmax": p_t = e^{s_t} / (n + sum_u e^{s_u}), out = sum_t p_t v_t.
 * No causal mask: the query is the newest token.
 *   q [D], kc, vc [T][D], out [D], p_out [T] or NULL.
 * ---------------------------------------------------------------------- */
void csp_oracle_decode(const double* q, const double* kc, const double* vc, int T, int D,
                       double n, double* out, double* p_out)
{
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    double* s = (double*)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
    double m = -INFINITY;
    for (int t = 0; t < T; ++t) {
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += q[d] * kc[(size_t)t * D + d];
        s[t] = dot * inv_sqrt_d;
        if (s[t] > m) m = s[t];
    }
    for (int d = 0; d < D; ++d) out[d] = 0.0;
    if (T == 0) { free(s); return; }            /* n + empty sum: every weight is 0 */
    double denom = n * exp(-m);
    for (int t = 0; t < T; ++t) denom += exp(s[t] - m);
    for (int t = 0; t < T; ++t) {
        const double p = exp(s[t] - m) / denom;
        if (p_out) p_out[t] = p;
        for (int d = 0; d < D; ++d) out[d] += p * vc[(size_t)t * D + d];
    }
    free(s);
}

/* ------------------------------------------------------------------------
 * Batch drivers: the same per-head functions in a loop over independent
 * problems (OpenMP over problems only; used for the timed CPU baseline and to
 * keep the Python wrapper out of the inner loops).
 *
 * Scores of n_prob independent (sequence, head) problems that share L, O, R,
 * D.  q: [n_prob][O][D], k: [n_prob][L][D], mod: [n_prob][L],
 * a_self/a_cross: [n_prob][L] (accumulated into).
 * ---------------------------------------------------------------------- */
void csp_oracle_scores_batch(const double* q, const double* k, const uint8_t* mod, int n_prob,
                             int L, int O, int R, int D, double n_score, int causal,
                             double* a_self, double* a_cross)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int p = 0; p < n_prob; ++p)
        csp_oracle_head_scores(q + (size_t)p * O * D, k + (size_t)p * L * D, mod + (size_t)p * L,
                               L, O, R, D, n_score, causal,
                               a_self + (size_t)p * L, a_cross + (size_t)p * L, NULL);
}

void csp_oracle_decode_batch(const double* q, const double* kc, const double* vc, int n_prob,
                             int T, int D, double n, double* out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int p = 0; p < n_prob; ++p)
        csp_oracle_decode(q + (size_t)p * D, kc + (size_t)p * T * D, vc + (size_t)p * T * D,
                          T, D, n, out + (size_t)p * D, NULL);
}

int csp_oracle_max_threads(void);
#ifdef _OPENMP
#include <omp.h>
int csp_oracle_max_threads(void) { return omp_get_max_threads(); }
void csp_oracle_set_threads(int n) { omp_set_num_threads(n); }
#else
int csp_oracle_max_threads(void) { return 1; }
void csp_oracle_set_threads(int n) { (void)n; }
#endif
