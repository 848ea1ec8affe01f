/*
 * Runs every function of the CPU oracle once under AddressSanitizer and
 * UndefinedBehaviorSanitizer.  Built by tests/test_oracle_sanitized.py from this
 * file plus oracle/csp_oracle.c (host compiler only), as an executable of its
 * own so that the sanitizer runtime never enters the test process.
 *
 * Input file (little endian): int32 L, O, R, D, T, causal, n_prob;
 * double n_score, n_decode, cross_ratio; then per problem q[O*D], k[L*D],
 * v[L*D] as doubles and mod[L] as bytes.  Output file: per problem
 * a_self[L], a_cross[L], row_sum[O] (doubles), int32 kept, int32 cnt[4],
 * int32 idx[L], double out[D]; then the batch drivers' a_self / a_cross
 * [n_prob*L] and decode outputs [n_prob*D].
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void csp_oracle_head_scores(const double*, const double*, const uint8_t*, int, int, int, int, double, int, double*,
                            double*, double*);
int csp_oracle_select(const double*, const double*, const uint8_t*, int, int, int, int, double, int, int32_t*, int32_t*);
void csp_oracle_gather(const void*, size_t, const int32_t*, int, void*);
void csp_oracle_decode(const double*, const double*, const double*, int, int, double, double*, double*);
void csp_oracle_scores_batch(const double*, const double*, const uint8_t*, int, int, int, int, int, double, int, double*,
                             double*);
void csp_oracle_decode_batch(const double*, const double*, const double*, int, int, int, double, double*);

static void rd(void* p, size_t n, FILE* f) { if (fread(p, 1, n, f) != n) { fprintf(stderr, "short read\n"); exit(2); } }
static void wr(const void* p, size_t n, FILE* f) { if (fwrite(p, 1, n, f) != n) { fprintf(stderr, "short write\n"); exit(2); } }

int main(int argc, char** argv) {
    if (argc != 3) return 2;
    FILE* in = fopen(argv[1], "rb");
    FILE* out = fopen(argv[2], "wb");
    if (!in || !out) return 2;
    int32_t h[7];
    double f[3];
    rd(h, sizeof h, in);
    rd(f, sizeof f, in);
    const int L = h[0], O = h[1], R = h[2], D = h[3], T = h[4], causal = h[5], P = h[6];
    /* exact-size heap blocks: any access past an end is an ASan report */
    double* q = malloc(sizeof(double) * P * O * D);
    double* k = malloc(sizeof(double) * P * L * D);
    double* v = malloc(sizeof(double) * P * L * D);
    uint8_t* mod = malloc((size_t)P * L);
    for (int p = 0; p < P; ++p) {
        rd(q + (size_t)p * O * D, sizeof(double) * O * D, in);
        rd(k + (size_t)p * L * D, sizeof(double) * L * D, in);
        rd(v + (size_t)p * L * D, sizeof(double) * L * D, in);
        rd(mod + (size_t)p * L, L, in);
    }
    const int cap = T < L ? T : L;
    double* kc_all = calloc((size_t)P * cap * D, sizeof(double));
    double* vc_all = calloc((size_t)P * cap * D, sizeof(double));
    for (int p = 0; p < P; ++p) {
        double* a_s = calloc(L, sizeof(double));
        double* a_c = calloc(L, sizeof(double));
        double* rs = calloc(O, sizeof(double));
        csp_oracle_head_scores(q + (size_t)p * O * D, k + (size_t)p * L * D, mod + (size_t)p * L, L, O, R, D, f[0], causal,
                               a_s, a_c, rs);
        int32_t* idx = malloc(sizeof(int32_t) * L);
        for (int j = 0; j < L; ++j) idx[j] = -1;
        int32_t cnt[4] = {0, 0, 0, 0};
        const int32_t kept = csp_oracle_select(a_s, a_c, mod + (size_t)p * L, L, O, R, T, f[2], 0, idx, cnt);
        if (kept < 0 || kept > cap) { fprintf(stderr, "select returned %d\n", kept); return 3; }
        double* kc = malloc(sizeof(double) * (kept ? kept : 1) * D);
        double* vc = malloc(sizeof(double) * (kept ? kept : 1) * D);
        csp_oracle_gather(k + (size_t)p * L * D, sizeof(double) * D, idx, kept, kc);
        csp_oracle_gather(v + (size_t)p * L * D, sizeof(double) * D, idx, kept, vc);
        double* o = calloc(D, sizeof(double));
        csp_oracle_decode(q + (size_t)p * O * D, kc, vc, kept, D, f[1], o, NULL);
        memcpy(kc_all + (size_t)p * cap * D, kc, sizeof(double) * kept * D);
        memcpy(vc_all + (size_t)p * cap * D, vc, sizeof(double) * kept * D);
        wr(a_s, sizeof(double) * L, out); wr(a_c, sizeof(double) * L, out); wr(rs, sizeof(double) * O, out);
        wr(&kept, 4, out); wr(cnt, 16, out); wr(idx, sizeof(int32_t) * L, out); wr(o, sizeof(double) * D, out);
        free(a_s); free(a_c); free(rs); free(idx); free(kc); free(vc); free(o);
    }
    /* the batch drivers (OpenMP over independent problems) */
    double* bs = calloc((size_t)P * L, sizeof(double));
    double* bc = calloc((size_t)P * L, sizeof(double));
    csp_oracle_scores_batch(q, k, mod, P, L, O, R, D, f[0], causal, bs, bc);
    wr(bs, sizeof(double) * P * L, out); wr(bc, sizeof(double) * P * L, out);
    double* qd = malloc(sizeof(double) * P * D);
    for (int p = 0; p < P; ++p) memcpy(qd + (size_t)p * D, q + (size_t)p * O * D, sizeof(double) * D);
    double* bo = calloc((size_t)P * D, sizeof(double));
    csp_oracle_decode_batch(qd, kc_all, vc_all, P, cap, D, f[1], bo);
    wr(bo, sizeof(double) * P * D, out);
    free(q); free(k); free(v); free(mod); free(kc_all); free(vc_all); free(bs); free(bc); free(qd); free(bo);
    fclose(in); fclose(out);
    return 0;
}
