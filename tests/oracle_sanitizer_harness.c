/*
 * CPU harness for the sanitizer build of the fp64 oracle (tests/test_oracle_sanitizers.py compiles this
 * file together with oracle/ttt_oracle.c under -fsanitize=address,undefined and runs it).
 * It drives both input-type entry points and the mask-row routine over shapes that reach every
 * boundary of the oracle's buffers -- packed documents with empty ones, a length-1 document, GQA,
 * a sampled row list with repeats, forward-only and forward+backward calls, zero tokens -- and
 * checks facts that need no second implementation: constant values give O = that constant (rows of P
 * sum to one), the mass of dV equals the mass of dO, and the mask row has (i - start + 1) + j ones.
 * Exit code 0 = every check passed and no sanitizer report.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
    int32_t k, T, n_docs, hq, hkv, d;
    double scale;
} ttt_oracle_shape;

int ttt_oracle_run_f32in(const ttt_oracle_shape*, const int32_t*, const float*, const float*, const float*, int64_t,
                         const int32_t*, const int32_t*, const float*, double*, double*, double*, double*, double*);
int ttt_oracle_run_f64in(const ttt_oracle_shape*, const int32_t*, const double*, const double*, const double*, int64_t,
                         const int32_t*, const int32_t*, const double*, double*, double*, double*, double*, double*);
void ttt_oracle_mask_row(int j, int i, int k, int T, const int32_t* tok_doc, uint8_t* row);

static uint32_t lcg_state = 12345u;
static double lcg(void) { /* uniform in [-1, 1) */
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (double)(lcg_state >> 8) / 8388608.0 - 1.0;
}

#define CHECK(cond, ...) do { if (!(cond)) { fprintf(stderr, __VA_ARGS__); fprintf(stderr, "\n"); return 1; } } while (0)

static int run_case(int k, int n_docs, const int32_t* cu, int hq, int hkv, int d, int use_f64, int full_rows)
{
    const int T = cu[n_docs];
    const ttt_oracle_shape sh = {k, T, n_docs, hq, hkv, d, 1.0 / sqrt((double)d)};
    const size_t nq = (size_t)k * T * hq * d, nkv = (size_t)k * T * hkv * d;
    double* Q = malloc(sizeof(double) * (nq + 1));
    double* K = malloc(sizeof(double) * (nkv + 1));
    double* V = malloc(sizeof(double) * (nkv + 1));
    float *Qf = malloc(sizeof(float) * (nq + 1)), *Kf = malloc(sizeof(float) * (nkv + 1)), *Vf = malloc(sizeof(float) * (nkv + 1));
    for (size_t x = 0; x < nq; ++x) Qf[x] = (float)(Q[x] = (double)(float)lcg());
    for (size_t x = 0; x < nkv; ++x) Kf[x] = (float)(K[x] = (double)(float)lcg());
    for (size_t x = 0; x < nkv; ++x) Vf[x] = (float)(V[x] = 0.75);   /* constant values: O must be 0.75 */
    /* row list: every row, or a sample with a repeated row */
    int64_t n_rows = full_rows ? (int64_t)k * T : (T > 0 ? 5 : 0);
    int32_t* rs = malloc(sizeof(int32_t) * (size_t)(n_rows + 1));
    int32_t* rt = malloc(sizeof(int32_t) * (size_t)(n_rows + 1));
    for (int64_t r = 0; r < n_rows; ++r) {
        if (full_rows) { rs[r] = (int32_t)(r / T); rt[r] = (int32_t)(r % T); }
        else { rs[r] = (int32_t)((r * 7) % k); rt[r] = (int32_t)(r == 4 ? rt[0] : (r * 13 + T - 1) % T); if (r == 4) rs[r] = rs[0]; }
    }
    const size_t nr = (size_t)n_rows * hq * d;
    double* dO = malloc(sizeof(double) * (nr + 1));
    float* dOf = malloc(sizeof(float) * (nr + 1));
    for (size_t x = 0; x < nr; ++x) dOf[x] = (float)(dO[x] = (double)(float)lcg());
    double* O = malloc(sizeof(double) * (nr + 1));
    double* LSE = malloc(sizeof(double) * ((size_t)n_rows * hq + 1));
    double* dQ = malloc(sizeof(double) * (nr + 1));
    double* dK = malloc(sizeof(double) * (nkv + 1));
    double* dV = malloc(sizeof(double) * (nkv + 1));
    int rc;
    /* forward only first (no cotangent, no gradient buffers), then forward + backward */
    rc = use_f64 ? ttt_oracle_run_f64in(&sh, cu, Q, K, V, n_rows, rs, rt, NULL, O, LSE, NULL, NULL, NULL)
                 : ttt_oracle_run_f32in(&sh, cu, Qf, Kf, Vf, n_rows, rs, rt, NULL, O, LSE, NULL, NULL, NULL);
    CHECK(rc == 0, "forward-only call returned %d", rc);
    rc = use_f64 ? ttt_oracle_run_f64in(&sh, cu, Q, K, V, n_rows, rs, rt, dO, O, LSE, dQ, dK, dV)
                 : ttt_oracle_run_f32in(&sh, cu, Qf, Kf, Vf, n_rows, rs, rt, dOf, O, LSE, dQ, dK, dV);
    CHECK(rc == 0, "forward+backward call returned %d", rc);
    for (size_t x = 0; x < nr; ++x) CHECK(fabs(O[x] - 0.75) < 1e-12, "O[%zu] = %.17g, expected the constant value", x, O[x]);
    for (size_t x = 0; x < nr; ++x) CHECK(fabs(dQ[x]) < 1e-9, "dQ[%zu] = %.3g, expected 0 for constant values", x, dQ[x]);
    double mass_dv = 0.0, mass_do = 0.0;
    for (size_t x = 0; x < nkv; ++x) mass_dv += dV[x];
    for (size_t x = 0; x < nr; ++x) mass_do += dO[x];
    CHECK(fabs(mass_dv - mass_do) < 1e-9 * (1.0 + fabs(mass_do)), "sum dV = %.12g but sum dO = %.12g", mass_dv, mass_do);
    /* mask rows: count of visible slots */
    if (T > 0) {
        int32_t* tok_doc = malloc(sizeof(int32_t) * (size_t)T);
        int32_t* start = malloc(sizeof(int32_t) * (size_t)T);
        for (int r = 0; r < n_docs; ++r)
            for (int i = cu[r]; i < cu[r + 1]; ++i) { tok_doc[i] = r; start[i] = cu[r]; }
        uint8_t* row = malloc((size_t)k * T);
        for (int j = 0; j < k; ++j)
            for (int i = 0; i < T; ++i) {
                ttt_oracle_mask_row(j, i, k, T, tok_doc, row);
                int cnt = 0;
                for (int s = 0; s < k * T; ++s) cnt += row[s];
                CHECK(cnt == i - start[i] + 1 + j, "mask row (%d,%d) has %d ones, expected %d", j, i, cnt, i - start[i] + 1 + j);
            }
        free(tok_doc); free(start); free(row);
    }
    free(Q); free(K); free(V); free(Qf); free(Kf); free(Vf); free(rs); free(rt);
    free(dO); free(dOf); free(O); free(LSE); free(dQ); free(dK); free(dV);
    return 0;
}

int main(void)
{
    const int32_t cu_a[] = {0, 0, 9, 10, 10, 23};      /* empty documents, a length-1 document */
    const int32_t cu_b[] = {0, 17};
    const int32_t cu_c[] = {0, 0};                     /* no tokens at all */
    const int32_t cu_d[] = {0, 1, 2, 3, 4};            /* only length-1 documents */
    int bad = 0;
    bad |= run_case(3, 5, cu_a, 4, 2, 8, 0, 1);
    bad |= run_case(3, 5, cu_a, 4, 2, 8, 1, 0);
    bad |= run_case(1, 1, cu_b, 2, 2, 4, 1, 1);
    bad |= run_case(4, 1, cu_b, 6, 2, 16, 0, 0);
    bad |= run_case(2, 1, cu_c, 2, 1, 4, 0, 1);
    bad |= run_case(5, 4, cu_d, 3, 3, 4, 1, 1);
    if (!bad) printf("oracle sanitizer harness: all cases passed\n");
    return bad;
}
