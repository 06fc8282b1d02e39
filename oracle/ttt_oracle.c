/*
 * TEST INFRASTRUCTURE ONLY -- fp64 CPU oracle for training-time-test (TTT) attention.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use it; the GPU library
 * never does, and the two share no code.
 *
 * What it computes (plain definition, no tiling, no analytic skipping):
 *   The draft layer is unrolled over k steps.  Step j appends its keys/values K_j, V_j (one block
 *   of T rows) to the cache and then attends with Q_j (Sec. 4.2.1, "Sparse Tree Attention").
 *   Query (step j, token i, head h) uses kv head g = h / (hq/hkv) and sees key slot (block l, token m)
 *   iff the BlockMask predicate of Alg. 2 holds:
 *        causal part:  l == 0, m <= i           (prefix keys, own position included)
 *        suffix part:  1 <= l <= j, m == i      (one diagonal key per cached later block)
 *   and, for packed batches, only inside the query's own document.
 *   Scores s = scale * <Q_j[i,h], K_l[m,g]>, one softmax over all visible slots, output
 *   O_j[i,h] = sum p * V_l[m,g]   (Alg. 1; Sec. 2.4 equation for o_t), LSE = log sum exp s.
 *   Backward is the softmax-attention vector-Jacobian product of that forward (the paper defers
 *   it to autograd): D = <dO,O>, dp = <dO,V>, ds = p (dp - D), dQ = scale sum ds K,
 *   dK = scale sum ds Q, dV = sum p dO, the last two summed over every (step, head in group, row)
 *   that sees the key.
 *
 * Pins (tests/test_oracle_*.py): k=1 against a library causal attention; the k-step form against a
 * library attention over the concatenated sequence with an explicit boolean mask built from
 * Alg. 2's modular-arithmetic predicate; central finite differences; closed forms (all-zero keys,
 * constant values, length-1 documents); shift / scale / mass invariants; row sums.
 *
 * Layouts: Q [k][T][hq][d], K,V [k][T][hkv][d] contiguous; per-row outputs are indexed by the
 * position r in the caller's row list: O_rows,dQ_rows [n_rows][hq][d], LSE_rows [n_rows][hq];
 * dK,dV [k][T][hkv][d] hold the sums over the listed rows only (so a full run lists every row, and
 * a sampled run equals a full run whose cotangent is zero off the sample).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t k;        /* number of TTT steps (cache blocks) */
    int32_t T;        /* packed tokens */
    int32_t n_docs;   /* documents; cu_seqlens has n_docs+1 entries */
    int32_t hq, hkv, d;
    double scale;     /* 1/sqrt(d_k) in the paper; passed by the caller */
} ttt_oracle_shape;

/* Alg. 2 restated on (block, token) coordinates for packed documents. */
int ttt_oracle_visible(int j, int i, int l, int m, const int32_t* tok_doc)
{
    if (tok_doc[i] != tok_doc[m]) return 0;
    if (l == 0) return m <= i;
    return l <= j && m == i;
}

/* Explicit mask row of query (j,i) over all k*T key slots, slot = l*T + m. */
void ttt_oracle_mask_row(int j, int i, int k, int T, const int32_t* tok_doc, uint8_t* row)
{
    for (int l = 0; l < k; ++l)
        for (int m = 0; m < T; ++m)
            row[(int64_t)l * T + m] = (uint8_t)ttt_oracle_visible(j, i, l, m, tok_doc);
}

#define CAT2(a, b) a##b
#define CAT(a, b) CAT2(a, b)

#define REAL float
#define FN(name) CAT(name, _f32in)
#include "ttt_oracle_core.inc"
#undef REAL
#undef FN

#define REAL double
#define FN(name) CAT(name, _f64in)
#include "ttt_oracle_core.inc"
#undef REAL
#undef FN
