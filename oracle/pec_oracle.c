/*
 * CPU oracle for blockwise causal prefill attention -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker, not the product: only tests, the smoke check and the
 * benchmark's cpu_baseline leg may build, load or call it.  It shares no code,
 * header, table or helper with the HIP path.
 *
 * What it computes is the plain definition, in fp64, with no tiling, no online
 * softmax and no reordering:
 *   - scaled dot-product attention per head, Eq. 2 of the paper (Self-attention,
 *     section "LLM Foundations"):  O^h = Softmax(Q^h (K^h)^T / sqrt(d_h)) V^h ;
 *   - the row softmax of Eq. 3, whose denominator runs over keys 1..t_i where t_i
 *     is the position of the token on row i, i.e. an inclusive causal mask;
 *   - the exact combination of two partial softmax results over disjoint key sets
 *     (the "online-softmax" step that ring attention relies on, section
 *     "Sequence Parallelism for Long Requests"), derived from Eq. 3 by splitting
 *     the denominator's sum into two parts.
 *
 * Pins (see tests/test_oracle_pins.py): literal Eq. 3 brute force on tiny inputs,
 * rows of softmax weights summing to 1, closed forms for Q = 0 / constant V /
 * row 0, a library attention routine in fp64, and chunk-split invariance.
 *
 * Layouts: q, out [sq, n_q_heads, d]; k, v [sk, n_kv_heads, d]; lse [n_q_heads, sq].
 * Inputs are either fp64 (in_dtype = 0) or bf16 bit patterns (in_dtype = 1), the
 * latter widened exactly.  Outputs are fp64.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F64 = 0, ORACLE_BF16 = 1 };

static inline double load_elem(const void *base, int in_dtype, size_t idx)
{
    if (in_dtype == ORACLE_F64)
        return ((const double *)base)[idx];
    /* bf16 is the top half of an IEEE fp32: shifting it back is an exact widening */
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Attention of sq query rows against sk keys (Eq. 2 with the softmax of Eq. 3).
 *
 * q_pos[i] is the global token position of query row i (for a contiguous segment
 * it is q_off + i); key j sits at global position kv_off + j.  Key j is visible to
 * row i when causal == 0, or when kv_off + j <= q_pos[i] (the sum of Eq. 3 stops at
 * the row's own token, which is included).  Query head h reads KV head h / g with
 * g = n_q_heads / n_kv_heads (contiguous groups, the grouped-query convention the
 * paper's cost model assumes in "Fast Sequence Parallelism for Long-Request
 * Prefill").
 *
 * A row with no visible key gets out = 0 and lse = -inf.
 * probs, when not NULL, receives the softmax weights b_ij as [n_q_heads, sq, sk]
 * (zero where masked) so that tests can check the rows sum to one.
 *
 * Returns 0, or -1 on invalid arguments.
 */
int oracle_attention(const void *q, const void *k, const void *v, int in_dtype,
                     int64_t sq, int64_t sk, int n_q_heads, int n_kv_heads, int d,
                     const int64_t *q_pos, int64_t kv_off, int causal, double scale,
                     double *out, double *lse, double *probs)
{
    if (sq < 0 || sk < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || d <= 0)
        return -1;
    if (n_q_heads % n_kv_heads != 0)
        return -1;
    const int g = n_q_heads / n_kv_heads;
    const int64_t n_rows = sq * (int64_t)n_q_heads;

#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * (size_t)(sk > 0 ? sk : 1));
#pragma omp for schedule(dynamic, 1)
        for (int64_t row = 0; row < n_rows; ++row) {
            const int64_t i = row / n_q_heads;
            const int h = (int)(row % n_q_heads);
            const int hk = h / g;
            const size_t qbase = ((size_t)i * n_q_heads + h) * d;
            double *o = out + qbase;
            for (int c = 0; c < d; ++c)
                o[c] = 0.0;

            /* a_ij = (q_i . k_j) * scale for every key, then the visible maximum */
            double m = -INFINITY;
            int64_t n_visible = 0;
            for (int64_t j = 0; j < sk; ++j) {
                const int visible = !causal || (kv_off + j <= q_pos[i]);
                if (!visible) {
                    a[j] = -INFINITY;
                    continue;
                }
                const size_t kbase = ((size_t)j * n_kv_heads + hk) * d;
                double dot = 0.0;
                for (int c = 0; c < d; ++c)
                    dot += load_elem(q, in_dtype, qbase + c) * load_elem(k, in_dtype, kbase + c);
                a[j] = dot * scale;
                if (a[j] > m)
                    m = a[j];
                ++n_visible;
            }

            if (n_visible == 0) {
                lse[(size_t)h * sq + i] = -INFINITY;
                if (probs)
                    for (int64_t j = 0; j < sk; ++j)
                        probs[((size_t)h * sq + i) * sk + j] = 0.0;
                continue;
            }

            /* denominator of Eq. 3 (shifted by m so that exp never overflows) */
            double l = 0.0;
            for (int64_t j = 0; j < sk; ++j)
                if (a[j] != -INFINITY) /* -inf marks a masked key */
                    l += exp(a[j] - m);

            /* O_i = sum_j b_ij v_j  with  b_ij = exp(a_ij - m) / l */
            for (int64_t j = 0; j < sk; ++j) {
                double b = 0.0;
                if (a[j] != -INFINITY) {
                    b = exp(a[j] - m) / l;
                    const size_t vbase = ((size_t)j * n_kv_heads + hk) * d;
                    for (int c = 0; c < d; ++c)
                        o[c] += b * load_elem(v, in_dtype, vbase + c);
                }
                if (probs)
                    probs[((size_t)h * sq + i) * sk + j] = b;
            }
            lse[(size_t)h * sq + i] = m + log(l);
        }
        free(a);
    }
    return 0;
}

/*
 * Exact combination of two partial results over disjoint key sets A and B.
 * With L_X = ln sum_{j in X} exp(a_ij) and O_X the softmax-weighted mean of v over
 * X, splitting the sum in Eq. 3's denominator gives
 *     L = ln(exp(L_A) + exp(L_B)),   O = O_A exp(L_A - L) + O_B exp(L_B - L).
 * An empty set is (O = 0, L = -inf) and is the identity.
 * o_* are [sq, n_q_heads, d], lse_* are [n_q_heads, sq]; result written to o, lse
 * (which may alias the A inputs).
 */
int oracle_merge(const double *o_a, const double *lse_a, const double *o_b, const double *lse_b,
                 int64_t sq, int n_q_heads, int d, double *o, double *lse)
{
    if (sq < 0 || n_q_heads <= 0 || d <= 0)
        return -1;
    for (int64_t i = 0; i < sq; ++i)
        for (int h = 0; h < n_q_heads; ++h) {
            const size_t li = (size_t)h * sq + i;
            const size_t ob = ((size_t)i * n_q_heads + h) * d;
            const double la = lse_a[li], lb = lse_b[li];
            if (la == -INFINITY && lb == -INFINITY) {
                lse[li] = -INFINITY;
                for (int c = 0; c < d; ++c)
                    o[ob + c] = 0.0;
                continue;
            }
            const double mx = la > lb ? la : lb;
            const double L = mx + log(exp(la - mx) + exp(lb - mx));
            const double wa = exp(la - L), wb = exp(lb - L);
            for (int c = 0; c < d; ++c)
                o[ob + c] = o_a[ob + c] * wa + o_b[ob + c] * wb;
            lse[li] = L;
        }
    return 0;
}
