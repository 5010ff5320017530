/*
 * TEST INFRASTRUCTURE -- not part of the product path.
 *
 * Plain fp64 CPU oracle for block-causal attention against a KV cache, the
 * operation the Inferix paper describes in its Introduction (framework
 * paragraph: at every denoising step the attention of the current block reads
 * a global KV cache holding the previously generated blocks) and in its
 * abstract (diffusion inside a block, conditioning on the previous blocks,
 * hence: bidirectional within the block, causal across blocks).
 *
 * The result has a plain definition, so the oracle is that definition written
 * out, with no tiling, no running maximum and no rescaling:
 *
 *   J        = { all C cached tokens }  U  { all n tokens of the current block, if one is given }
 *   s_ij     = scale * sum_d q[i,h,d] * k[j,h,d]                 j in J
 *   m_i      = max_j s_ij
 *   Z_i      = sum_j exp(s_ij - m_i)
 *   out[i,h] = sum_j (exp(s_ij - m_i) / Z_i) * v[j,h,:]
 *   lse_i    = m_i + log(Z_i)
 *
 * Three passes per row (scores and max; exponentials and sum; weighted sum),
 * everything in double. The cache is visited oldest token first, then the
 * block. Only tests/, the smoke check and the benchmark's cpu_baseline leg may
 * call this file; it shares nothing with the HIP library.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC ifx_oracle.c -o libifx_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of OpenMP threads the attention loop will use. */
int ifx_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Attention for a chosen list of (query row, head) pairs.
 *
 *   n, C, H, D   block tokens, cached tokens, heads, head dimension
 *   q            [n, H, D]   queries of the current block
 *   kc, vc       [C, H, D]   cached keys / values, any order (may be NULL if C == 0)
 *   kb, vb       [n, H, D]   keys / values of the current block; both NULL: the key set is the
 *                            cached tokens alone (attention over a chosen part of the cache,
 *                            KV Management section: range-based chunked access)
 *   scale        softmax scale (the caller passes 1/sqrt(D))
 *   n_sel        number of selected pairs
 *   sel_row      [n_sel] query row index i in [0, n)
 *   sel_head     [n_sel] head index h in [0, H)
 *   out          [n_sel, D]  result rows
 *   lse          [n_sel]     natural-log sum-exp of the scaled scores (may be NULL)
 *
 * Returns 0, or -1 on an invalid argument or allocation failure.
 */
int ifx_oracle_attention(int64_t n, int64_t C, int64_t H, int64_t D,
                         const double *q,
                         const double *kc, const double *vc,
                         const double *kb, const double *vb,
                         double scale,
                         int64_t n_sel, const int64_t *sel_row, const int64_t *sel_head,
                         double *out, double *lse)
{
    if (n <= 0 || C < 0 || H <= 0 || D <= 0 || n_sel < 0) return -1;
    if (!q || !out) return -1;
    if ((kb == NULL) != (vb == NULL)) return -1;
    if (C > 0 && (!kc || !vc)) return -1;
    if (C == 0 && !kb) return -1; /* no key at all */
    for (int64_t t = 0; t < n_sel; ++t) {
        if (sel_row[t] < 0 || sel_row[t] >= n) return -1;
        if (sel_head[t] < 0 || sel_head[t] >= H) return -1;
    }
    const int64_t Lk = C + (kb ? n : 0);
    int failed = 0;

#pragma omp parallel
    {
        double *s = (double *)malloc((size_t)Lk * sizeof(double));
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 4)
        for (int64_t t = 0; t < n_sel; ++t) {
            if (!s) continue;
            const int64_t i = sel_row[t], h = sel_head[t];
            const double *qi = q + (i * H + h) * D;

            /* pass 1: scores over cache then block, and their maximum */
            double m = -INFINITY;
            for (int64_t j = 0; j < Lk; ++j) {
                const double *kj = (j < C) ? kc + (j * H + h) * D
                                           : kb + ((j - C) * H + h) * D;
                double acc = 0.0;
                for (int64_t d = 0; d < D; ++d) acc += qi[d] * kj[d];
                s[j] = scale * acc;
                if (s[j] > m) m = s[j];
            }
            /* pass 2: exponentials and normaliser */
            double Z = 0.0;
            for (int64_t j = 0; j < Lk; ++j) {
                s[j] = exp(s[j] - m);
                Z += s[j];
            }
            /* pass 3: probability-weighted sum of values */
            double *o = out + t * D;
            for (int64_t d = 0; d < D; ++d) o[d] = 0.0;
            for (int64_t j = 0; j < Lk; ++j) {
                const double *vj = (j < C) ? vc + (j * H + h) * D
                                           : vb + ((j - C) * H + h) * D;
                const double p = s[j] / Z;
                for (int64_t d = 0; d < D; ++d) o[d] += p * vj[d];
            }
            if (lse) lse[t] = m + log(Z);
        }
        free(s);
    }
    return failed ? -1 : 0;
}
