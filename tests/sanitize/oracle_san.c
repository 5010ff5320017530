/*
 * Driver that runs the C oracle under AddressSanitizer and UndefinedBehaviorSanitizer on the
 * CPU (tests/test_sanitizers.py compiles it together with oracle/ifx_oracle.c).  Buffers are
 * heap allocations of exactly the documented sizes, so any access past an end is reported.
 * Cases: cache + block, cache only, block only, a single key, every error return.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int ifx_oracle_attention(int64_t n, int64_t C, int64_t H, int64_t D, const double *q, const double *kc, const double *vc,
                         const double *kb, const double *vb, double scale, int64_t n_sel, const int64_t *sel_row,
                         const int64_t *sel_head, double *out, double *lse);

static uint64_t state = 88172645463325252ull;
static double rnd(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static double *fill(int64_t count)
{
    double *p = (double *)malloc((size_t)(count > 0 ? count : 1) * sizeof(double));
    for (int64_t i = 0; i < count; ++i) p[i] = rnd();
    return p;
}

static int run(int64_t n, int64_t C, int64_t H, int64_t D, int with_block)
{
    double *q = fill(n * H * D), *kc = fill(C * H * D), *vc = fill(C * H * D), *kb = fill(n * H * D), *vb = fill(n * H * D);
    const int64_t n_sel = n * H;
    int64_t *rows = (int64_t *)malloc((size_t)n_sel * sizeof(int64_t)), *heads = (int64_t *)malloc((size_t)n_sel * sizeof(int64_t));
    for (int64_t t = 0; t < n_sel; ++t) {
        rows[t] = t / H;
        heads[t] = t % H;
    }
    double *out = (double *)malloc((size_t)(n_sel * D) * sizeof(double)), *lse = (double *)malloc((size_t)n_sel * sizeof(double));
    const int rc = ifx_oracle_attention(n, C, H, D, q, C ? kc : NULL, C ? vc : NULL, with_block ? kb : NULL, with_block ? vb : NULL,
                                        1.0 / sqrt((double)D), n_sel, rows, heads, out, lse);
    int bad = rc != 0;
    for (int64_t i = 0; i < n_sel * D && !bad; ++i) bad = !isfinite(out[i]);
    for (int64_t i = 0; i < n_sel && !bad; ++i) bad = !isfinite(lse[i]);
    free(q), free(kc), free(vc), free(kb), free(vb), free(rows), free(heads), free(out), free(lse);
    return bad;
}

int main(void)
{
    int bad = 0;
    bad |= run(7, 19, 3, 8, 1);
    bad |= run(5, 12, 2, 16, 0);
    bad |= run(9, 0, 2, 4, 1);
    bad |= run(1, 0, 1, 1, 1);
    /* error returns must not touch anything */
    double x[8] = {0};
    int64_t r0 = 0, h0 = 0, r_bad = 5;
    bad |= ifx_oracle_attention(0, 0, 1, 1, x, NULL, NULL, x, x, 1.0, 1, &r0, &h0, x, NULL) != -1;
    bad |= ifx_oracle_attention(1, 0, 1, 1, x, NULL, NULL, NULL, NULL, 1.0, 1, &r0, &h0, x, NULL) != -1;
    bad |= ifx_oracle_attention(1, 0, 1, 1, x, NULL, NULL, x, NULL, 1.0, 1, &r0, &h0, x, NULL) != -1;
    bad |= ifx_oracle_attention(1, 2, 1, 1, x, NULL, NULL, x, x, 1.0, 1, &r0, &h0, x, NULL) != -1;
    bad |= ifx_oracle_attention(1, 0, 1, 1, x, NULL, NULL, x, x, 1.0, 1, &r_bad, &h0, x, NULL) != -1;
    printf(bad ? "FAILED\n" : "ok\n");
    return bad;
}
