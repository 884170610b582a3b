/* Fixed-order single-precision references.  TEST INFRASTRUCTURE ONLY.
 *
 * SplitLoRA (arXiv 2407.00952), step b2, Eq. (8)-(9): the aggregated client adapter is
 * sum_i (|D_i|/|D|) x_i.  The GPU library promises a bit-exact fp32 result for ONE
 * stated evaluation order; this file is that order written out with C99 fmaf:
 *     w_i = (float)((double)n_i / (double)sum_j n_j)
 *     acc = 0.0f;  for i = 0 .. K-1 in client order:  acc = fmaf(w_i, x_i[j], acc)
 * Eq. (4)-(5), the SGD update, in the same spirit:  p = fmaf(-lr, g, p).
 *
 * Built by gcc into libslora_oracle_c.so; shares nothing with the HIP sources.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

int oracle_fedavg_weights_f32(int K, const int64_t *counts, float *w)
{
    double tot = 0.0;
    for (int i = 0; i < K; ++i) {
        if (counts[i] < 0) return -1;
        tot += (double)counts[i];
    }
    if (!(tot > 0.0)) return -1;
    for (int i = 0; i < K; ++i) w[i] = (float)((double)counts[i] / tot);
    return 0;
}

void oracle_fedavg_f32(int K, const float *const *x, const float *w, size_t n, float *out)
{
    for (size_t j = 0; j < n; ++j) {
        float acc = 0.0f;
        for (int i = 0; i < K; ++i) acc = fmaf(w[i], x[i][j], acc);
        out[j] = acc;
    }
}

void oracle_sgd_f32(float *p, const float *g, float lr, size_t n)
{
    for (size_t j = 0; j < n; ++j) p[j] = fmaf(-lr, g[j], p[j]);
}
