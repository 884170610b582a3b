/* Fixed-order single-precision references.  TEST INFRASTRUCTURE ONLY.
 *
 * SplitLoRA (arXiv 2407.00952), step b2, Eq. (8)-(9): the aggregated client adapter is
 * sum_i (|D_i|/|D|) x_i.  The GPU library promises a bit-exact fp32 result for ONE
 * stated evaluation order; this file is that order written out with C99 fmaf:
 *     w_i = (float)((double)n_i / (double)sum_j n_j)
 *     acc = 0.0f;  for i = 0 .. K-1 in client order:  acc = fmaf(w_i, x_i[j], acc)
 * Eq. (4)-(5), the SGD update, in the same spirit:  p = fmaf(-lr, g, p).
 * The AdamW variant (not in the paper) in one stated order, host scalars in double:
 *     decay = (float)(1 - lr*wd), a = (float)(lr / (1 - b1^t)), c = (float)(1 / sqrt(1 - b2^t)),
 *     o1 = (float)(1 - b1), o2 = (float)(1 - b2);
 *     m = fmaf(b1, m, o1*g);  v = fmaf(b2, v, (o2*g)*g);
 *     p = fmaf(-a, m / fmaf(sqrtf(v), c, eps), p*decay).
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

void oracle_adamw_f32(float *p, const float *g, float *m, float *v, size_t n, float lr, float b1, float b2,
                      float eps, float wd, int step)
{
    const float decay = (float)(1.0 - (double)lr * (double)wd);
    const float a = (float)((double)lr / (1.0 - pow((double)b1, (double)step)));
    const float c = (float)(1.0 / sqrt(1.0 - pow((double)b2, (double)step)));
    const float o1 = (float)(1.0 - (double)b1), o2 = (float)(1.0 - (double)b2);
    for (size_t j = 0; j < n; ++j) {
        const float gj = g[j];
        const float t1 = o1 * gj;
        const float mj = fmaf(b1, m[j], t1);
        const float t2 = o2 * gj;
        const float t3 = t2 * gj;
        const float vj = fmaf(b2, v[j], t3);
        const float den = fmaf(sqrtf(vj), c, eps);
        const float q = mj / den;
        const float pd = p[j] * decay;
        p[j] = fmaf(-a, q, pd);
        m[j] = mj;
        v[j] = vj;
    }
}
