/* CPU oracle for the SiDA-MoE layer output.  TEST INFRASTRUCTURE ONLY: it may be called from
 * tests/, from __graft_entry__.smoke() and from bench.py's cpu_baseline leg, never from the
 * product path.  It shares no code with the HIP kernels.
 *
 * What it computes (paper Section 2.1, Eq. 1, with the Switch top-1 selection |I| = 1, and the
 * table lookup of Section 3.1 in place of the router: the expert id k_t and the scaling factor
 * alpha_t of every token are inputs):
 *
 *     h_t[j] = max(0, sum_i x[t,i] * W_in[k_t][j,i])            j < F      (ReLU MLP, no bias)
 *     y[t,c] = alpha_t * sum_j h_t[j] * W_out[k_t][c,j]         c < d
 *
 * Each token is handled on its own, in token order, straight from this definition: no sorting,
 * grouping, tiling or fusion.  Inputs are bfloat16 bit patterns, upcast exactly; every sum runs
 * in index order in fp64, h is kept in fp64, and y is rounded once to fp32 on output.
 *
 * Pins (tests/test_oracle_*.py): E = 1 equals numpy's dense matmul FFN; pure-Python brute force
 * and hand-computed integer cases on tiny shapes; permutation equivariance; linearity in alpha;
 * independence of a token's output from the other tokens; identity experts give y == x.
 * The k-expert form: equals the top-1 form for k = 1, the sum of k top-1 layers, a repeated
 * expert equals one term with the alphas added, hand-computed integer case.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline float bf16_up(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* x: bf16 [T,d]; ids: [T]; alpha: fp32 [T]; blocks[e] -> bf16 block of expert e laid out as
 * W_in [F,d] followed by W_out [d,F]; y: fp32 [T,d].
 * Returns 0, or -1 when an id is outside [0,E) (nothing is written then). */
int sida_oracle_moe_forward(const uint16_t *x, const int32_t *ids, const float *alpha,
                            const uint16_t *const *blocks, int32_t E, int32_t T, int32_t d,
                            int32_t F, float *y)
{
    for (int32_t t = 0; t < T; ++t)
        if (ids[t] < 0 || ids[t] >= E) return -1;

#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)F);
        double *xt = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
        for (int32_t t = 0; t < T; ++t) {
            const uint16_t *w_in = blocks[ids[t]];
            const uint16_t *w_out = w_in + (size_t)F * (size_t)d;
            for (int32_t i = 0; i < d; ++i) xt[i] = (double)bf16_up(x[(size_t)t * d + i]);
            for (int32_t j = 0; j < F; ++j) {
                const uint16_t *row = w_in + (size_t)j * d;
                double s = 0.0;
                for (int32_t i = 0; i < d; ++i) s += xt[i] * (double)bf16_up(row[i]);
                h[j] = s > 0.0 ? s : 0.0;
            }
            for (int32_t c = 0; c < d; ++c) {
                const uint16_t *row = w_out + (size_t)c * F;
                double s = 0.0;
                for (int32_t j = 0; j < F; ++j) s += h[j] * (double)bf16_up(row[j]);
                y[(size_t)t * d + c] = (float)((double)alpha[t] * s);
            }
        }
        free(h);
        free(xt);
    }
    return 0;
}

/* Eq. 1 of Section 2.1 with a selected set I of k experts per token (the paper evaluates with the
 * top-3 experts of the hash function on two of its datasets, Section 4, hyperparameters):
 *
 *     y[t,c] = sum_{j<k} alpha[t,j] * ( W_out[e] relu(W_in[e] x_t) )[c],      e = ids[t,j]
 *
 * ids, alpha: [T,k] row-major.  Same conventions as above: per token, straight from the
 * definition, fp64 throughout, the k terms added in the order j = 0..k-1, one rounding to fp32.
 * Returns 0, or -1 when an id is outside [0,E) or k < 1 (nothing is written then). */
int sida_oracle_moe_forward_topk(const uint16_t *x, const int32_t *ids, const float *alpha,
                                 const uint16_t *const *blocks, int32_t E, int32_t T, int32_t k,
                                 int32_t d, int32_t F, float *y)
{
    if (k < 1) return -1;
    for (int64_t i = 0; i < (int64_t)T * k; ++i)
        if (ids[i] < 0 || ids[i] >= E) return -1;

#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)F);
        double *xt = (double *)malloc(sizeof(double) * (size_t)d);
        double *yt = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
        for (int32_t t = 0; t < T; ++t) {
            for (int32_t i = 0; i < d; ++i) xt[i] = (double)bf16_up(x[(size_t)t * d + i]);
            for (int32_t c = 0; c < d; ++c) yt[c] = 0.0;
            for (int32_t j = 0; j < k; ++j) {
                const uint16_t *w_in = blocks[ids[(size_t)t * k + j]];
                const uint16_t *w_out = w_in + (size_t)F * (size_t)d;
                const double a = (double)alpha[(size_t)t * k + j];
                for (int32_t u = 0; u < F; ++u) {
                    const uint16_t *row = w_in + (size_t)u * d;
                    double s = 0.0;
                    for (int32_t i = 0; i < d; ++i) s += xt[i] * (double)bf16_up(row[i]);
                    h[u] = s > 0.0 ? s : 0.0;
                }
                for (int32_t c = 0; c < d; ++c) {
                    const uint16_t *row = w_out + (size_t)c * F;
                    double s = 0.0;
                    for (int32_t u = 0; u < F; ++u) s += h[u] * (double)bf16_up(row[u]);
                    yt[c] += a * s;
                }
            }
            for (int32_t c = 0; c < d; ++c) y[(size_t)t * d + c] = (float)yt[c];
        }
        free(h);
        free(xt);
        free(yt);
    }
    return 0;
}

int sida_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
