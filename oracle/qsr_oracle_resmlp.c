/*
 * qsr_oracle_resmlp.c -- local gradient (Eq. (1) of arXiv 2310.14423) of the
 * residual-MLP workload, in plain double-precision loops.
 *
 * TEST INFRASTRUCTURE, like qsr_oracle.c: never on the product path.
 *
 * The paper's transformer workload (Sec. 4, App. C.2: ViT-B, width 768, MLP
 * width 3072, 12 blocks) is stood in for by its MLP sub-blocks only:
 *
 *   x_0   = tokens [M][d], standard normal single-precision data
 *   y     = x_0 W_T / sqrt(d)                 (fixed random linear teacher)
 *   u_l   = gamma_l * (x_l - mean)/sqrt(var + 1e-5) + beta_l     (LayerNorm)
 *   h_l   = u_l W1_l + b1_l ;  a_l = h_l * Phi(h_l)              (erf GELU)
 *   x_l+1 = x_l + a_l W2_l + b2_l
 *   loss  = 1/(2 M d) * sum (x_L - y)^2
 *
 * Per-block parameter packing: gamma[d], beta[d], W1[d][dh], b1[dh],
 * W2[dh][d], b2[d].  No value of this model is printed by the paper: the
 * gradient is pinned by library autograd and finite differences (parity
 * otherwise unpinned).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include "qsr_oracle.h"


#define LN_EPS 1e-5

/* tokens of worker k at iteration t and their teacher targets */
void qsro_resmlp_batch(const qsro_config *c, int32_t k, int64_t t, double *x0, double *y)
{
    int64_t M = c->B_loc, d = c->d_in;
    int64_t total = M * d;
    for (int64_t e = 0; e < total; e += 4) {
        float z[4];
        qsro_normal4(c->seed, 1u /* stream X */, (uint32_t)k, (uint64_t)t, (uint64_t)(e >> 2), z);
        for (int64_t r = 0; r < 4 && e + r < total; ++r) x0[e + r] = (double)z[r];
    }
    double sc = 1.0 / sqrt((double)d);
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < d; ++j) y[i * d + j] = 0.0;
        for (int64_t l = 0; l < d; ++l) {
            double xv = x0[i * d + l];
            for (int64_t j = 0; j < d; ++j) y[i * d + j] += xv * (double)c->model_const[l * d + j];
        }
        for (int64_t j = 0; j < d; ++j) y[i * d + j] *= sc;
    }
}

double qsro_grad_resmlp(const qsro_config *c, int32_t k, int64_t t, const double *th, double *g)
{
    int64_t M = c->B_loc, d = c->d_in, dh = c->d_hidden;
    int32_t L = c->n_blocks;
    int64_t per_block = 2 * d + d * dh + dh + dh * d + d;
    double *xs = (double *)malloc(sizeof(double) * (size_t)((L + 1) * M * d)); /* x_0..x_L   */
    double *y = (double *)malloc(sizeof(double) * (size_t)(M * d));
    double *uh = (double *)malloc(sizeof(double) * (size_t)(L * M * d));       /* normalised */
    double *rs = (double *)malloc(sizeof(double) * (size_t)(L * M));           /* 1/std      */
    double *hs = (double *)malloc(sizeof(double) * (size_t)(L * M * dh));      /* pre-GELU   */
    double *u = (double *)malloc(sizeof(double) * (size_t)d);
    double *a = (double *)malloc(sizeof(double) * (size_t)dh);
    double *dx = (double *)malloc(sizeof(double) * (size_t)(M * d));
    double *da = (double *)malloc(sizeof(double) * (size_t)dh);
    double *du = (double *)malloc(sizeof(double) * (size_t)d);

    qsro_resmlp_batch(c, k, t, xs, y);

    /* forward */
    for (int32_t l = 0; l < L; ++l) {
        const double *gam = th + (int64_t)l * per_block, *bet = gam + d, *W1 = bet + d,
                     *b1 = W1 + d * dh, *W2 = b1 + dh, *b2 = W2 + dh * d;
        const double *x = xs + (int64_t)l * M * d;
        double *xn = xs + (int64_t)(l + 1) * M * d;
        for (int64_t i = 0; i < M; ++i) {
            double mean = 0.0, var = 0.0;
            for (int64_t j = 0; j < d; ++j) mean += x[i * d + j];
            mean /= (double)d;
            for (int64_t j = 0; j < d; ++j) var += (x[i * d + j] - mean) * (x[i * d + j] - mean);
            var /= (double)d;
            double rstd = 1.0 / sqrt(var + LN_EPS);
            rs[(int64_t)l * M + i] = rstd;
            double *uhat = uh + ((int64_t)l * M + i) * d;
            for (int64_t j = 0; j < d; ++j) {
                uhat[j] = (x[i * d + j] - mean) * rstd;
                u[j] = gam[j] * uhat[j] + bet[j];
            }
            double *h = hs + ((int64_t)l * M + i) * dh;
            for (int64_t j = 0; j < dh; ++j) h[j] = b1[j];
            for (int64_t q = 0; q < d; ++q)
                for (int64_t j = 0; j < dh; ++j) h[j] += u[q] * W1[q * dh + j];
            for (int64_t j = 0; j < dh; ++j) a[j] = 0.5 * h[j] * (1.0 + erf(h[j] * M_SQRT1_2));
            for (int64_t j = 0; j < d; ++j) xn[i * d + j] = x[i * d + j] + b2[j];
            for (int64_t q = 0; q < dh; ++q)
                for (int64_t j = 0; j < d; ++j) xn[i * d + j] += a[q] * W2[q * d + j];
        }
    }

    /* loss and its gradient with respect to x_L */
    const double *xL = xs + (int64_t)L * M * d;
    double loss = 0.0, inv = 1.0 / ((double)M * (double)d);
    for (int64_t e = 0; e < M * d; ++e) {
        double r = xL[e] - y[e];
        loss += 0.5 * r * r;
        dx[e] = r * inv;
    }
    loss *= inv;

    /* backward */
    for (int64_t e = 0; e < (int64_t)L * per_block; ++e) g[e] = 0.0;
    for (int32_t l = L - 1; l >= 0; --l) {
        const double *gam = th + (int64_t)l * per_block, *bet = gam + d, *W1 = bet + d,
                     *b1 = W1 + d * dh, *W2 = b1 + dh;
        double *ggam = g + (int64_t)l * per_block, *gbet = ggam + d, *gW1 = gbet + d,
               *gb1 = gW1 + d * dh, *gW2 = gb1 + dh, *gb2 = gW2 + dh * d;
        (void)b1;
        for (int64_t i = 0; i < M; ++i) {
            const double *uhat = uh + ((int64_t)l * M + i) * d;
            const double *h = hs + ((int64_t)l * M + i) * dh;
            double *dxi = dx + i * d;                     /* d loss / d x_{l+1}[i] */
            for (int64_t j = 0; j < d; ++j) gb2[j] += dxi[j];
            for (int64_t q = 0; q < dh; ++q) {
                double cdf = 0.5 * (1.0 + erf(h[q] * M_SQRT1_2));
                double aq = h[q] * cdf;
                double acc = 0.0;
                for (int64_t j = 0; j < d; ++j) {
                    gW2[q * d + j] += aq * dxi[j];
                    acc += W2[q * d + j] * dxi[j];
                }
                double pdf = exp(-0.5 * h[q] * h[q]) / sqrt(2.0 * M_PI);
                da[q] = acc * (cdf + h[q] * pdf);         /* d loss / d h[q] */
                gb1[q] += da[q];
            }
            for (int64_t q = 0; q < d; ++q) {
                double uq = gam[q] * uhat[q] + bet[q];
                double acc = 0.0;
                for (int64_t j = 0; j < dh; ++j) {
                    gW1[q * dh + j] += uq * da[j];
                    acc += W1[q * dh + j] * da[j];
                }
                du[q] = acc;                              /* d loss / d u[q] */
            }
            double m1 = 0.0, m2 = 0.0;
            for (int64_t q = 0; q < d; ++q) {
                ggam[q] += du[q] * uhat[q];
                gbet[q] += du[q];
                double dn = du[q] * gam[q];
                m1 += dn;
                m2 += dn * uhat[q];
            }
            m1 /= (double)d; m2 /= (double)d;
            double rstd = rs[(int64_t)l * M + i];
            for (int64_t q = 0; q < d; ++q) {
                double dn = du[q] * gam[q];
                dxi[q] += rstd * (dn - m1 - uhat[q] * m2); /* residual + LayerNorm path */
            }
        }
    }
    free(xs); free(y); free(uh); free(rs); free(hs); free(u); free(a); free(dx); free(da); free(du);
    return loss;
}
