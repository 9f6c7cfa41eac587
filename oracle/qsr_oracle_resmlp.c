/*
 * qsr_oracle_resmlp.c -- local gradient (Eq. (1) of arXiv 2310.14423) of the
 * residual-MLP workload, in plain double-precision loops.
 *
 * TEST INFRASTRUCTURE, like qsr_oracle.c: never on the product path.
 *
 * The paper's transformer workload (Sec. 4, App. C.2: ViT-B, width 768, MLP
 * width 3072, 12 blocks) is stood in for by its MLP sub-blocks (and, on
 * request, its attention sub-blocks, see below):
 *
 *   x_0   = tokens [M][d], standard normal single-precision data
 *   y     = x_0 W_T / sqrt(d)                 (fixed random linear teacher)
 *   u_l   = gamma_l * (x_l - mean)/sqrt(var + 1e-5) + beta_l     (LayerNorm)
 *   h_l   = u_l W1_l + b1_l ;  a_l = h_l * Phi(h_l)              (erf GELU)
 *   x_l+1 = x_l + a_l W2_l + b2_l
 *   loss  = 1/(2 M d) * sum (x_L - y)^2
 *
 * Per-block parameter packing: gamma[d], beta[d], W1[d][dh], b1[dh],
 * W2[dh][d], b2[d].
 *
 * With n_heads > 0 every block starts with the other half of a ViT encoder
 * block (App. C.2 trains ViT-B: 12 heads of width 64, sequences of 196 or 197
 * tokens), pre-LayerNorm multi-head self-attention over the tokens of one
 * sequence (seq_len consecutive token rows), bidirectional, no dropout:
 *
 *   u     = LayerNorm(x_l; gamma_a, beta_a)
 *   q|k|v = u Wqkv + bqkv            (columns [0,d) q, [d,2d) k, [2d,3d) v;
 *                                     head j owns columns j*dk..(j+1)*dk of each)
 *   p_ij  = softmax_j(q_i . k_j / sqrt(dk))   over the tokens j of i's sequence
 *   o_i   = sum_j p_ij v_j           (heads side by side, [M][d])
 *   x_l'  = x_l + o Wo + bo          and the MLP sub-block then starts from x_l'
 *
 * and the block's parameters are gamma_a[d], beta_a[d], Wqkv[d][3d], bqkv[3d],
 * Wo[d][d], bo[d] followed by the six arrays above.  No value of this model is
 * printed by the paper: the gradient is pinned by library autograd (with the
 * library's own attention routine), finite differences and two special cases
 * with closed forms (parity otherwise unpinned).
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


/* LayerNorm of M rows: uhat = (x - mean)/sqrt(var + eps), u = gamma*uhat + beta */
static void ln_forward(const double *x, const double *gam, const double *bet, int64_t M, int64_t d,
                       double *uhat, double *rstd, double *u)
{
    for (int64_t i = 0; i < M; ++i) {
        double mean = 0.0, var = 0.0;
        for (int64_t j = 0; j < d; ++j) mean += x[i * d + j];
        mean /= (double)d;
        for (int64_t j = 0; j < d; ++j) var += (x[i * d + j] - mean) * (x[i * d + j] - mean);
        var /= (double)d;
        rstd[i] = 1.0 / sqrt(var + LN_EPS);
        for (int64_t j = 0; j < d; ++j) {
            uhat[i * d + j] = (x[i * d + j] - mean) * rstd[i];
            u[i * d + j] = gam[j] * uhat[i * d + j] + bet[j];
        }
    }
}

/* attention probabilities of query i (a token row) in head hd: p[0..S) over its sequence */
static void attn_probs(const double *qkv, int64_t d, int64_t dk, int64_t S, int64_t i, int64_t hd,
                       double *p)
{
    int64_t j0 = (i / S) * S;
    const double *q = qkv + i * 3 * d + hd * dk;
    double mx = -INFINITY, sum = 0.0;
    for (int64_t j = 0; j < S; ++j) {
        const double *k = qkv + (j0 + j) * 3 * d + d + hd * dk;
        double s = 0.0;
        for (int64_t c = 0; c < dk; ++c) s += q[c] * k[c];
        p[j] = s / sqrt((double)dk);
        if (p[j] > mx) mx = p[j];
    }
    for (int64_t j = 0; j < S; ++j) { p[j] = exp(p[j] - mx); sum += p[j]; }
    for (int64_t j = 0; j < S; ++j) p[j] /= sum;
}

/* x_out = x + MultiHeadAttention(LayerNorm(x)) Wo + bo; keeps uhat, rstd, u, qkv, o for backward */
static void attn_forward(const double *x, const double *par, int64_t M, int64_t d, int64_t heads,
                         int64_t S, double *uhat, double *rstd, double *u, double *qkv, double *o,
                         double *x_out)
{
    const double *gam = par, *bet = gam + d, *Wqkv = bet + d, *bqkv = Wqkv + d * 3 * d,
                 *Wo = bqkv + 3 * d, *bo = Wo + d * d;
    int64_t dk = d / heads;
    double *p = (double *)malloc(sizeof(double) * (size_t)S);
    ln_forward(x, gam, bet, M, d, uhat, rstd, u);
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t c = 0; c < 3 * d; ++c) qkv[i * 3 * d + c] = bqkv[c];
        for (int64_t q = 0; q < d; ++q)
            for (int64_t c = 0; c < 3 * d; ++c) qkv[i * 3 * d + c] += u[i * d + q] * Wqkv[q * 3 * d + c];
    }
    for (int64_t i = 0; i < M; ++i) {
        int64_t j0 = (i / S) * S;
        for (int64_t hd = 0; hd < heads; ++hd) {
            attn_probs(qkv, d, dk, S, i, hd, p);
            for (int64_t c = 0; c < dk; ++c) {
                double acc = 0.0;
                for (int64_t j = 0; j < S; ++j) acc += p[j] * qkv[(j0 + j) * 3 * d + 2 * d + hd * dk + c];
                o[i * d + hd * dk + c] = acc;
            }
        }
    }
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < d; ++j) x_out[i * d + j] = x[i * d + j] + bo[j];
        for (int64_t q = 0; q < d; ++q)
            for (int64_t j = 0; j < d; ++j) x_out[i * d + j] += o[i * d + q] * Wo[q * d + j];
    }
    free(p);
}

/* dx holds d loss / d x_out on entry and d loss / d x on return; the parameter gradients of the
 * sub-block are added into gpar (same packing as par) */
static void attn_backward(const double *par, double *gpar, int64_t M, int64_t d, int64_t heads,
                          int64_t S, const double *uhat, const double *rstd, const double *u,
                          const double *qkv, const double *o, double *dx)
{
    const double *gam = par, *Wqkv = gam + 2 * d, *Wo = Wqkv + d * 3 * d + 3 * d;
    double *ggam = gpar, *gbet = ggam + d, *gWqkv = gbet + d, *gbqkv = gWqkv + d * 3 * d,
           *gWo = gbqkv + 3 * d, *gbo = gWo + d * d;
    int64_t dk = d / heads;
    double scale = 1.0 / sqrt((double)dk);
    double *dout = (double *)calloc((size_t)(M * d), sizeof(double));      /* d loss / d o   */
    double *dqkv = (double *)calloc((size_t)(M * 3 * d), sizeof(double));  /* d loss / d qkv */
    double *p = (double *)malloc(sizeof(double) * (size_t)S);
    double *dp = (double *)malloc(sizeof(double) * (size_t)S);
    double *du = (double *)malloc(sizeof(double) * (size_t)d);
    /* output projection */
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < d; ++j) gbo[j] += dx[i * d + j];
        for (int64_t q = 0; q < d; ++q) {
            double acc = 0.0;
            for (int64_t j = 0; j < d; ++j) {
                gWo[q * d + j] += o[i * d + q] * dx[i * d + j];
                acc += Wo[q * d + j] * dx[i * d + j];
            }
            dout[i * d + q] = acc;
        }
    }
    /* softmax(q k^T / sqrt(dk)) v, one query row at a time */
    for (int64_t i = 0; i < M; ++i) {
        int64_t j0 = (i / S) * S;
        for (int64_t hd = 0; hd < heads; ++hd) {
            const double *q = qkv + i * 3 * d + hd * dk;
            const double *doi = dout + i * d + hd * dk;
            double *dq = dqkv + i * 3 * d + hd * dk;
            attn_probs(qkv, d, dk, S, i, hd, p);
            double dot = 0.0;
            for (int64_t j = 0; j < S; ++j) {
                const double *v = qkv + (j0 + j) * 3 * d + 2 * d + hd * dk;
                double *dv = dqkv + (j0 + j) * 3 * d + 2 * d + hd * dk;
                double acc = 0.0;
                for (int64_t c = 0; c < dk; ++c) {
                    acc += doi[c] * v[c];
                    dv[c] += p[j] * doi[c];
                }
                dp[j] = acc;
                dot += p[j] * acc;
            }
            for (int64_t j = 0; j < S; ++j) {
                double ds = p[j] * (dp[j] - dot) * scale;      /* d loss / d (q_i . k_j) */
                const double *k = qkv + (j0 + j) * 3 * d + d + hd * dk;
                double *dkk = dqkv + (j0 + j) * 3 * d + d + hd * dk;
                for (int64_t c = 0; c < dk; ++c) {
                    dq[c] += ds * k[c];
                    dkk[c] += ds * q[c];
                }
            }
        }
    }
    /* q|k|v projection, then LayerNorm backward + the residual path */
    for (int64_t i = 0; i < M; ++i) {
        const double *dz = dqkv + i * 3 * d;
        for (int64_t c = 0; c < 3 * d; ++c) gbqkv[c] += dz[c];
        for (int64_t q = 0; q < d; ++q) {
            double acc = 0.0;
            for (int64_t c = 0; c < 3 * d; ++c) {
                gWqkv[q * 3 * d + c] += u[i * d + q] * dz[c];
                acc += Wqkv[q * 3 * d + c] * dz[c];
            }
            du[q] = acc;
        }
        double m1 = 0.0, m2 = 0.0;
        for (int64_t q = 0; q < d; ++q) {
            ggam[q] += du[q] * uhat[i * d + q];
            gbet[q] += du[q];
            double dn = du[q] * gam[q];
            m1 += dn;
            m2 += dn * uhat[i * d + q];
        }
        m1 /= (double)d; m2 /= (double)d;
        for (int64_t q = 0; q < d; ++q) {
            double dn = du[q] * gam[q];
            dx[i * d + q] += rstd[i] * (dn - m1 - uhat[i * d + q] * m2);
        }
    }
    free(dout); free(dqkv); free(p); free(dp); free(du);
}

double qsro_grad_resmlp(const qsro_config *c, int32_t k, int64_t t, const double *th, double *g)
{
    int64_t M = c->B_loc, d = c->d_in, dh = c->d_hidden;
    int32_t L = c->n_blocks;
    int64_t heads = c->n_heads, S = c->seq_len;
    int64_t per_attn = heads > 0 ? 2 * d + d * 3 * d + 3 * d + d * d + d : 0;
    int64_t per_block = per_attn + 2 * d + d * dh + dh + dh * d + d;
    int64_t nsub = heads > 0 ? 2 : 1;                  /* residual-stream states per block */
    double *xs = (double *)malloc(sizeof(double) * (size_t)((nsub * L + 1) * M * d)); /* x_0..x_L and the x_l' */
    /* kept by the attention sub-blocks for their backward pass */
    size_t na = heads > 0 ? (size_t)(L * M * d) : 1;
    double *a_uh = (double *)malloc(sizeof(double) * na), *a_u = (double *)malloc(sizeof(double) * na);
    double *a_o = (double *)malloc(sizeof(double) * na), *a_qkv = (double *)malloc(sizeof(double) * 3 * na);
    double *a_rs = (double *)malloc(sizeof(double) * (size_t)(L * M));
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
        const double *gam = th + (int64_t)l * per_block + per_attn, *bet = gam + d, *W1 = bet + d,
                     *b1 = W1 + d * dh, *W2 = b1 + dh, *b2 = W2 + dh * d;
        if (heads > 0)
            attn_forward(xs + (int64_t)(2 * l) * M * d, th + (int64_t)l * per_block, M, d, heads, S,
                         a_uh + (int64_t)l * M * d, a_rs + (int64_t)l * M, a_u + (int64_t)l * M * d,
                         a_qkv + (int64_t)l * M * 3 * d, a_o + (int64_t)l * M * d,
                         xs + (int64_t)(2 * l + 1) * M * d);
        const double *x = xs + (int64_t)(nsub * l + nsub - 1) * M * d;
        double *xn = xs + (int64_t)(nsub * l + nsub) * M * d;
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
    const double *xL = xs + (int64_t)(nsub * L) * M * d;
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
        const double *gam = th + (int64_t)l * per_block + per_attn, *bet = gam + d, *W1 = bet + d,
                     *b1 = W1 + d * dh, *W2 = b1 + dh;
        double *ggam = g + (int64_t)l * per_block + per_attn, *gbet = ggam + d, *gW1 = gbet + d,
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
        if (heads > 0)          /* dx now holds d loss / d x_l' */
            attn_backward(th + (int64_t)l * per_block, g + (int64_t)l * per_block, M, d, heads, S,
                          a_uh + (int64_t)l * M * d, a_rs + (int64_t)l * M, a_u + (int64_t)l * M * d,
                          a_qkv + (int64_t)l * M * 3 * d, a_o + (int64_t)l * M * d, dx);
    }
    free(a_uh); free(a_u); free(a_o); free(a_qkv); free(a_rs);
    free(xs); free(y); free(uh); free(rs); free(hs); free(u); free(a); free(dx); free(da); free(du);
    return loss;
}
