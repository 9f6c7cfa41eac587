/*
 * qsr_oracle.c -- plain CPU reference for Local SGD / Local AdamW with the
 * Quadratic Synchronization Rule (QSR).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is slow on purpose, shares no code
 * with the GPU library, and is called only by the tests, by the smoke check
 * and by the benchmark's CPU-baseline leg.  It must never serve the product
 * path.
 *
 * What it follows (arXiv 2310.14423):
 *   - Sec. 2 "Local Gradient Methods", Eq. (1), and Alg. 2 (Local OPT):
 *     K workers, H^(s) local steps per round, then parameter averaging.
 *   - Sec. 2 "Quadratic Synchronization Rule", Eq. (2):
 *     H^(s) = max{H_base, floor((alpha/eta_t)^2)} at the iteration t at which
 *     a round starts; the last round is cut so that it ends at T.
 *   - Sec. 2 "Dealing with Learning Rate Warmup": a round that starts inside
 *     the warm-up uses the H of the round right after the warm-up.
 *   - App. C: OPT is SGD with momentum and weight decay (ResNet recipe) or
 *     AdamW (ViT recipe).  The paper never writes OPT out; the update rules
 *     here are the textbook ones (heavy-ball momentum with coupled L2 decay;
 *     Adam with decoupled decay and bias correction).
 *
 * Arithmetic: everything in IEEE double.  Synthetic *data* (gradient noise,
 * input features, observation noise) are defined as fp32 values: they are
 * computed in double and rounded once to float, because the workload defines
 * them as single-precision numbers.  Random draws come from Philox4x32-10
 * (Salmon, Moraes, Dror, Shaw, SC'11), implemented here from its published
 * definition, keyed (seed; group index, stream, worker, iteration).
 *
 * Parity pins (tests/test_oracle_*.py): Eq. (2) by hand, the communication
 * volumes printed in Tables 1-3 and 6(a), Philox known-answer vectors, closed
 * forms of the optimizers, library autograd / library optimizers for special
 * cases, H=1 == minibatch SGD, K=1 == serial, brute force on tiny sizes.
 * The residual-MLP model has no value printed by the paper: its gradient is
 * pinned by library autograd and finite differences only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include "qsr_oracle.h"

#define QSRO_PI 3.14159265358979323846

/* ------------------------------------------------------------------ */
/* Learning-rate schedules (Sec. 4 "Training Setup": cosine decay with  */
/* linear warm-up from 0; step decay divides by a factor at milestones) */
/* ------------------------------------------------------------------ */

/* eta_t = eta_max * t / T_warm                          for t <  T_warm
 * eta_t = eta_min + (eta_max-eta_min)/2 * (1+cos(pi*(t-T_warm)/(T-T_warm)))
 *                                                       for t >= T_warm   */
void qsro_lr_cosine(int64_t T, int64_t T_warm, double eta_max, double eta_min,
                    double *eta)
{
    for (int64_t t = 0; t < T; ++t) {
        if (t < T_warm) {
            eta[t] = eta_max * (double)t / (double)T_warm;
        } else {
            double frac = (double)(t - T_warm) / (double)(T - T_warm);
            eta[t] = eta_min + 0.5 * (eta_max - eta_min) * (1.0 + cos(QSRO_PI * frac));
        }
    }
}

/* Linear decay (Sec. 4.1): eta_t = eta_max - (eta_max - eta_min) * (t-T_warm)/(T-T_warm) after
 * the same linear warm-up. */
void qsro_lr_linear(int64_t T, int64_t T_warm, double eta_max, double eta_min, double *eta)
{
    for (int64_t t = 0; t < T; ++t) {
        if (t < T_warm) {
            eta[t] = eta_max * (double)t / (double)T_warm;
        } else {
            double frac = (double)(t - T_warm) / (double)(T - T_warm);
            eta[t] = eta_max - (eta_max - eta_min) * frac;
        }
    }
}

/* The step schedule the paper derives from the cosine one (Sec. 4.1):
 * eta_step(t) = 2^round(log2(eta_cos(t))). */
void qsro_lr_pow2cos(int64_t T, int64_t T_warm, double eta_max, double eta_min, double *eta)
{
    qsro_lr_cosine(T, T_warm, eta_max, eta_min, eta);
    for (int64_t t = T_warm; t < T; ++t)
        if (eta[t] > 0.0) eta[t] = exp2(round(log2(eta[t])));
}

/* eta_t = eta_max / factor^j, j = number of milestones m with m <= t
 * (after the same linear warm-up). */
void qsro_lr_step(int64_t T, int64_t T_warm, double eta_max, int32_t n_ms,
                  const int64_t *ms, double factor, double *eta)
{
    for (int64_t t = 0; t < T; ++t) {
        if (t < T_warm) {
            eta[t] = eta_max * (double)t / (double)T_warm;
            continue;
        }
        double div = 1.0;
        for (int32_t i = 0; i < n_ms; ++i)
            if (ms[i] <= t) div = div * factor;
        eta[t] = eta_max / div;
    }
}

/* ------------------------------------------------------------------ */
/* QSR scheduler, Eq. (2) with the truncation and warm-up rules         */
/* ------------------------------------------------------------------ */

/* Synchronization period of the round whose first local step is global
 * iteration t.  gamma is the power (2 for QSR; Sec. 2 also names the general
 * power rule, App. F the cubic one); it is applied by repeated
 * multiplication, never by pow(). */
int64_t qsro_get_H_power(const double *eta, int64_t T, int64_t T_warm, int64_t t,
                         int64_t H_base, double alpha, int32_t gamma)
{
    int64_t rem = T - t;                       /* steps left in the schedule   */
    int64_t te = t < T_warm ? T_warm : t;      /* warm-up: look past it        */
    if (te >= T) return rem;
    double e = eta[te];
    if (!(e > 0.0)) return rem;                /* eta -> 0: one last round     */
    double q = alpha / e;
    double v = q;
    for (int32_t i = 1; i < gamma; ++i) v = v * q;
    if (!(v < (double)rem)) return rem;        /* forced sync at the last step */
    int64_t H = (int64_t)floor(v);
    if (H < H_base) H = H_base;
    if (H > rem) H = rem;                      /* H_base itself may overshoot  */
    return H;
}

int64_t qsro_get_H(const double *eta, int64_t T, int64_t T_warm, int64_t t,
                   int64_t H_base, double alpha)
{
    return qsro_get_H_power(eta, T, T_warm, t, H_base, alpha, 2);
}

/* The rule of a configured run: power rule (gamma = 0: constant H_base), preceded by the
 * post-local phase of Lin et al. (Sec. 1, Sec. 4 "Comparison with other synchronization
 * strategies"): H = 1 for rounds that start before t_local_start; and followed, if asked, by
 * the modified SWAP phase of App. G: from t_swap_start on, local steps only and one final
 * averaging. */
static int64_t run_get_H(const qsro_config *c, const double *eta, int64_t t)
{
    if (c->t_swap_start > 0 && t >= c->t_swap_start) return c->T - t;
    if (t < c->t_local_start) return 1;
    if (c->power == 0) {
        int64_t rem = c->T - t;
        return c->H_base < rem ? c->H_base : rem;
    }
    return qsro_get_H_power(eta, c->T, c->T_warm, t, c->H_base, c->alpha, c->power);
}

/* Whole-run schedule: writes H^(s) and the iteration count after which each
 * averaging runs; returns the number of rounds (also when it exceeds cap). */
int64_t qsro_schedule(const double *eta, int64_t T, int64_t T_warm, int64_t H_base,
                      double alpha, int32_t gamma, int64_t *H_out, int64_t *sync_t,
                      int64_t cap)
{
    int64_t t = 0, s = 0;
    while (t < T) {
        int64_t H = qsro_get_H_power(eta, T, T_warm, t, H_base, alpha, gamma);
        t += H;
        if (s < cap) {
            if (H_out) H_out[s] = H;
            if (sync_t) sync_t[s] = t;
        }
        ++s;
    }
    return s;
}

/* ------------------------------------------------------------------ */
/* Philox4x32-10 and the normal / integer draws built on it             */
/* ------------------------------------------------------------------ */

void qsro_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;                     /* key schedule between rounds */
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* streams (second counter word) */
enum { QSRO_STREAM_GRAD = 0, QSRO_STREAM_X = 1, QSRO_STREAM_NOISE = 2, QSRO_STREAM_LABEL = 3 };

static void draw4(uint64_t seed, uint32_t stream, uint32_t k, uint64_t t, uint64_t group,
                  uint32_t r[4])
{
    uint32_t ctr[4] = { (uint32_t)group, stream, k, (uint32_t)t };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    qsro_philox4x32_10(ctr, key, r);
}

/* Box-Muller on one pair of words: u1 = ((a>>9)+1/2) 2^-23 in (0,1),
 * u2 = (b>>8) 2^-24 in [0,1); both are exact in single precision. */
static void box_muller(uint32_t a, uint32_t b, double *za, double *zb)
{
    double u1 = ((double)(a >> 9) + 0.5) * (1.0 / 8388608.0);
    double u2 = (double)(b >> 8) * (1.0 / 16777216.0);
    double rad = sqrt(-2.0 * log(u1));
    double ang = 2.0 * QSRO_PI * u2;
    *za = rad * cos(ang);
    *zb = rad * sin(ang);
}

/* The four standard normals of group `group` (elements 4*group .. 4*group+3),
 * each rounded once to single precision. */
void qsro_normal4(uint64_t seed, uint32_t stream, uint32_t k, uint64_t t, uint64_t group,
                  float z[4])
{
    uint32_t r[4];
    double a, b;
    draw4(seed, stream, k, t, group, r);
    box_muller(r[0], r[1], &a, &b); z[0] = (float)a; z[1] = (float)b;
    box_muller(r[2], r[3], &a, &b); z[2] = (float)a; z[3] = (float)b;
}

/* standard normal number `e` of a stream */
static float normal_at(uint64_t seed, uint32_t stream, uint32_t k, uint64_t t, uint64_t e)
{
    float z[4];
    qsro_normal4(seed, stream, k, t, e >> 2, z);
    return z[e & 3];
}

/* integer in [0, n) number `e` of a stream: high word of r * n */
static uint32_t index_at(uint64_t seed, uint32_t stream, uint32_t k, uint64_t t, uint64_t e,
                         uint32_t n)
{
    uint32_t r[4];
    draw4(seed, stream, k, t, e >> 2, r);
    return (uint32_t)(((uint64_t)r[e & 3] * (uint64_t)n) >> 32);
}

/* ------------------------------------------------------------------ */
/* OPT: one step on one worker's vector (Alg. 2, the OPT(.) line)       */
/* ------------------------------------------------------------------ */

/* SGD with heavy-ball momentum mu and coupled weight decay lambda:
 *   g' = g + lambda*theta ; buf = mu*buf + g' ; theta = theta - eta*buf   */
void qsro_sgdm_step(double *theta, double *buf, const double *g, int64_t n,
                    double eta, double mu, double lambda)
{
    for (int64_t i = 0; i < n; ++i) {
        double gp = g[i] + lambda * theta[i];
        buf[i] = mu * buf[i] + gp;
        theta[i] = theta[i] - eta * buf[i];
    }
}

/* AdamW, step number `step` (1-based, counts global iterations):
 *   m = b1 m + (1-b1) g ; v = b2 v + (1-b2) g^2
 *   mhat = m/(1-b1^step) ; vhat = v/(1-b2^step)
 *   theta = theta - eta*lambda*theta - eta * mhat/(sqrt(vhat)+eps)        */
void qsro_adamw_step(double *theta, double *m, double *v, const double *g, int64_t n,
                     double eta, double b1, double b2, double eps, double lambda,
                     int64_t step)
{
    double bc1 = 1.0 - pow(b1, (double)step);
    double bc2 = 1.0 - pow(b2, (double)step);
    for (int64_t i = 0; i < n; ++i) {
        m[i] = b1 * m[i] + (1.0 - b1) * g[i];
        v[i] = b2 * v[i] + (1.0 - b2) * g[i] * g[i];
        double mhat = m[i] / bc1;
        double vhat = v[i] / bc2;
        theta[i] = theta[i] - eta * lambda * theta[i] - eta * mhat / (sqrt(vhat) + eps);
    }
}

/* theta_bar = (1/K) sum_k theta_k, written back to every worker
 * (Alg. 2, the All-Reduce line). theta is [K][n]. */
void qsro_average(double *theta, int32_t K, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int32_t k = 0; k < K; ++k) s += theta[(int64_t)k * n + i];
        double mean = s / (double)K;
        for (int32_t k = 0; k < K; ++k) theta[(int64_t)k * n + i] = mean;
    }
}

/* ------------------------------------------------------------------ */
/* Workloads: Sample() and the local gradient of Eq. (1)                */
/* ------------------------------------------------------------------ */


/* model 1: g_p = fl32(sigma * z_p), z from stream GRAD keyed (k, t, p/4) */
void qsro_grad_noise(const qsro_config *c, int32_t k, int64_t t, double *g)
{
    float sig = (float)c->grad_sigma;
    for (int64_t i = 0; i < c->n; ++i) {
        uint64_t p = c->p_idx ? (uint64_t)c->p_idx[i] : (uint64_t)i;
        float z = normal_at(c->seed, QSRO_STREAM_GRAD, (uint32_t)k, (uint64_t)t, p);
        g[i] = (double)(sig * z);
    }
}

/* model 2 batch: X[i][j] = z(stream X, i*d+j); y_i = X_i . w* + sigma z(stream NOISE, i) */
void qsro_linreg_batch(const qsro_config *c, int32_t k, int64_t t, double *X, double *y)
{
    int64_t B = c->B_loc, d = c->d_in;
    float sig = (float)c->data_sigma;
    for (int64_t i = 0; i < B; ++i) {
        double acc = 0.0;
        for (int64_t j = 0; j < d; ++j) {
            double x = (double)normal_at(c->seed, QSRO_STREAM_X, (uint32_t)k, (uint64_t)t,
                                         (uint64_t)(i * d + j));
            X[i * d + j] = x;
            acc += x * (double)c->model_const[j];
        }
        double e = (double)normal_at(c->seed, QSRO_STREAM_NOISE, (uint32_t)k, (uint64_t)t,
                                     (uint64_t)i);
        y[i] = acc + (double)sig * e;
    }
}

/* model 2: loss = 1/(2B) sum_i (x_i.w - y_i)^2 ; g = (1/B) sum_i (x_i.w - y_i) x_i */
double qsro_grad_linreg(const qsro_config *c, int32_t k, int64_t t, const double *w, double *g)
{
    int64_t B = c->B_loc, d = c->d_in;
    double *X = (double *)malloc(sizeof(double) * (size_t)(B * d));
    double *y = (double *)malloc(sizeof(double) * (size_t)B);
    qsro_linreg_batch(c, k, t, X, y);
    for (int64_t j = 0; j < d; ++j) g[j] = 0.0;
    double loss = 0.0;
    for (int64_t i = 0; i < B; ++i) {
        double r = 0.0;
        for (int64_t j = 0; j < d; ++j) r += X[i * d + j] * w[j];
        r -= y[i];
        loss += 0.5 * r * r;
        for (int64_t j = 0; j < d; ++j) g[j] += r * X[i * d + j];
    }
    for (int64_t j = 0; j < d; ++j) g[j] /= (double)B;
    free(X); free(y);
    return loss / (double)B;
}

/* model 3 batch: label_i = floor(r * C / 2^32) from stream LABEL;
 * x_i = mean[label_i] + sigma * z(stream X, i*d_in + j) */
void qsro_mlp2_batch(const qsro_config *c, int32_t k, int64_t t, double *X, int32_t *label)
{
    int64_t B = c->B_loc, d = c->d_in;
    float sig = (float)c->data_sigma;
    for (int64_t i = 0; i < B; ++i) {
        uint32_t cl = index_at(c->seed, QSRO_STREAM_LABEL, (uint32_t)k, (uint64_t)t,
                               (uint64_t)i, (uint32_t)c->d_out);
        label[i] = (int32_t)cl;
        for (int64_t j = 0; j < d; ++j) {
            float z = normal_at(c->seed, QSRO_STREAM_X, (uint32_t)k, (uint64_t)t,
                                (uint64_t)(i * d + j));
            /* the input is a single-precision datum: mean + sigma*z rounded once */
            X[i * d + j] = (double)(float)((double)c->model_const[(int64_t)cl * d + j]
                                           + (double)sig * (double)z);
        }
    }
}

/* model 3: two-layer perceptron, parameters packed as
 *   W1 [d_in][d_hidden], b1 [d_hidden], W2 [d_hidden][d_out], b2 [d_out];
 * hidden = relu(x W1 + b1); logits = hidden W2 + b2;
 * loss = mean_i ( logsumexp(logits_i) - logits_i[label_i] ). */
double qsro_grad_mlp2(const qsro_config *c, int32_t k, int64_t t, const double *th, double *g)
{
    int64_t B = c->B_loc, di = c->d_in, dh = c->d_hidden, dz = c->d_out;
    const double *W1 = th, *b1 = W1 + di * dh, *W2 = b1 + dh, *b2 = W2 + dh * dz;
    double *gW1 = g, *gb1 = gW1 + di * dh, *gW2 = gb1 + dh, *gb2 = gW2 + dh * dz;
    double *X = (double *)malloc(sizeof(double) * (size_t)(B * di));
    int32_t *label = (int32_t *)malloc(sizeof(int32_t) * (size_t)B);
    double *hid = (double *)malloc(sizeof(double) * (size_t)dh);
    double *dhid = (double *)malloc(sizeof(double) * (size_t)dh);
    double *lg = (double *)malloc(sizeof(double) * (size_t)dz);
    qsro_mlp2_batch(c, k, t, X, label);
    for (int64_t i = 0; i < c->n; ++i) g[i] = 0.0;
    double loss = 0.0;
    for (int64_t s = 0; s < B; ++s) {
        const double *x = X + s * di;
        for (int64_t j = 0; j < dh; ++j) hid[j] = b1[j];
        for (int64_t i = 0; i < di; ++i)
            for (int64_t j = 0; j < dh; ++j) hid[j] += x[i] * W1[i * dh + j];
        for (int64_t j = 0; j < dh; ++j) if (hid[j] < 0.0) hid[j] = 0.0;
        for (int64_t o = 0; o < dz; ++o) lg[o] = b2[o];
        for (int64_t j = 0; j < dh; ++j)
            for (int64_t o = 0; o < dz; ++o) lg[o] += hid[j] * W2[j * dz + o];
        double mx = lg[0];
        for (int64_t o = 1; o < dz; ++o) if (lg[o] > mx) mx = lg[o];
        double se = 0.0;
        for (int64_t o = 0; o < dz; ++o) se += exp(lg[o] - mx);
        loss += (mx + log(se)) - lg[label[s]];
        /* dlogits = softmax - onehot */
        for (int64_t o = 0; o < dz; ++o)
            lg[o] = exp(lg[o] - mx) / se - (o == label[s] ? 1.0 : 0.0);
        for (int64_t o = 0; o < dz; ++o) gb2[o] += lg[o];
        for (int64_t j = 0; j < dh; ++j) {
            double a = 0.0;
            for (int64_t o = 0; o < dz; ++o) {
                gW2[j * dz + o] += hid[j] * lg[o];
                a += W2[j * dz + o] * lg[o];
            }
            dhid[j] = hid[j] > 0.0 ? a : 0.0;   /* relu'(0) = 0 */
            gb1[j] += dhid[j];
        }
        for (int64_t i = 0; i < di; ++i)
            for (int64_t j = 0; j < dh; ++j) gW1[i * dh + j] += x[i] * dhid[j];
    }
    for (int64_t i = 0; i < c->n; ++i) g[i] /= (double)B;
    free(X); free(label); free(hid); free(dhid); free(lg);
    return loss / (double)B;
}

/* model 4 (residual MLP stack) lives in qsr_oracle_resmlp.c */

/* ------------------------------------------------------------------ */
/* Alg. 2 driver                                                        */
/* ------------------------------------------------------------------ */


/* Advance the run by n_steps global iterations.  theta/st0/st1 are [K][n]
 * (st1 unused for SGD).  ext_g, for model 0, is [n_steps][K][n].
 * Averaging runs right after the H-th local step of a round; H_log[s] and
 * sync_log[s] receive H^(s) and the iteration count at that moment.
 * loss_out, if not NULL, is [n_steps][K] (models 2-4).
 * Returns 0, or -1 on a step past T or a bad model id. */
/* Gradient clipping by global norm, one worker's gradient (App. C, "gradient clipping": threshold
 * 1 for parallel AdamW, 4 for Local AdamW with constant H in the linear / step-decay runs, off in
 * the QSR runs):  g <- g * min(1, c / (||g||_2 + 1e-6)), the convention of the framework the
 * paper trained with.  Returns the norm before clipping. */
double qsro_clip(double *g, int64_t n, double max_norm)
{
    double ss = 0.0;
    for (int64_t i = 0; i < n; ++i) ss += g[i] * g[i];
    double norm = sqrt(ss);
    double coef = max_norm / (norm + 1e-6);
    if (coef < 1.0)
        for (int64_t i = 0; i < n; ++i) g[i] *= coef;
    return norm;
}

int qsro_run(const qsro_config *c, const double *eta, qsro_state *st, double *theta,
             double *st0, double *st1, int64_t n_steps, const double *ext_g,
             int64_t *H_log, int64_t *sync_log, int64_t log_cap, double *loss_out)
{
    int32_t K = c->K;
    int64_t n = c->n;
    double *gbuf = NULL, *gavg = NULL, *gclip = NULL;
    if (c->model != 0) gbuf = (double *)malloc(sizeof(double) * (size_t)K * (size_t)n);
    int rc = 0;
    for (int64_t it = 0; it < n_steps; ++it) {
        if (st->t >= c->T || c->model < 0 || c->model > 4) { rc = -1; break; }
        if (st->H == 0) {                          /* a round starts at st->t */
            st->H = run_get_H(c, eta, st->t);
            if (H_log && st->s < log_cap) H_log[st->s] = st->H;
        }
        int64_t t = st->t;
#ifdef _OPENMP
#pragma omp parallel for num_threads(c->n_threads > 0 ? c->n_threads : 1) schedule(static)
#endif
        for (int32_t k = 0; k < K; ++k) {          /* "for each worker in parallel" */
            double *th = theta + (int64_t)k * n;
            double loss = 0.0;
            if (c->model != 0) {
                double *gk = gbuf + (int64_t)k * n;
                if (c->model == 1) qsro_grad_noise(c, k, t, gk);
                else if (c->model == 2) loss = qsro_grad_linreg(c, k, t, th, gk);
                else if (c->model == 3) loss = qsro_grad_mlp2(c, k, t, th, gk);
                else loss = qsro_grad_resmlp(c, k, t, th, gk);
            }
            if (loss_out) loss_out[it * K + k] = loss;
        }
        const double *gall = c->model == 0 ? ext_g + (int64_t)it * K * n : gbuf;
        if (c->parallel) {                         /* Alg. 1: All-Reduce of the local gradients */
            if (!gavg) gavg = (double *)malloc(sizeof(double) * (size_t)K * (size_t)n);
            memcpy(gavg, gall, sizeof(double) * (size_t)K * (size_t)n);
            qsro_average(gavg, K, n);
            gall = gavg;
        }
        if (c->clip_norm > 0.0) {                  /* clipping sits between the gradient and OPT */
            if (!gclip) gclip = (double *)malloc(sizeof(double) * (size_t)K * (size_t)n);
            memcpy(gclip, gall, sizeof(double) * (size_t)K * (size_t)n);
            for (int32_t k = 0; k < K; ++k) qsro_clip(gclip + (int64_t)k * n, n, c->clip_norm);
            gall = gclip;
        }
#ifdef _OPENMP
#pragma omp parallel for num_threads(c->n_threads > 0 ? c->n_threads : 1) schedule(static)
#endif
        for (int32_t k = 0; k < K; ++k) {
            double *th = theta + (int64_t)k * n;
            const double *g = gall + (int64_t)k * n;
            if (c->opt == 0)
                qsro_sgdm_step(th, st0 + (int64_t)k * n, g, n, eta[t], c->mu, c->lambda);
            else
                qsro_adamw_step(th, st0 + (int64_t)k * n, st1 + (int64_t)k * n, g, n, eta[t],
                                c->beta1, c->beta2, c->eps, c->lambda, t + 1);
        }
        st->t += 1;
        st->h += 1;
        if (st->h == st->H) {
            qsro_average(theta, K, n);
            if (c->average_state) {
                qsro_average(st0, K, n);
                if (c->opt == 1) qsro_average(st1, K, n);
            }
            if (sync_log && st->s < log_cap) sync_log[st->s] = st->t;
            st->s += 1;
            st->h = 0;
            st->H = 0;
        }
    }
    free(gbuf);
    free(gavg);
    free(gclip);
    return rc;
}
