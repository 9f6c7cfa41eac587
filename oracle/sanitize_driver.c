/*
 * sanitize_driver.c -- runs the oracle's routines on small cases under AddressSanitizer and
 * UndefinedBehaviorSanitizer (built and run by tests/test_oracle_sanitize.py).
 *
 * TEST INFRASTRUCTURE, like the rest of oracle/.  Exactly sized heap buffers, so that any read
 * or write past an array, and any signed overflow, misaligned access or bad shift, stops the run.
 * It also repeats three pins on the way (the schedules of the linear-least-squares and MLP
 * workloads from Eq. (2) of arXiv 2310.14423, and "every worker holds the same parameters after
 * an averaging"), so that a sanitized build that computes something else is noticed.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "qsr_oracle.h"

void qsro_lr_cosine(int64_t T, int64_t T_warm, double eta_max, double eta_min, double *eta);
void qsro_lr_linear(int64_t T, int64_t T_warm, double eta_max, double eta_min, double *eta);
void qsro_lr_pow2cos(int64_t T, int64_t T_warm, double eta_max, double eta_min, double *eta);
void qsro_lr_step(int64_t T, int64_t T_warm, double eta_max, int32_t n_ms, const int64_t *ms, double factor,
                  double *eta);
int64_t qsro_schedule(const double *eta, int64_t T, int64_t T_warm, int64_t H_base, double alpha, int32_t gamma,
                      int64_t *H, int64_t *st, int64_t cap);
void qsro_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
double qsro_clip(double *g, int64_t n, double max_norm);
int qsro_run(const qsro_config *c, const double *eta, qsro_state *st, double *theta, double *st0, double *st1,
             int64_t n_steps, const double *ext_g, int64_t *H_log, int64_t *sync_log, int64_t log_cap,
             double *loss_out);

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "sanitize_driver: failed: %s (line %d)\n", #cond, __LINE__); return 1; } } while (0)

static double *doubles(size_t n) { double *p = (double *)calloc(n ? n : 1, sizeof(double)); if (!p) abort(); return p; }

/* one Local-OPT run of model `model` with K workers; returns 0 if all workers agree after the last averaging */
static int run_model(int model, int opt, int K, int64_t n, int64_t T, qsro_config base, const float *mc)
{
    qsro_config c = base;
    c.K = K; c.opt = opt; c.model = model; c.n = n; c.T = T; c.model_const = mc; c.n_threads = 2;
    double *eta = doubles((size_t)T);
    qsro_lr_cosine(T, c.T_warm, 0.01, 0.0, eta);
    double *theta = doubles((size_t)K * n), *s0 = doubles((size_t)K * n), *s1 = doubles((size_t)K * n);
    for (int64_t i = 0; i < (int64_t)K * n; ++i) theta[i] = 0.02 * sin(1.0 + (double)(i % n));
    double *ext = model == 0 ? doubles((size_t)T * K * n) : NULL;
    if (ext) for (int64_t i = 0; i < T * K * n; ++i) ext[i] = cos((double)i);
    int64_t *Hl = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t)), *sl = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t));
    double *loss = doubles((size_t)T * K);
    qsro_state st = {0, 0, 0, 0};
    int rc = qsro_run(&c, eta, &st, theta, s0, s1, T, ext, Hl, sl, T + 1, loss);
    int bad = rc != 0 || st.t != T || st.s < 1 || sl[st.s - 1] != T;
    for (int k = 1; k < K && !bad; ++k) bad = memcmp(theta, theta + (size_t)k * n, sizeof(double) * (size_t)n) != 0;
    for (int64_t i = 0; i < (int64_t)K * n && !bad; ++i) bad = !isfinite(theta[i]);
    free(eta); free(theta); free(s0); free(s1); free(ext); free(Hl); free(sl); free(loss);
    return bad;
}

int main(void)
{
    /* schedules (Eq. (2), truncation, warm-up): the least-squares workload has 28 rounds, the MLP's 307 */
    {
        int64_t T = 256;
        double *eta = doubles((size_t)T);
        int64_t *H = (int64_t *)calloc((size_t)T, sizeof(int64_t)), *st = (int64_t *)calloc((size_t)T, sizeof(int64_t));
        qsro_lr_cosine(T, 0, 0.1, 0.0, eta);
        CHECK(qsro_schedule(eta, T, 0, 2, 0.2, 2, H, st, T) == 28 && H[0] == 4 && H[27] == 62 && st[27] == 256);
        free(eta); free(H); free(st);
        T = 2000;
        eta = doubles((size_t)T);
        H = (int64_t *)calloc((size_t)T, sizeof(int64_t)); st = (int64_t *)calloc((size_t)T, sizeof(int64_t));
        const int64_t ms[2] = {1000, 1500};
        qsro_lr_step(T, 0, 0.8, 2, ms, 10.0, eta);
        CHECK(qsro_schedule(eta, T, 0, 4, 0.25, 2, H, st, T) == 307 && H[249] == 4 && H[250] == 9 && H[306] == 496);
        qsro_lr_linear(T, 100, 0.008, 1e-4, eta);
        CHECK(qsro_schedule(eta, T, 100, 4, 0.0175, 2, H, st, T) > 3);
        qsro_lr_pow2cos(T, 100, 0.008, 1e-6, eta);
        CHECK(qsro_schedule(eta, T, 100, 4, 0.015, 3, H, st, T) > 3);
        CHECK(qsro_schedule(eta, T, 100, 4, 0.015, 2, NULL, NULL, 0) > 3);
        free(eta); free(H); free(st);
    }
    /* the counter-based generator and the normals */
    {
        const uint32_t ctr[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu}, key[2] = {0xffffffffu, 0xffffffffu};
        uint32_t out[4];
        qsro_philox4x32_10(ctr, key, out);
        CHECK(out[0] == 0x408f276du);          /* published known-answer vector of Philox4x32-10 */
        float z[4];
        qsro_normal4(0xffffffffffffffffull, 3u, 0xffffffffu, 0xffffffffull, 0xffffffffull, z);
        CHECK(isfinite(z[0]) && isfinite(z[3]));
    }
    /* clipping */
    {
        double *g = doubles(5);
        for (int i = 0; i < 5; ++i) g[i] = 3.0;
        double nrm = qsro_clip(g, 5, 1.0);
        CHECK(fabs(nrm - sqrt(45.0)) < 1e-12 && fabs(g[0] - 3.0 / (sqrt(45.0) + 1e-6)) < 1e-12);
        free(g);
    }
    /* Alg. 2 on every model, tiny shapes with ragged sizes */
    qsro_config c;
    memset(&c, 0, sizeof c);
    c.H_base = 2; c.power = 2; c.alpha = 0.03; c.mu = 0.9; c.beta1 = 0.9; c.beta2 = 0.999; c.eps = 1e-8;
    c.lambda = 0.01; c.grad_sigma = 1e-3; c.data_sigma = 0.1; c.seed = 7; c.T_warm = 3;
    CHECK(run_model(0, 0, 3, 5, 20, c, NULL) == 0);                 /* external gradients, SGD */
    CHECK(run_model(0, 1, 2, 3, 17, c, NULL) == 0);                 /* external gradients, AdamW */
    CHECK(run_model(1, 1, 3, 7, 19, c, NULL) == 0);                 /* noise gradients */
    {
        qsro_config a = c; a.average_state = 1; a.clip_norm = 0.5;
        CHECK(run_model(1, 1, 3, 6, 15, a, NULL) == 0);
        a = c; a.parallel = 1; a.H_base = 1; a.power = 0;
        CHECK(run_model(1, 0, 3, 6, 9, a, NULL) == 0);
        a = c; a.power = 0; a.H_base = 4; a.t_local_start = 6; a.t_swap_start = 14;
        CHECK(run_model(1, 0, 2, 5, 21, a, NULL) == 0);
    }
    {
        float wstar[5] = {0.3f, -0.2f, 0.1f, 0.5f, -0.4f};
        qsro_config a = c; a.B_loc = 3; a.d_in = 5;
        CHECK(run_model(2, 0, 2, 5, 12, a, wstar) == 0);           /* linear least squares */
    }
    {
        float means[3 * 5];
        for (int i = 0; i < 15; ++i) means[i] = (float)sin(0.7 * i);
        qsro_config a = c; a.B_loc = 7; a.d_in = 5; a.d_hidden = 6; a.d_out = 3; a.data_sigma = 1.0;
        CHECK(run_model(3, 0, 2, 5 * 6 + 6 + 6 * 3 + 3, 10, a, means) == 0);   /* two-layer perceptron */
    }
    {
        float teacher[8 * 8];
        for (int i = 0; i < 64; ++i) teacher[i] = (float)cos(0.3 * i);
        qsro_config a = c; a.B_loc = 6; a.d_in = 8; a.d_hidden = 12; a.n_blocks = 2;
        const int64_t per = 2 * 8 + 8 * 12 + 12 + 12 * 8 + 8;
        CHECK(run_model(4, 1, 2, 2 * per, 6, a, teacher) == 0);    /* residual MLP blocks */
        a.n_heads = 2; a.seq_len = 3;
        const int64_t attn = 2 * 8 + 8 * 24 + 24 + 8 * 8 + 8;
        CHECK(run_model(4, 1, 2, 2 * (per + attn), 6, a, teacher) == 0);   /* with attention sub-blocks */
    }
    printf("sanitize_driver: ok\n");
    return 0;
}
