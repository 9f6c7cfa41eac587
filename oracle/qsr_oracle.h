/* qsr_oracle.h -- declarations shared by the oracle's own C files.
 * TEST INFRASTRUCTURE: nothing outside oracle/ includes this header. */
#ifndef QSR_ORACLE_H
#define QSR_ORACLE_H
#include <stdint.h>

typedef struct {
    int32_t K;            /* workers                                          */
    int32_t opt;          /* 0 SGD-momentum, 1 AdamW                          */
    int32_t model;        /* 0 external gradients, 1 noise, 2 linear least
                             squares, 3 two-layer MLP, 4 residual MLP stack   */
    int32_t H_base;
    int32_t n_threads;    /* OpenMP threads over the worker loop (>=1)        */
    int32_t n_blocks;     /* model 4                                          */
    int32_t power;        /* exponent of the rule, 2 = QSR (Eq. 2); 1, 3: the
                             variants of Sec. 2 / App. F; 0 = constant H_base    */
    int32_t parallel;     /* 1 = Parallel OPT (Alg. 1): gradients are averaged
                             every step and all workers take the same update  */
    int32_t average_state;/* 1 = the optimizer state is averaged at a sync too
                             (Alg. 2 averages the parameters only: 0)           */
    int32_t n_heads;      /* model 4: attention heads per block, 0 = MLP
                             sub-blocks only                                  */
    int64_t n;            /* tracked parameters per worker (= P, or a sample) */
    int64_t T, T_warm;
    int64_t t_local_start;/* post-local schedule: rounds that start before this
                             iteration have H = 1; 0 = off                     */
    int64_t t_swap_start; /* Local OPT + SWAP (App. G): a round that starts at or
                             after this iteration lasts until T; 0 = off        */
    int64_t B_loc;        /* samples (model 4: tokens) per worker per step    */
    int64_t d_in, d_hidden, d_out;
    int64_t seq_len;      /* model 4 with n_heads > 0: tokens per sequence
                             (divides B_loc)                                  */
    double mu, beta1, beta2, eps, lambda;
    double alpha;
    double grad_sigma;    /* model 1: std of the gradient noise               */
    double data_sigma;    /* model 2: observation noise; model 3: input noise */
    double clip_norm;     /* > 0: each worker's gradient is clipped to this
                             Euclidean norm before OPT (App. C); 0 = off      */
    uint64_t seed;
    const float *model_const; /* model 2: w* [d]; 3: class means [C][d_in];
                                 4: teacher map [d][d]                        */
    const int64_t *p_idx;     /* model 1: global parameter index of each
                                 tracked element, or NULL for 0..n-1          */
} qsro_config;

typedef struct {
    int64_t t;   /* global iteration count so far                     */
    int64_t s;   /* finished rounds                                   */
    int64_t h;   /* local steps done in the current round             */
    int64_t H;   /* period of the current round, 0 = not yet computed */
} qsro_state;

void qsro_normal4(uint64_t seed, uint32_t stream, uint32_t k, uint64_t t, uint64_t group,
                  float z[4]);
double qsro_grad_resmlp(const qsro_config *c, int32_t k, int64_t t, const double *th, double *g);
#endif
