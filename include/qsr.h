/*
 * qsr.h -- C ABI of the MI355X (gfx950) library for Local SGD / Local AdamW with the
 * Quadratic Synchronization Rule (arXiv 2310.14423).
 *
 * K simulated workers are held on ONE GPU as replica-stacked row-major buffers [K][P]
 * (worker k owns elements k*P .. k*P+P-1).  One global iteration of Alg. 2 (Local OPT) is
 *
 *     qsr_local_step   -- every worker's local gradient (Eq. (1)) and its OPT update
 *     qsr_maybe_sync   -- if the round's H-th local step has just run: parameter averaging
 *                         (the All-Reduce line of Alg. 2) and the next round's H from
 *                         Eq. (2), H = max{H_base, floor((alpha/eta_t)^2)}
 *     qsr_run          -- n such iterations in one call
 *
 * The scheduler state (t, s, h, H), the learning-rate table and the log of averaging
 * points live in device memory; the two calls above only enqueue kernels on the caller's
 * stream and never synchronise.  The host keeps a mirror of the four integers, advanced with the
 * same arithmetic from the same table, which only decides which kernels are enqueued for an
 * iteration (an averaging kernel where a round ends; where none ends, the update kernel may carry the
 * scheduler's counting step instead of a launch of its own); the device takes every decision again,
 * logs the rounds, and any disagreement
 * between the two is reported as QSR_EMIRROR by the calls that read the state.  All `float*` / `void*` buffer arguments are DEVICE
 * pointers unless marked (host); they stay owned by the caller, who must keep them alive
 * and untouched by other streams until qsr_destroy.  The library allocates only its own
 * small scheduler tables.  Every function returns QSR_OK (0) or a negative QSR_E* code;
 * nothing throws or aborts across this boundary.  Argument checks happen on the host
 * before any GPU work.  A context is not thread-safe.
 */
#ifndef QSR_H
#define QSR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct qsr_ctx qsr_ctx; /* opaque, library-owned */

enum {
    QSR_OK = 0,
    QSR_EINVAL = -1,   /* bad argument or configuration                                 */
    QSR_ESTATE = -2,   /* call out of protocol (e.g. a local step after iteration T)    */
    QSR_EHIP = -3,     /* a HIP runtime call failed; qsr_last_hip_error() has its code  */
    QSR_ENOMEM = -4,   /* workspace too small / allocation failed                       */
    QSR_ENOGPU = -5,   /* no usable gfx950 device                                       */
    QSR_EMIRROR = -6,  /* the host's mirror of the schedule and the device scheduler took
                          different decisions (a defect: results after it are not Alg. 2's) */
    QSR_ELIMIT = -7    /* size beyond the fixed capacity of an entry point that allocates nothing */
};

enum { QSR_OPT_SGDM = 0, QSR_OPT_ADAMW = 1 };
enum {
    QSR_LR_COSINE = 0,  /* cosine decay eta_max -> eta_min (Sec. 4 "Training Setup")              */
    QSR_LR_STEP = 1,    /* eta_max divided by step_factor at each milestone                       */
    QSR_LR_TABLE = 2,   /* caller-supplied table                                                  */
    QSR_LR_LINEAR = 3,  /* linear decay eta_max -> eta_min (Sec. 4.1 "Other learning rate
                           schedules")                                                            */
    QSR_LR_POW2COS = 4  /* the step schedule the paper derives from the cosine one:
                           2^round(log2(eta_cos(t))) (Sec. 4.1)                                   */
};
enum {
    QSR_MODEL_EXTERNAL = 0, /* caller writes `grads` before each qsr_local_step          */
    QSR_MODEL_NOISE = 1,    /* g = grad_sigma * N(0,1), optimizer-only workloads          */
    QSR_MODEL_LINREG = 2,   /* linear least squares, P = d_in                             */
    QSR_MODEL_MLP2 = 3,     /* d_in - d_hidden - d_out perceptron, ReLU, softmax CE       */
    QSR_MODEL_RESMLP = 4    /* n_blocks pre-LN residual MLP blocks (optionally each with its
                               attention sub-block, see n_heads), bf16 GEMMs              */
};

/* Plain-data configuration (Alg. 2's inputs and hyper-parameters, Eq. (2)'s alpha and H_base,
 * OPT's hyper-parameters per App. C).  Pointers inside are HOST pointers, read during
 * qsr_init only. */
typedef struct {
    int32_t K;            /* workers (replica rows), >= 1                                  */
    int32_t opt;          /* QSR_OPT_*                                                     */
    int32_t model;        /* QSR_MODEL_*                                                   */
    int32_t lr_kind;      /* QSR_LR_*                                                      */
    int32_t H_base;       /* minimum synchronization period, >= 1 (Eq. (2))                */
    int32_t n_milestones; /* QSR_LR_STEP: entries of `milestones`                          */
    int32_t n_blocks;     /* QSR_MODEL_RESMLP                                              */
    int32_t power;        /* exponent gamma of H = max{H_base, floor((alpha/eta_t)^gamma)}:
                             2 = QSR (Eq. (2)); 1 = the H ~ 1/eta rule and 3 = the cubic rule the
                             paper compares with (Sec. 2, App. F; alpha then plays beta / rho);
                             0 = constant H = H_base (conventional Local OPT)               */
    int32_t parallel;     /* 1 = Parallel OPT (Alg. 1): the K local gradients are averaged every
                             step before OPT, so all workers take the same update; every step
                             counts as a round.  Needs H_base = 1, power = 0.  0 = Local OPT  */
    int32_t average_state;/* 0: optimizer state stays local at a synchronization, as in Alg. 2, which
                             averages the model parameters only; 1: the state buffers (momentum /
                             m, v) are averaged with them                                   */
    int32_t fuse_sync;    /* 1: the local step that completes a round also averages (one pass over
                             the buffers: 28 B per replica-parameter for AdamW on that step instead
                             of 28 + 8); qsr_maybe_sync then only opens the next round.  Same
                             results bit for bit.  Not with parallel or average_state.  0 = off */
    int32_t n_heads;      /* QSR_MODEL_RESMLP: > 0 puts a multi-head self-attention sub-block (heads of
                             width 64, so d_in = 64 n_heads) in front of every MLP sub-block: the
                             encoder block of the paper's ViT-B (App. C.2).  0 = MLP sub-blocks only */
    int32_t fuse_gradient;/* QSR_MODEL_NOISE: the gradient is drawn inside the update kernel: one pass instead
                             of a fill and an update, parameters and optimizer state the same bit for
                             bit.  1 = the draw is also written to `grads` (28 B per replica-parameter as
                             before); 2 = `grads` is left untouched, the gradient never exists in memory
                             (24 B).  Needs P % 4 == 0; not with parallel, fuse_sync or clip_norm.
                             0 = off                                                          */
    int32_t reserved;     /* must be 0                                                    */
    int64_t P;            /* parameters per worker, >= 1                                   */
    int64_t T;            /* total iterations, eta_t is defined for t in 0..T-1, >= 1      */
    int64_t T_warm;       /* linear warm-up 0 -> eta_max over the first T_warm iterations  */
    int64_t t_local_start;/* post-local schedule (Sec. 1): rounds that start before this
                             iteration use H = 1; 0 = off                                  */
    int64_t t_swap_start; /* Local OPT + SWAP (App. G): a round that starts at or after this
                             iteration runs to the end of training, with one final averaging;
                             0 = off                                                        */
    int64_t B_loc;        /* local batch: samples (RESMLP: tokens) per worker per step     */
    int64_t d_in, d_hidden, d_out;
    int64_t seq_len;      /* n_heads > 0: tokens per sequence, 1..224, dividing B_loc; attention
                             acts within runs of seq_len consecutive tokens                */
    double momentum;      /* SGD heavy-ball coefficient                                    */
    double beta1, beta2, eps; /* AdamW                                                     */
    double weight_decay;  /* SGD: coupled (added to the gradient); AdamW: decoupled        */
    double eta_max, eta_min;  /* peak; floor of the cosine / linear / pow2cos decays            */
    double step_factor;   /* QSR_LR_STEP: eta = eta_max / step_factor^(#milestones <= t)   */
    double alpha;         /* growth coefficient of Eq. (2); 0 gives constant H = H_base    */
    double grad_sigma;    /* QSR_MODEL_NOISE: standard deviation of the gradient           */
    double data_sigma;    /* LINREG: observation noise; MLP2: input noise                  */
    double clip_norm;     /* > 0: gradient clipping by global norm, per worker, before OPT (App. C):
                             g_k <- g_k * min(1, clip_norm / (||g_k||_2 + 1e-6)); with parallel = 1
                             it acts on the averaged gradient.  0 = off                     */
    uint64_t seed;        /* Philox4x32-10 key of all per-iteration draws                  */
    const int64_t *milestones; /* (host) ascending iteration indices, QSR_LR_STEP          */
    const double *eta_table;   /* (host) T entries, QSR_LR_TABLE                           */
    void *stream;         /* hipStream_t all work is enqueued on (NULL = default stream)   */
} qsr_config;

/* Checks a configuration on the host (no GPU needed).  QSR_OK or QSR_EINVAL;
 * *why, if given, receives a static string naming the offending field. */
int qsr_validate(const qsr_config *cfg, const char **why);

/* Bytes of device workspace qsr_init needs for this configuration (activations, batches,
 * bf16 weight copies).  0 for the EXTERNAL and NOISE models.  QSR_EINVAL on a bad config. */
int qsr_workspace_bytes(const qsr_config *cfg, size_t *bytes);

/* The whole schedule of a configuration, computed on the host alone (no GPU): Eq. (2) with the
 * truncation and warm-up rules of Sec. 2 (and the variants `power`, `t_local_start`,
 * `t_swap_start` select) on the configuration's learning-rate table.  t_out[i] = iteration count
 * after which averaging i runs, H_out[i] = that round's period; writes min(*n, cap) entries, *n =
 * number of rounds (communication volume relative to Parallel OPT = *n / T, App. F).  It is the
 * routine the context's mirror uses; the device-side scheduler, which runs must match, is a
 * separate implementation. */
int qsr_host_schedule(const qsr_config *cfg, int64_t *t_out, int64_t *H_out, int64_t cap, int64_t *n);

/* Creates a context.  Alg. 2's initialisation: copies theta0 [P] into each of the K rows
 * of `params`, zeroes the optimizer state, sets t = s = h = 0 and computes H^(0).
 *   params, grads, state0 : [K][P] float, 16-byte aligned; state1 likewise for AdamW
 *                           (second moment), NULL for SGD.  state0 = momentum buffer / m.
 *   theta0                : [P] float, or NULL to keep what `params` holds.
 *   model_const           : LINREG w* [d_in]; MLP2 class means [d_out][d_in];
 *                           RESMLP teacher [d_in][d_in]; else NULL.  Borrowed like the rest.
 *   workspace             : at least qsr_workspace_bytes() bytes, 256-byte aligned, or NULL
 *                           when that is 0.
 * Synchronises the stream once.  On failure *out is NULL. */
int qsr_init(const qsr_config *cfg, float *params, float *grads, float *state0, float *state1,
             const float *theta0, const float *model_const, void *workspace,
             size_t workspace_bytes, qsr_ctx **out);

/* One global iteration for all K workers: local gradients at each worker's own parameters
 * (Eq. (1)) unless the model is EXTERNAL, then the fused OPT update with eta_t (Alg. 2's
 * inner loop body), then t += 1, h += 1.  Asynchronous.  QSR_ESTATE once T steps have run
 * or when the previous step's qsr_maybe_sync is missing. */
int qsr_local_step(qsr_ctx *ctx);

/* If h == H^(s): theta_k <- (1/K) sum_k theta_k for every k, the pair (t, H^(s)) is appended
 * to the log, s += 1, h = 0 and H^(s+1) follows from Eq. (2) at the new t (cut to T - t;
 * warm-up rule of Sec. 2).  Otherwise nothing changes.  The decision is taken on the device.
 * Asynchronous. */
int qsr_maybe_sync(qsr_ctx *ctx);

/* n global iterations of Alg. 2, each a qsr_local_step followed by its qsr_maybe_sync, with the
 * same results bit for bit.  Every kernel reads t, h, H and the averaging decision from device
 * memory, so the launches of an iteration do not depend on t: on a stream other than the null
 * stream, with qsr_timing off and n large enough to pay for it, they are recorded once into a
 * HIP graph (kernel nodes only) that is replayed, which removes most of the launch cost of the
 * short iterations of small models; otherwise the iterations are enqueued one by one.
 * Asynchronous.  n >= 0; QSR_ESTATE if a qsr_maybe_sync is pending or fewer than n iterations
 * are left before T. */
int qsr_run(qsr_ctx *ctx, int64_t n);

/* Synchronises the stream and reads the scheduler state: period of the current round (0 once
 * t == T), number of finished rounds, iteration counter.  Any pointer may be NULL. */
int qsr_get_H(qsr_ctx *ctx, int64_t *H, int64_t *round, int64_t *t);

/* Synchronises and copies the log of finished rounds: t_out[i] = iteration count after which
 * averaging i ran, H_out[i] = that round's period.  Writes min(*n, cap) entries; *n = rounds
 * so far.  t_out / H_out may be NULL. */
int qsr_read_sync_log(qsr_ctx *ctx, int64_t *t_out, int64_t *H_out, int64_t cap, int64_t *n);

/* The rounds the host's mirror of the schedule has counted since qsr_init / qsr_restart (after
 * qsr_set_state: entries of earlier rounds read as 0), in the format of qsr_read_sync_log, which it
 * must equal.  Does not synchronise. */
int qsr_read_host_schedule(qsr_ctx *ctx, int64_t *t_out, int64_t *H_out, int64_t cap, int64_t *n);

/* (host) copy of the learning-rate table eta_0..eta_{T-1} the context uses. */
int qsr_eta_table(qsr_ctx *ctx, double *eta_out, int64_t cap);

/* Synchronises and copies the K per-worker losses of the last local step (models LINREG,
 * MLP2, RESMLP) to the host array loss_out [K]. */
int qsr_read_loss(qsr_ctx *ctx, float *loss_out);

/* Checkpoint / resume of the scheduler.  qsr_get_state synchronises and returns
 * state[0..3] = (t, s, h, H).  qsr_set_state installs such a tuple (asynchronously) in a context
 * of the same configuration whose parameter and optimizer-state buffers the caller has restored;
 * 0 <= t <= T, 0 <= h < H <= T - t + h required (H = 0 allowed only at t == T).  The log entries
 * of rounds finished before the restored state read as 0. */
int qsr_get_state(qsr_ctx *ctx, int64_t state[4]);
int qsr_set_state(qsr_ctx *ctx, const int64_t state[4]);

/* Puts the scheduler back to t = s = h = 0 (H^(0) recomputed, log cleared) without touching
 * parameters or optimizer state.  Asynchronous. */
int qsr_restart(qsr_ctx *ctx);

/* Per-kernel timing with HIP events on the context's stream.  After qsr_timing(ctx, 1) each
 * gradient stage, update kernel and averaging kernel is bracketed by an event pair;
 * qsr_read_timing synchronises, adds up the pairs recorded since the last read and recycles
 * them.  ms[i] / count[i]: 0 = gradient stage, 1 = update kernel, 2 = averaging launches that
 * averaged, 3 = averaging launches that the device-side decision skipped (none when the
 * iterations are enqueued one by one: an averaging kernel is then launched only where a round
 * ends).  With fuse_sync, 2 holds the fused update-and-average launches and 1 the plain updates
 * of the other steps.  Read before qsr_restart: the split of 2 and 3 uses the log of the
 * current run. */
int qsr_timing(qsr_ctx *ctx, int enable);
int qsr_read_timing(qsr_ctx *ctx, double ms[4], int64_t count[4]);
/* The same read with the shortest and the median bracket of each kind as well (0 where count is 0);
 * ms_min and ms_median may be NULL. */
int qsr_read_timing_stats(qsr_ctx *ctx, double ms[4], int64_t count[4], double ms_min[4], double ms_median[4]);

int qsr_destroy(qsr_ctx *ctx);

/* Stateless replica averaging (the All-Reduce line of Alg. 2 / Alg. 1 on any [K][P] buffer):
 * buf_k <- (1/K) sum_k buf_k for every k.  Asynchronous on `stream`. */
int qsr_average_rows(float *buf, int32_t K, int64_t P, void *stream);

/* Stateless gradient clipping factors (App. C: clipping by global norm, per worker) of any [K][P]
 * gradient buffer: coef[k] = min(1, max_norm / (||g_k||_2 + 1e-6)), norm[k] = ||g_k||_2, both DEVICE
 * arrays of K floats; the caller multiplies row k by coef[k] (the update kernels of a context with
 * clip_norm do so as they read the gradient).  workspace: DEVICE memory for the partial sums of
 * squares, qsr_clip_workspace_bytes(K, P) bytes, 8-byte aligned, contents irrelevant before and
 * after.  The sums are deterministic (fixed order).  Asynchronous on `stream`.  QSR_EINVAL on bad
 * arguments (K outside 1..65535, P < 1, max_norm not positive and finite), QSR_ENOMEM if the
 * workspace is too small. */
int qsr_clip_workspace_bytes(int32_t K, int64_t P, size_t *bytes);
int qsr_clip_factors(const float *grads, int32_t K, int64_t P, float max_norm, void *workspace,
                     size_t workspace_bytes, float *coef, float *norm, void *stream);

/* qsr_clip_factors for callers that cannot allocate device memory or bring a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without
 * the workspace, same results bit for bit; the partial sums live in a 512 KiB array inside the
 * library's device image, which every GPU the library runs on holds until the process ends.
 * Limits: K <= 64 (QSR_ELIMIT beyond).  Calls no hipMalloc / hipFree or other allocating routine;
 * the array's address on a device is looked up once, by the first qsr_init or the first call of
 * this function there (make that first call outside a capture).  All calls on one GPU share the
 * array: calls that overlap on one GPU (other streams, other threads) race.  Asynchronous on
 * `stream`. */
int qsr_clip_factors_static(const float *grads, int32_t K, int64_t P, float max_norm, float *coef,
                            float *norm, void *stream);

const char *qsr_strerror(int code);
int qsr_last_hip_error(void); /* hipError_t of the last failed runtime call in this thread */

#ifdef __cplusplus
}
#endif
#endif /* QSR_H */
