// qsr_api.hip -- host side of the C ABI declared in include/qsr.h: configuration checks,
// learning-rate and per-step scalar tables (double precision on the host), context life
// cycle, and the launch sequence of one iteration of Alg. 2 (arXiv 2310.14423).
#include <cmath>
#include <cstring>
#include <new>
#include <algorithm>
#include <vector>

#include "qsr_internal.h"

using namespace qsr;

static thread_local int g_last_hip = 0;
void qsr::set_last_hip_error(int code) { g_last_hip = code; (void)hipGetLastError(); }

#define HIP_TRY(expr)                                    \
    do {                                                 \
        hipError_t e_ = (expr);                          \
        if (e_ != hipSuccess) {                          \
            g_last_hip = (int)e_;                        \
            (void)hipGetLastError();                     \
            return QSR_EHIP;                             \
        }                                                \
    } while (0)

struct TimedPair {
    hipEvent_t a, b;
    int kind;            // 0 gradient stage, 1 update, 2 averaging
    long long t_after;   // host iteration counter when recorded (averaging: value of t)
};

struct qsr_ctx {
    qsr_config cfg;
    hipStream_t stream;
    int device;
    float *params, *grads, *state0, *state1;
    const float *model_const;
    void *workspace;
    size_t workspace_bytes;
    // library-owned device memory
    DevState *d_state;       // two copies; `cur` is the one this iteration's kernels read (see fold_tick)
    int cur;
    bool fold_tick;          // the update kernel takes the scheduler's step on iterations that end no round
    bool ticked;             // ... and has done so for the local step whose qsr_maybe_sync is pending
    double *d_eta;
    StepScalars *d_scal;
    long long *d_log_t, *d_log_H;
    float *d_loss;
    double *d_clip_part;     // gradient clipping: partial sums of squares, [K][blocks per row]
    float *d_clip_coef;      // [K] factors, then [K] gradient norms
    // host mirrors
    std::vector<double> eta;
    DevState *h_state;       // pinned
    long long t_host;        // local steps enqueued
    bool need_sync_call;     // a local step was enqueued and its maybe_sync not yet
    // Mirror of the device scheduler's integers (t, s, h, H), advanced on the host with the same
    // arithmetic from the same learning-rate table.  It decides only which kernels are enqueued (an
    // averaging launch where a round ends, none elsewhere); the device state stays the truth: the
    // averaging kernels still test it, the advance kernel compares the two decisions and latches a
    // flag if they ever differ, and every read of the state reports that flag as QSR_EMIRROR.
    long long m_t, m_s, m_h, m_H;
    std::vector<long long> m_log_t, m_log_H;
    bool capturing;          // launches are being recorded into a graph: device-side decisions only
    SchedParams sp;
    ModelDims dims;
    // timing
    bool timing;
    std::vector<TimedPair> pairs;
    std::vector<hipEvent_t> free_events;
    // replay: the launches of graph_iters iterations, captured once (qsr_run)
    hipGraphExec_t graph_exec;
    int graph_iters;
};

static inline DevState *st_cur(qsr_ctx *c) { return c->d_state + c->cur; }


// ------------------------------------------------------------------------------------------
// configuration
// ------------------------------------------------------------------------------------------
static long long mlp2_params(const qsr_config *c)
{
    return c->d_in * c->d_hidden + c->d_hidden + c->d_hidden * c->d_out + c->d_out;
}
static long long resmlp_params(const qsr_config *c)
{
    const long long d = c->d_in;
    const long long attn = c->n_heads > 0 ? 2 * d + 3 * d * d + 3 * d + d * d + d : 0;
    return (long long)c->n_blocks * (attn + 2 * d + d * c->d_hidden + c->d_hidden + c->d_hidden * d + d);
}

extern "C" int qsr_validate(const qsr_config *c, const char **why)
{
    const char *w = nullptr;
    auto finite_ge0 = [](double x) { return std::isfinite(x) && x >= 0.0; };
    if (!c) w = "cfg is NULL";
    else if (c->K < 1 || c->K > 65535) w = "K";
    else if (c->P < 1) w = "P";
    else if (c->P > ((long long)1 << 34)) w = "P (above 2^34)";
    else if (c->T < 1 || c->T > 0xFFFFFFFFll) w = "T";
    else if (c->T_warm < 0 || c->T_warm > c->T) w = "T_warm";
    else if (c->opt != QSR_OPT_SGDM && c->opt != QSR_OPT_ADAMW) w = "opt";
    else if (c->model < QSR_MODEL_EXTERNAL || c->model > QSR_MODEL_RESMLP) w = "model";
    else if (c->lr_kind < QSR_LR_COSINE || c->lr_kind > QSR_LR_POW2COS) w = "lr_kind";
    else if (c->H_base < 1) w = "H_base";
    else if (c->average_state != 0 && c->average_state != 1) w = "average_state";
    else if (c->fuse_sync != 0 && c->fuse_sync != 1) w = "fuse_sync";
    else if (c->fuse_sync == 1 && (c->parallel == 1 || c->average_state == 1)) w = "fuse_sync with parallel or average_state";
    else if (c->n_heads < 0 || (c->n_heads > 0 && c->model != QSR_MODEL_RESMLP)) w = "n_heads";
    else if (c->reserved != 0) w = "reserved";
    else if (c->fuse_gradient < 0 || c->fuse_gradient > 2) w = "fuse_gradient";
    else if (c->fuse_gradient && (c->model != QSR_MODEL_NOISE || c->parallel || c->fuse_sync || c->clip_norm > 0.0 || c->P % 4 != 0))
        w = "fuse_gradient needs the noise model, P % 4 = 0, no parallel, fuse_sync or clip_norm";
    else if (!finite_ge0(c->clip_norm)) w = "clip_norm";
    else if (c->power < 0 || c->power > 8) w = "power";
    else if (c->parallel != 0 && c->parallel != 1) w = "parallel";
    else if (c->parallel == 1 && (c->H_base != 1 || c->power != 0 || c->t_local_start != 0 || c->t_swap_start != 0))
        w = "parallel needs H_base = 1, power = 0";
    else if (c->t_local_start < 0 || c->t_local_start > c->T) w = "t_local_start";
    else if (c->t_swap_start < 0 || c->t_swap_start > c->T) w = "t_swap_start";
    else if (!finite_ge0(c->alpha)) w = "alpha";
    else if (!finite_ge0(c->weight_decay)) w = "weight_decay";
    else if (c->opt == QSR_OPT_SGDM && !(finite_ge0(c->momentum) && c->momentum < 1.0)) w = "momentum";
    else if (c->opt == QSR_OPT_ADAMW &&
             !(finite_ge0(c->beta1) && c->beta1 < 1.0 && finite_ge0(c->beta2) && c->beta2 < 1.0))
        w = "beta1/beta2";
    else if (c->opt == QSR_OPT_ADAMW && !(std::isfinite(c->eps) && c->eps > 0.0)) w = "eps";
    else if (c->lr_kind != QSR_LR_TABLE && !(std::isfinite(c->eta_max) && c->eta_max > 0.0)) w = "eta_max";
    else if ((c->lr_kind == QSR_LR_COSINE || c->lr_kind == QSR_LR_LINEAR || c->lr_kind == QSR_LR_POW2COS) &&
             !(finite_ge0(c->eta_min) && c->eta_min <= c->eta_max))
        w = "eta_min";
    else if (c->lr_kind == QSR_LR_STEP &&
             (c->n_milestones < 0 || (c->n_milestones > 0 && !c->milestones) ||
              !(std::isfinite(c->step_factor) && c->step_factor > 0.0)))
        w = "milestones/step_factor";
    else if (c->lr_kind == QSR_LR_TABLE && !c->eta_table) w = "eta_table";
    if (!w && c->lr_kind == QSR_LR_TABLE) {
        for (long long t = 0; t < c->T; ++t)
            if (!(std::isfinite(c->eta_table[t]) && c->eta_table[t] >= 0.0)) { w = "eta_table entry"; break; }
    }
    if (!w && c->lr_kind == QSR_LR_STEP) {
        for (int i = 1; i < c->n_milestones; ++i)
            if (c->milestones[i] < c->milestones[i - 1]) { w = "milestones not ascending"; break; }
    }
    if (!w) {
        switch (c->model) {
        case QSR_MODEL_NOISE:
            if (!finite_ge0(c->grad_sigma)) w = "grad_sigma";
            break;
        case QSR_MODEL_LINREG:
            if (c->d_in < 1 || c->B_loc < 1) w = "d_in/B_loc";
            else if (c->P != c->d_in) w = "P != d_in";
            else if (c->B_loc * c->d_in > ((long long)1 << 34)) w = "B_loc*d_in";
            else if (!finite_ge0(c->data_sigma)) w = "data_sigma";
            break;
        case QSR_MODEL_MLP2:
            if (c->d_in < 1 || c->d_hidden < 1 || c->d_out < 1 || c->B_loc < 1) w = "d_in/d_hidden/d_out/B_loc";
            else if (c->d_out > 1024) w = "d_out (above 1024)";
            else if (c->P != mlp2_params(c)) w = "P != MLP parameter count";
            else if (c->B_loc * c->d_in > ((long long)1 << 34)) w = "B_loc*d_in";
            else if (!finite_ge0(c->data_sigma)) w = "data_sigma";
            break;
        case QSR_MODEL_RESMLP:
            if (c->d_in < 1 || c->d_hidden < 1 || c->n_blocks < 1 || c->B_loc < 1) w = "d_in/d_hidden/n_blocks/B_loc";
            else if (c->d_in % 64 != 0 || c->d_hidden % 64 != 0) w = "d_in/d_hidden not multiples of 64";
            else if (c->d_in > 1024) w = "d_in (above 1024)";
            else if (c->B_loc > (1 << 24) || c->d_hidden > (1 << 20)) w = "B_loc/d_hidden too large";
            else if (c->n_heads > 0 && c->d_in != 64LL * c->n_heads) w = "n_heads (heads are 64 wide: d_in = 64 n_heads)";
            else if (c->n_heads > 0 && (c->seq_len < 1 || c->seq_len > 224 || c->B_loc % c->seq_len != 0))
                w = "seq_len (1..224, dividing B_loc)";
            else if (c->P != resmlp_params(c)) w = "P != residual-MLP parameter count";
            else if (c->B_loc * c->d_in > ((long long)1 << 34)) w = "B_loc*d_in";
            break;
        default: break;
        }
    }
    if (why) *why = w ? w : "ok";
    return w ? QSR_EINVAL : QSR_OK;
}

static ModelDims make_dims(const qsr_config *c)
{
    ModelDims d;
    d.K = c->K; d.P = c->P; d.B = c->B_loc; d.d_in = c->d_in; d.d_hidden = c->d_hidden;
    d.d_out = c->d_out; d.n_blocks = c->n_blocks; d.data_sigma = (float)c->data_sigma;
    d.n_heads = c->n_heads; d.seq_len = c->seq_len;
    d.seed = c->seed;
    return d;
}

extern "C" int qsr_workspace_bytes(const qsr_config *cfg, size_t *bytes)
{
    if (!bytes) return QSR_EINVAL;
    *bytes = 0;
    int rc = qsr_validate(cfg, nullptr);
    if (rc != QSR_OK) return rc;
    ModelDims d = make_dims(cfg);
    switch (cfg->model) {
    case QSR_MODEL_LINREG: *bytes = linreg_workspace_bytes(d); break;
    case QSR_MODEL_MLP2: *bytes = mlp2_workspace_bytes(d); break;
    case QSR_MODEL_RESMLP: *bytes = resmlp_workspace_bytes(d); break;
    default: break;
    }
    return QSR_OK;
}

// Learning-rate schedules (Sec. 4 of the paper: cosine decay, optionally after a linear warm-up
// from 0; step decay divides the peak by a factor at each milestone).
static void build_eta(const qsr_config *c, std::vector<double> &eta)
{
    const long long T = c->T, Tw = c->T_warm;
    eta.resize((size_t)T);
    const double pi = 3.14159265358979323846;
    for (long long t = 0; t < T; ++t) {
        double e;
        if (c->lr_kind == QSR_LR_TABLE) {
            e = c->eta_table[t];
        } else if (t < Tw) {
            e = c->eta_max * (double)t / (double)Tw;
        } else if (c->lr_kind == QSR_LR_COSINE || c->lr_kind == QSR_LR_POW2COS) {
            double frac = (double)(t - Tw) / (double)(T - Tw);
            e = c->eta_min + 0.5 * (c->eta_max - c->eta_min) * (1.0 + std::cos(pi * frac));
            if (c->lr_kind == QSR_LR_POW2COS && e > 0.0) e = std::exp2(std::round(std::log2(e)));
        } else if (c->lr_kind == QSR_LR_LINEAR) {
            double frac = (double)(t - Tw) / (double)(T - Tw);
            e = c->eta_max - (c->eta_max - c->eta_min) * frac;
        } else {
            double div = 1.0;
            for (int i = 0; i < c->n_milestones; ++i)
                if (c->milestones[i] <= t) div *= c->step_factor;
            e = c->eta_max / div;
        }
        eta[(size_t)t] = e;
    }
}

static void build_scalars(const qsr_config *c, const std::vector<double> &eta,
                          std::vector<StepScalars> &sc)
{
    sc.resize(eta.size());
    for (size_t t = 0; t < eta.size(); ++t) {
        StepScalars s{0.f, 0.f, 0.f, 0.f};
        if (c->opt == QSR_OPT_SGDM) {
            s.x = (float)eta[t];
        } else {
            double n = (double)(t + 1);      // Adam's step count = global iteration count
            double bc1 = 1.0 - std::pow(c->beta1, n);
            double bc2 = 1.0 - std::pow(c->beta2, n);
            s.x = (float)(eta[t] * c->weight_decay);
            s.y = (float)(eta[t] / bc1);
            s.z = (float)(1.0 / std::sqrt(bc2));
        }
        sc[t] = s;
    }
}

// Eq. (2) on the host, for the mirror: the same operations in the same order as the device
// scheduler's routine (IEEE double division and multiplications, no fused operations, floor), on
// the same table, so the two integer sequences are equal.
static long long host_get_H(const SchedParams &sp, const double *eta, long long t)
{
#pragma STDC FP_CONTRACT OFF
    const long long rem = sp.T - t;
    if (rem <= 0) return 0;
    if (sp.t_swap_start > 0 && t >= sp.t_swap_start) return rem;
    if (t < sp.t_local_start) return 1;
    if (sp.power == 0) return sp.H_base < rem ? sp.H_base : rem;
    const long long te = t < sp.T_warm ? sp.T_warm : t;
    if (te >= sp.T) return rem;
    const volatile double e = eta[te];
    if (!(e > 0.0)) return rem;
    const volatile double q = sp.alpha / e;
    volatile double v = q;
    for (int i = 1; i < sp.power; ++i) v = v * q;
    if (!(v < (double)rem)) return rem;
    long long H = (long long)std::floor(v);
    if (H < sp.H_base) H = sp.H_base;
    if (H > rem) H = rem;
    return H;
}

static void mirror_reset(qsr_ctx *c, long long t, long long s, long long h, long long H)
{
    c->m_t = t; c->m_s = s; c->m_h = h; c->m_H = H;
    c->m_log_t.assign((size_t)s, 0);
    c->m_log_H.assign((size_t)s, 0);
}

// true if the iteration about to run (or just run, before mirror_advance) completes its round
static inline bool mirror_sync_now(const qsr_ctx *c) { return c->m_h + 1 == c->m_H; }

static void mirror_advance(qsr_ctx *c)
{
    c->m_t += 1; c->m_h += 1;
    if (c->m_h == c->m_H) {
        c->m_log_t.push_back(c->m_t);
        c->m_log_H.push_back(c->m_H);
        c->m_s += 1; c->m_h = 0;
        c->m_H = host_get_H(c->sp, c->eta.data(), c->m_t);
    }
}

static SchedParams sched_params_of(const qsr_config &cfg)
{
    SchedParams sp{};
    sp.T = cfg.T; sp.T_warm = cfg.T_warm; sp.H_base = cfg.H_base; sp.alpha = cfg.alpha;
    sp.power = cfg.power; sp.t_local_start = cfg.t_local_start; sp.t_swap_start = cfg.t_swap_start;
    return sp;
}

extern "C" int qsr_host_schedule(const qsr_config *cfg, int64_t *t_out, int64_t *H_out, int64_t cap, int64_t *n)
{
    if (!n || cap < 0) return QSR_EINVAL;
    int rc = qsr_validate(cfg, nullptr);
    if (rc != QSR_OK) return rc;
    std::vector<double> eta;
    build_eta(cfg, eta);
    const SchedParams sp = sched_params_of(*cfg);
    long long t = 0, rounds = 0;
    while (t < cfg->T) {
        const long long H = host_get_H(sp, eta.data(), t);
        if (H < 1) return QSR_EINVAL;
        t += H;
        if (rounds < cap) {
            if (t_out) t_out[rounds] = t;
            if (H_out) H_out[rounds] = H;
        }
        rounds += 1;
    }
    *n = rounds;
    return QSR_OK;
}

// ------------------------------------------------------------------------------------------
// life cycle
// ------------------------------------------------------------------------------------------
static void free_ctx(qsr_ctx *c)
{
    if (!c) return;
    for (auto &p : c->pairs) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
    for (auto e : c->free_events) (void)hipEventDestroy(e);
    if (c->d_state) (void)hipFree(c->d_state);
    if (c->d_eta) (void)hipFree(c->d_eta);
    if (c->d_scal) (void)hipFree(c->d_scal);
    if (c->d_log_t) (void)hipFree(c->d_log_t);
    if (c->d_log_H) (void)hipFree(c->d_log_H);
    if (c->d_loss) (void)hipFree(c->d_loss);
    if (c->d_clip_part) (void)hipFree(c->d_clip_part);
    if (c->d_clip_coef) (void)hipFree(c->d_clip_coef);
    if (c->h_state) (void)hipHostFree(c->h_state);
    if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
    delete c;
}

static int init_impl(qsr_ctx *c, const float *theta0)
{
    const qsr_config &cfg = c->cfg;
    const size_t T = (size_t)cfg.T;
    HIP_TRY(hipGetDevice(&c->device));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, c->device));
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return QSR_ENOGPU;
    {   // set-up of the entry point that must not allocate later: find its array on this device now
        int rc = clip_static_setup(nullptr);
        if (rc != QSR_OK) return rc;
    }

    HIP_TRY(hipMalloc((void **)&c->d_state, 2 * sizeof(DevState)));
    HIP_TRY(hipMemset(c->d_state, 0, 2 * sizeof(DevState)));
    HIP_TRY(hipMalloc((void **)&c->d_eta, T * sizeof(double)));
    HIP_TRY(hipMalloc((void **)&c->d_scal, T * sizeof(StepScalars)));
    HIP_TRY(hipMalloc((void **)&c->d_log_t, T * sizeof(long long)));
    HIP_TRY(hipMalloc((void **)&c->d_log_H, T * sizeof(long long)));
    HIP_TRY(hipMalloc((void **)&c->d_loss, (size_t)cfg.K * sizeof(float)));
    if (cfg.clip_norm > 0.0) {
        HIP_TRY(hipMalloc((void **)&c->d_clip_part, (size_t)cfg.K * clip_blocks_per_row(cfg.P) * sizeof(double)));
        HIP_TRY(hipMalloc((void **)&c->d_clip_coef, 2 * (size_t)cfg.K * sizeof(float)));
    }
    HIP_TRY(hipHostMalloc((void **)&c->h_state, sizeof(DevState), hipHostMallocDefault));

    std::vector<StepScalars> sc;
    build_eta(&cfg, c->eta);
    build_scalars(&cfg, c->eta, sc);
    // the two tables are copied from pageable memory: finish the copies before `sc` dies
    HIP_TRY(hipMemcpyAsync(c->d_eta, c->eta.data(), T * sizeof(double), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipMemcpyAsync(c->d_scal, sc.data(), T * sizeof(StepScalars), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));

    c->sp = sched_params_of(cfg);
    c->sp.eta = c->d_eta; c->sp.log_t = c->d_log_t; c->sp.log_H = c->d_log_H;

    const long long n = (long long)cfg.K * cfg.P;
    if (theta0) HIP_TRY(launch_broadcast_rows(c->params, theta0, cfg.K, cfg.P, c->stream));
    HIP_TRY(launch_fill_zero(c->state0, n, c->stream));
    if (c->state1) HIP_TRY(launch_fill_zero(c->state1, n, c->stream));
    HIP_TRY(launch_fill_zero(c->d_loss, cfg.K, c->stream));
    HIP_TRY(launch_sched_init(st_cur(c), c->sp, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    mirror_reset(c, 0, 0, 0, host_get_H(c->sp, c->eta.data(), 0));
    return QSR_OK;
}

extern "C" int qsr_init(const qsr_config *cfg, float *params, float *grads, float *state0,
                        float *state1, const float *theta0, const float *model_const,
                        void *workspace, size_t workspace_bytes, qsr_ctx **out)
{
    if (!out) return QSR_EINVAL;
    *out = nullptr;
    int rc = qsr_validate(cfg, nullptr);
    if (rc != QSR_OK) return rc;
    if (!params || !grads || !state0) return QSR_EINVAL;
    if (cfg->opt == QSR_OPT_ADAMW && !state1) return QSR_EINVAL;
    auto misaligned = [](const void *p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) != 0; };
    if (misaligned(params, 16) || misaligned(grads, 16) || misaligned(state0, 16) ||
        (state1 && misaligned(state1, 16)))
        return QSR_EINVAL;
    size_t need = 0;
    rc = qsr_workspace_bytes(cfg, &need);
    if (rc != QSR_OK) return rc;
    if (need > 0 && (!workspace || misaligned(workspace, 256))) return QSR_EINVAL;
    if (workspace_bytes < need) return QSR_ENOMEM;
    if (cfg->model >= QSR_MODEL_LINREG && !model_const) return QSR_EINVAL;

    qsr_ctx *c = new (std::nothrow) qsr_ctx();
    if (!c) return QSR_ENOMEM;
    c->cfg = *cfg;                     // its host pointers are valid during this call only
    c->stream = (hipStream_t)cfg->stream;
    c->params = params; c->grads = grads; c->state0 = state0;
    c->state1 = cfg->opt == QSR_OPT_ADAMW ? state1 : nullptr;
    c->model_const = model_const; c->workspace = workspace; c->workspace_bytes = workspace_bytes;
    c->d_state = nullptr; c->d_eta = nullptr; c->d_scal = nullptr; c->d_log_t = nullptr;
    c->d_log_H = nullptr; c->d_loss = nullptr; c->h_state = nullptr;
    c->d_clip_part = nullptr; c->d_clip_coef = nullptr;
    c->t_host = 0; c->need_sync_call = false; c->timing = false; c->capturing = false;
    c->graph_exec = nullptr;
    // Iterations per captured graph: several where an iteration is a handful of short launches.
    // Larger problems are never replayed from a graph: replaying did not shorten their iterations
    // (timed: only the least-squares workload gained), and enqueued one by one an averaging kernel is
    // launched only where the mirror says a round ends, while a graph has to hold a launch in every
    // iteration for the device to skip (7 us per iteration for the perceptron's 814 090 parameters).
    c->graph_iters = (cfg->model == QSR_MODEL_RESMLP || (long long)cfg->K * cfg->P >= (1ll << 20)) ? 0 : 8;
    // Contexts whose iterations are never replayed from a graph (a recorded launch could not be handed the
    // copy of the scheduler state that alternates from iteration to iteration): the update kernel takes
    // the scheduler's step on the iterations that end no round, and no scheduler kernel is launched there.
    c->cur = 0; c->ticked = false;
    c->fold_tick = c->graph_iters == 0 && !cfg->parallel && (cfg->clip_norm <= 0.0 || (cfg->P & 3) == 0);
    c->dims = make_dims(cfg);
    rc = init_impl(c, theta0);
    c->cfg.milestones = nullptr;
    c->cfg.eta_table = nullptr;
    if (rc != QSR_OK) { free_ctx(c); return rc; }
    *out = c;
    return QSR_OK;
}

extern "C" int qsr_destroy(qsr_ctx *ctx)
{
    if (!ctx) return QSR_EINVAL;
    (void)hipStreamSynchronize(ctx->stream);
    free_ctx(ctx);
    return QSR_OK;
}

// ------------------------------------------------------------------------------------------
// timing helpers
// ------------------------------------------------------------------------------------------
static int get_event(qsr_ctx *c, hipEvent_t *e)
{
    if (!c->free_events.empty()) { *e = c->free_events.back(); c->free_events.pop_back(); return QSR_OK; }
    HIP_TRY(hipEventCreate(e));
    return QSR_OK;
}

struct Bracket {
    qsr_ctx *c; int kind; hipEvent_t a, b; bool on; int rc;
    Bracket(qsr_ctx *c_, int kind_) : c(c_), kind(kind_), a(nullptr), b(nullptr), on(c_->timing), rc(QSR_OK)
    {
        if (!on) return;
        rc = get_event(c, &a);
        if (rc == QSR_OK) rc = get_event(c, &b);
        if (rc == QSR_OK && hipEventRecord(a, c->stream) != hipSuccess) rc = QSR_EHIP;
    }
    int close(long long t_after)
    {
        if (!on || rc != QSR_OK) return rc;
        if (hipEventRecord(b, c->stream) != hipSuccess) return QSR_EHIP;
        c->pairs.push_back(TimedPair{a, b, kind, t_after});
        return QSR_OK;
    }
};

// ------------------------------------------------------------------------------------------
// the iteration
// ------------------------------------------------------------------------------------------
extern "C" int qsr_local_step(qsr_ctx *c)
{
    if (!c) return QSR_EINVAL;
    if (c->t_host >= c->cfg.T || c->need_sync_call) return QSR_ESTATE;
    const qsr_config &cfg = c->cfg;

    if (cfg.model != QSR_MODEL_EXTERNAL && !cfg.fuse_gradient) {   // Eq. (1): every worker's local gradient
        Bracket br(c, 0);
        if (br.rc != QSR_OK) return br.rc;
        switch (cfg.model) {
        case QSR_MODEL_NOISE:
            HIP_TRY(launch_noise_grad(c->grads, cfg.K, cfg.P, (float)cfg.grad_sigma, cfg.seed,
                                      st_cur(c), c->stream));
            break;
        case QSR_MODEL_LINREG:
            HIP_TRY(launch_linreg_grad(c->dims, c->params, c->grads, c->model_const, c->workspace,
                                       c->d_loss, st_cur(c), c->stream));
            break;
        case QSR_MODEL_MLP2:
            HIP_TRY(launch_mlp2_grad(c->dims, c->params, c->grads, c->model_const, c->workspace,
                                     c->d_loss, st_cur(c), c->stream));
            break;
        case QSR_MODEL_RESMLP:
            HIP_TRY(launch_resmlp_grad(c->dims, c->params, c->grads, c->model_const, c->workspace,
                                       c->d_loss, st_cur(c), c->stream));
            break;
        default: return QSR_EINVAL;
        }
        int rc = br.close(c->t_host);
        if (rc != QSR_OK) return rc;
    }
    if (cfg.parallel) {                                 // Alg. 1: All-Reduce of the local gradients
        Bracket br(c, 2);
        if (br.rc != QSR_OK) return br.rc;
        HIP_TRY(launch_average_rows(c->grads, cfg.K, cfg.P, nullptr, c->stream));
        int rc = br.close(c->t_host + 1);
        if (rc != QSR_OK) return rc;
    }
    // The step that completes a round (h + 1 == H): known to the host from its mirror; under graph
    // capture every launch is recorded and the device decides.
    const bool all = c->capturing;
    const bool sync_now = mirror_sync_now(c);
    const bool fused = cfg.fuse_sync != 0;
    DevState *st_next = (c->fold_tick && !all && !sync_now) ? c->d_state + (c->cur ^ 1) : nullptr;
    if (!fused || all || !sync_now) {                   // OPT for all K workers at once
        Bracket br(c, 1);
        if (br.rc != QSR_OK) return br.rc;
        if (cfg.clip_norm > 0.0)                        // App. C: per-worker factors min(1, c / (||g_k|| + 1e-6))
            HIP_TRY(launch_clip_coef(c->grads, cfg.K, cfg.P, (float)cfg.clip_norm, c->d_clip_part,
                                     c->d_clip_coef, c->d_clip_coef + cfg.K, c->stream));
        if (cfg.fuse_gradient && cfg.opt == QSR_OPT_SGDM)   // Eq. (1) and OPT in one pass (noise model)
            HIP_TRY(launch_update_sgdm_noise(c->params, c->grads, c->state0, cfg.K, cfg.P, st_cur(c), c->d_scal,
                                             (float)cfg.momentum, (float)cfg.weight_decay, (float)cfg.grad_sigma,
                                             cfg.seed, cfg.fuse_gradient == 1, c->stream, st_next, &c->sp));
        else if (cfg.fuse_gradient)
            HIP_TRY(launch_update_adamw_noise(c->params, c->grads, c->state0, c->state1, cfg.K, cfg.P, st_cur(c),
                                              c->d_scal, (float)(1.0 - cfg.beta1), (float)(1.0 - cfg.beta2),
                                              (float)cfg.eps, (float)cfg.grad_sigma, cfg.seed, cfg.fuse_gradient == 1,
                                              c->stream, st_next, &c->sp));
        else if (cfg.opt == QSR_OPT_SGDM)
            HIP_TRY(launch_update_sgdm(c->params, c->grads, c->state0, cfg.K, cfg.P, st_cur(c), c->d_scal,
                                       (float)cfg.momentum, (float)cfg.weight_decay, fused, c->d_clip_coef,
                                       c->stream, st_next, &c->sp));
        else
            HIP_TRY(launch_update_adamw(c->params, c->grads, c->state0, c->state1, cfg.K, cfg.P, st_cur(c),
                                        c->d_scal, (float)(1.0 - cfg.beta1), (float)(1.0 - cfg.beta2),
                                        (float)cfg.eps, fused, c->d_clip_coef, c->stream, st_next, &c->sp));
        int rc = br.close(c->t_host);
        if (rc != QSR_OK) return rc;
        if (st_next) { c->cur ^= 1; c->ticked = true; }    // the advanced state is in the other copy now
    }
    if (fused && (all || sync_now)) {                   // the round's last step: OPT and All-Reduce in one pass
        Bracket br(c, 2);                               // timed like an averaging launch
        if (br.rc != QSR_OK) return br.rc;
        if (cfg.clip_norm > 0.0 && !all)                // (under capture the plain launch above has computed them)
            HIP_TRY(launch_clip_coef(c->grads, cfg.K, cfg.P, (float)cfg.clip_norm, c->d_clip_part,
                                     c->d_clip_coef, c->d_clip_coef + cfg.K, c->stream));
        if (cfg.opt == QSR_OPT_SGDM)
            HIP_TRY(launch_update_sgdm_sync(c->params, c->grads, c->state0, cfg.K, cfg.P, st_cur(c), c->d_scal,
                                            (float)cfg.momentum, (float)cfg.weight_decay, c->d_clip_coef, c->stream));
        else
            HIP_TRY(launch_update_adamw_sync(c->params, c->grads, c->state0, c->state1, cfg.K, cfg.P, st_cur(c),
                                             c->d_scal, (float)(1.0 - cfg.beta1), (float)(1.0 - cfg.beta2),
                                             (float)cfg.eps, c->d_clip_coef, c->stream));
        int rc = br.close(c->t_host + 1);
        if (rc != QSR_OK) return rc;
    }
    c->t_host += 1;
    c->need_sync_call = true;
    return QSR_OK;
}

extern "C" int qsr_maybe_sync(qsr_ctx *c)
{
    if (!c) return QSR_EINVAL;
    if (!c->need_sync_call) return QSR_ESTATE;
    if (c->ticked) {                     // no round ends here and the update kernel has advanced the scheduler
        mirror_advance(c);
        c->ticked = false;
        c->need_sync_call = false;
        return QSR_OK;
    }
    const bool all = c->capturing;
    const bool sync_now = mirror_sync_now(c);
    // Replayed iterations of small problems: the averaging launch, which a graph holds in every
    // iteration, also closes the iteration (one launch less where a launch is a third of the work)
    if (all && !c->cfg.parallel && !c->cfg.fuse_sync && !c->cfg.average_state && average_can_advance(c->cfg.K, c->cfg.P)) {
        HIP_TRY(launch_average_rows_advance(c->params, c->cfg.K, c->cfg.P, st_cur(c), c->sp, c->stream));
        mirror_advance(c);
        c->need_sync_call = false;
        return QSR_OK;
    }
    // Parallel OPT keeps the workers identical, the fused form has averaged in qsr_local_step already
    if (!c->cfg.parallel && !c->cfg.fuse_sync && (all || sync_now)) {
        Bracket br(c, 2);
        if (br.rc != QSR_OK) return br.rc;
        HIP_TRY(launch_average_rows(c->params, c->cfg.K, c->cfg.P, st_cur(c), c->stream));
        int rc = br.close(c->t_host);
        if (rc != QSR_OK) return rc;
        if (c->cfg.average_state) {          // same device-side decision, taken before the scheduler advances
            HIP_TRY(launch_average_rows(c->state0, c->cfg.K, c->cfg.P, st_cur(c), c->stream));
            if (c->state1) HIP_TRY(launch_average_rows(c->state1, c->cfg.K, c->cfg.P, st_cur(c), c->stream));
        }
    }
    HIP_TRY(launch_sched_advance(st_cur(c), c->sp, all ? -1 : (sync_now ? 1 : 0), c->stream));
    mirror_advance(c);
    c->need_sync_call = false;
    return QSR_OK;
}

static int run_one_by_one(qsr_ctx *c, long long n)
{
    for (long long i = 0; i < n; ++i) {
        int rc = qsr_local_step(c);
        if (rc == QSR_OK) rc = qsr_maybe_sync(c);
        if (rc != QSR_OK) return rc;
    }
    return QSR_OK;
}

// Every kernel of an iteration takes t, h, H and the averaging decision from device memory, and
// launch shapes depend on the configuration only: the launches of one iteration are the same for
// every t, so they are recorded once into a HIP graph (kernel nodes only) and replayed.
extern "C" int qsr_run(qsr_ctx *c, int64_t n)
{
    if (!c || n < 0) return QSR_EINVAL;
    if (c->need_sync_call || n > c->cfg.T - c->t_host) return QSR_ESTATE;
    const long long per = c->graph_iters;
    // the null stream cannot be captured; with timing on every launch gets its own event bracket
    if (c->timing || c->stream == nullptr || per < 1 || n < 1 + 2 * per) return run_one_by_one(c, n);
    if (!c->graph_exec) {
        // whatever a kernel sets up at its first launch happens here, outside the capture
        int rc = run_one_by_one(c, 1);
        if (rc != QSR_OK) return rc;
        n -= 1;
        // recorded, not run: the host's counters and its mirror of the schedule are put back afterwards
        const long long t_keep = c->t_host, m_keep[4] = {c->m_t, c->m_s, c->m_h, c->m_H};
        const size_t log_keep = c->m_log_t.size();
        if (hipStreamBeginCapture(c->stream, hipStreamCaptureModeRelaxed) != hipSuccess) {
            (void)hipGetLastError();                  // a stream that cannot be captured: one by one from now on
            c->graph_iters = 0;
            return run_one_by_one(c, n);
        }
        c->capturing = true;
        rc = run_one_by_one(c, per);
        c->capturing = false;
        hipGraph_t g = nullptr;
        hipError_t e = hipStreamEndCapture(c->stream, &g);
        c->t_host = t_keep;
        c->need_sync_call = false;
        c->m_t = m_keep[0]; c->m_s = m_keep[1]; c->m_h = m_keep[2]; c->m_H = m_keep[3];
        c->m_log_t.resize(log_keep); c->m_log_H.resize(log_keep);
        if (rc == QSR_OK && e == hipSuccess) e = hipGraphInstantiate(&c->graph_exec, g, nullptr, nullptr, 0);
        if (g) (void)hipGraphDestroy(g);
        if (rc != QSR_OK) return rc;
        if (e != hipSuccess) { c->graph_exec = nullptr; g_last_hip = (int)e; return QSR_EHIP; }
    }
    while (n >= per) {
        HIP_TRY(hipGraphLaunch(c->graph_exec, c->stream));
        c->t_host += per;
        for (long long i = 0; i < per; ++i) mirror_advance(c);
        n -= per;
    }
    return run_one_by_one(c, n);
}

// Device scheduler state to the host.  Between qsr_local_step and its qsr_maybe_sync the device has
// not advanced its counters yet where the advance is the last launch of an iteration: the step just
// enqueued is added here, so that callers see t and h count it, as the protocol says.  (Where the
// update kernel has taken the step itself, the counters already include it.)
static int fetch_state(qsr_ctx *c)
{
    HIP_TRY(hipMemcpyAsync(c->h_state, st_cur(c), sizeof(DevState), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    if (c->h_state->mismatch) return QSR_EMIRROR;
    if (c->need_sync_call && !c->ticked) { c->h_state->t += 1; c->h_state->h += 1; }
    return QSR_OK;
}

extern "C" int qsr_get_H(qsr_ctx *c, int64_t *H, int64_t *round, int64_t *t)
{
    if (!c) return QSR_EINVAL;
    int rc = fetch_state(c);
    if (rc != QSR_OK) return rc;
    if (H) *H = c->h_state->H;
    if (round) *round = c->h_state->s;
    if (t) *t = c->h_state->t;
    return QSR_OK;
}

extern "C" int qsr_read_sync_log(qsr_ctx *c, int64_t *t_out, int64_t *H_out, int64_t cap, int64_t *n)
{
    if (!c || !n || cap < 0) return QSR_EINVAL;
    int rc = fetch_state(c);
    if (rc != QSR_OK) return rc;
    long long rounds = c->h_state->s;
    *n = rounds;
    long long m = rounds < cap ? rounds : cap;
    if (m > 0 && t_out) HIP_TRY(hipMemcpy(t_out, c->d_log_t, (size_t)m * sizeof(long long), hipMemcpyDeviceToHost));
    if (m > 0 && H_out) HIP_TRY(hipMemcpy(H_out, c->d_log_H, (size_t)m * sizeof(long long), hipMemcpyDeviceToHost));
    return QSR_OK;
}

extern "C" int qsr_read_host_schedule(qsr_ctx *c, int64_t *t_out, int64_t *H_out, int64_t cap, int64_t *n)
{
    if (!c || !n || cap < 0) return QSR_EINVAL;
    const long long rounds = (long long)c->m_log_t.size();
    *n = rounds;
    const long long m = rounds < cap ? rounds : cap;
    for (long long i = 0; i < m; ++i) {
        if (t_out) t_out[i] = c->m_log_t[(size_t)i];
        if (H_out) H_out[i] = c->m_log_H[(size_t)i];
    }
    return QSR_OK;
}

extern "C" int qsr_eta_table(qsr_ctx *c, double *eta_out, int64_t cap)
{
    if (!c || !eta_out || cap < c->cfg.T) return QSR_EINVAL;
    std::memcpy(eta_out, c->eta.data(), (size_t)c->cfg.T * sizeof(double));
    return QSR_OK;
}

extern "C" int qsr_read_loss(qsr_ctx *c, float *loss_out)
{
    if (!c || !loss_out) return QSR_EINVAL;
    HIP_TRY(hipStreamSynchronize(c->stream));
    HIP_TRY(hipMemcpy(loss_out, c->d_loss, (size_t)c->cfg.K * sizeof(float), hipMemcpyDeviceToHost));
    return QSR_OK;
}

extern "C" int qsr_get_state(qsr_ctx *c, int64_t state[4])
{
    if (!c || !state) return QSR_EINVAL;
    int rc = fetch_state(c);
    if (rc != QSR_OK) return rc;
    state[0] = c->h_state->t; state[1] = c->h_state->s; state[2] = c->h_state->h; state[3] = c->h_state->H;
    return QSR_OK;
}

extern "C" int qsr_set_state(qsr_ctx *c, const int64_t state[4])
{
    if (!c || !state) return QSR_EINVAL;
    const long long t = state[0], s = state[1], h = state[2], H = state[3], T = c->cfg.T;
    if (t < 0 || t > T || s < 0 || s > t || h < 0 || h > t) return QSR_EINVAL;
    if (t == T ? (H != 0 || h != 0) : (H < 1 || h >= H || H - h > T - t)) return QSR_EINVAL;
    if (c->need_sync_call) return QSR_ESTATE;
    HIP_TRY(launch_sched_set(st_cur(c), c->sp, t, s, h, H, c->stream));
    c->t_host = t;
    mirror_reset(c, t, s, h, H);
    return QSR_OK;
}

extern "C" int qsr_restart(qsr_ctx *c)
{
    if (!c) return QSR_EINVAL;
    HIP_TRY(launch_sched_init(st_cur(c), c->sp, c->stream));
    c->t_host = 0;
    c->need_sync_call = false;
    c->ticked = false;
    mirror_reset(c, 0, 0, 0, host_get_H(c->sp, c->eta.data(), 0));
    return QSR_OK;
}

extern "C" int qsr_timing(qsr_ctx *c, int enable)
{
    if (!c) return QSR_EINVAL;
    c->timing = enable != 0;
    return QSR_OK;
}

extern "C" int qsr_read_timing_stats(qsr_ctx *c, double ms[4], int64_t count[4], double ms_min[4],
                                     double ms_median[4])
{
    if (!c || !ms || !count) return QSR_EINVAL;
    for (int i = 0; i < 4; ++i) { ms[i] = 0.0; count[i] = 0; }
    int rc = fetch_state(c);
    if (rc != QSR_OK) return rc;
    // averaging really ran after exactly the iteration counts in the device's log
    long long rounds = c->h_state->s;
    std::vector<long long> log((size_t)rounds);
    if (rounds > 0) HIP_TRY(hipMemcpy(log.data(), c->d_log_t, (size_t)rounds * sizeof(long long), hipMemcpyDeviceToHost));
    size_t li = 0;
    std::vector<float> each[4];
    for (auto &p : c->pairs) {
        float e = 0.f;
        HIP_TRY(hipEventElapsedTime(&e, p.a, p.b));
        int slot = p.kind;
        if (p.kind == 2) {
            while (li < log.size() && log[li] < p.t_after) ++li;
            bool ran = li < log.size() && log[li] == p.t_after;
            slot = ran ? 2 : 3;
        }
        ms[slot] += (double)e; count[slot] += 1;
        if (ms_min || ms_median) each[slot].push_back(e);
        c->free_events.push_back(p.a);
        c->free_events.push_back(p.b);
    }
    c->pairs.clear();
    for (int i = 0; i < 4; ++i) {
        std::vector<float> &v = each[i];
        double lo = 0.0, med = 0.0;
        if (!v.empty()) {
            std::sort(v.begin(), v.end());
            lo = v.front();
            med = v.size() % 2 ? v[v.size() / 2] : 0.5 * ((double)v[v.size() / 2 - 1] + (double)v[v.size() / 2]);
        }
        if (ms_min) ms_min[i] = lo;
        if (ms_median) ms_median[i] = med;
    }
    return QSR_OK;
}

extern "C" int qsr_read_timing(qsr_ctx *c, double ms[4], int64_t count[4])
{
    return qsr_read_timing_stats(c, ms, count, nullptr, nullptr);
}

extern "C" int qsr_average_rows(float *buf, int32_t K, int64_t P, void *stream)
{
    if (!buf || K < 1 || P < 1 || ((uintptr_t)buf & 15) != 0) return QSR_EINVAL;
    HIP_TRY(launch_average_rows(buf, K, P, nullptr, (hipStream_t)stream));
    return QSR_OK;
}

extern "C" const char *qsr_strerror(int code)
{
    switch (code) {
    case QSR_OK: return "ok";
    case QSR_EINVAL: return "invalid argument or configuration";
    case QSR_ESTATE: return "call out of protocol";
    case QSR_EHIP: return "HIP runtime error";
    case QSR_ENOMEM: return "workspace too small or allocation failed";
    case QSR_ENOGPU: return "no gfx950 device";
    case QSR_EMIRROR: return "host schedule mirror and device scheduler disagree";
    case QSR_ELIMIT: return "beyond the fixed capacity of an entry point that allocates nothing";
    default: return "unknown error";
    }
}

extern "C" int qsr_last_hip_error(void) { return g_last_hip; }
