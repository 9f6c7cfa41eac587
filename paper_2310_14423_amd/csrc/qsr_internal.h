// qsr_internal.h -- declarations shared by the library's HIP sources (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qsr.h"

namespace qsr {

// Scheduler state of Alg. 2 (arXiv 2310.14423), resident in device memory.  Kernels read the
// iteration counter from here, so the host never has to wait for the device between steps.
struct DevState {
    long long t;        // global iterations done
    long long s;        // finished rounds
    long long h;        // local steps done in the current round
    long long H;        // synchronization period of the current round (0 once t == T)
    int mismatch;       // set (and kept) when the host's mirror of the schedule expected another decision
    unsigned ticket;    // workgroups of an averaging launch that have finished (that launch then closes the iteration)
};

// Per-iteration scalars of the OPT update, prepared on the host in double precision and
// rounded once to float.  SGD: x = eta_t.  AdamW: x = eta_t*lambda, y = eta_t/(1-beta1^n),
// z = 1/sqrt(1-beta2^n), n = t+1.
struct StepScalars {
    float x, y, z, w;
};

struct SchedParams {
    long long T, T_warm;
    long long H_base;
    long long t_local_start; // post-local phase: H = 1 for rounds starting before it
    long long t_swap_start;  // SWAP phase: a round starting at or after it runs to T; 0 = off
    int power;               // exponent of the rule; 0 = constant H_base
    double alpha;
    const double *eta;      // [T] device
    long long *log_t;       // [T] device: iteration count at each averaging
    long long *log_H;       // [T] device: period of each finished round
};

// 128-bit streaming (non-temporal) global accesses: data touched once per kernel
typedef float vf4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld_nt4(const float4 *p)
{
    vf4 v = __builtin_nontemporal_load((const vf4 *)p);
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_nt4(float4 *p, float4 v)
{
    vf4 w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, (vf4 *)p);
}

// streams of the counter-based generator (second counter word)
enum : uint32_t { STREAM_GRAD = 0, STREAM_X = 1, STREAM_NOISE = 2, STREAM_LABEL = 3 };

// records the hipError_t that qsr_last_hip_error() reports for the calling thread
void set_last_hip_error(int code);

// ---- launchers (each returns the hipError_t of its launch) --------------------------------
hipError_t launch_sched_init(DevState *st, SchedParams sp, hipStream_t s);
hipError_t launch_sched_set(DevState *st, SchedParams sp, long long t, long long s_, long long h, long long H,
                            hipStream_t s);
// end of an iteration: t += 1, h += 1 and, if that was the round's H-th step, the round is logged and
// the next one opened.  expect_sync: what the host's mirror of the schedule decided (1 / 0), checked
// against the device's own decision, or -1 for no check (launches replayed from a graph).
hipError_t launch_sched_advance(DevState *st, SchedParams sp, int expect_sync, hipStream_t s);

// fused_sync: leave the step that completes a round to launch_update_*_sync.
// row_coef: K clipping factors the gradient rows are multiplied by as they are read, or nullptr.
// st_next != nullptr (with sp; not for clipped rows whose length is not a multiple of 4): the kernel also
// takes the scheduler's end-of-iteration step, on an iteration that does not end a round: the advanced
// state goes to *st_next, a second copy that no kernel of this iteration reads.
hipError_t launch_update_sgdm(float *theta, float *g, float *buf, int K, long long P,
                              const DevState *st, const StepScalars *sc, float mu, float lambda,
                              bool fused_sync, const float *row_coef, hipStream_t s,
                              DevState *st_next = nullptr, const SchedParams *sp = nullptr);
hipError_t launch_update_adamw(float *theta, float *g, float *m, float *v, int K, long long P,
                               const DevState *st, const StepScalars *sc, float c1, float c2,
                               float eps, bool fused_sync, const float *row_coef, hipStream_t s,
                               DevState *st_next = nullptr, const SchedParams *sp = nullptr);
// the same updates with the optimizer-only workloads' gradient g = sigma * N(0,1) drawn inside the
// kernel (and written to g if store_g); P must be a multiple of 4
hipError_t launch_update_sgdm_noise(float *theta, float *g, float *buf, int K, long long P, const DevState *st,
                                    const StepScalars *sc, float mu, float lambda, float sigma, uint64_t seed,
                                    bool store_g, hipStream_t s, DevState *st_next = nullptr,
                                    const SchedParams *sp = nullptr);
hipError_t launch_update_adamw_noise(float *theta, float *g, float *m, float *v, int K, long long P,
                                     const DevState *st, const StepScalars *sc, float c1, float c2, float eps,
                                     float sigma, uint64_t seed, bool store_g, hipStream_t s,
                                     DevState *st_next = nullptr, const SchedParams *sp = nullptr);
// update + averaging in one pass over the [K][P] buffers, only on the step that completes a round
hipError_t launch_update_sgdm_sync(float *theta, const float *g, float *buf, int K, long long P,
                                   const DevState *st, const StepScalars *sc, float mu, float lambda,
                                   const float *row_coef, hipStream_t s);
hipError_t launch_update_adamw_sync(float *theta, const float *g, float *m, float *v, int K, long long P,
                                    const DevState *st, const StepScalars *sc, float c1, float c2,
                                    float eps, const float *row_coef, hipStream_t s);

// gradient clipping: coef[k] = min(1, max_norm / (||g_k|| + 1e-6)), norm[k] = ||g_k||;
// partial: K * clip_blocks_per_row(P) doubles of scratch
int clip_blocks_per_row(long long P);
hipError_t launch_clip_coef(const float *g, int K, long long P, float max_norm, double *partial, float *coef,
                            float *norm, hipStream_t s);
// device address, on the current device, of the partial-sum array inside the library's image
// (qsr_clip_factors_static); looked up at the first call on a device.  Returns a QSR_* code.
int clip_static_setup(double **out);

// mean over the K rows of buf [K][P], written to all rows; with st != nullptr the launch acts only
// if the iteration in progress completes its round (st->h + 1 == st->H, read before the advance)
hipError_t launch_average_rows(float *buf, int K, long long P, const DevState *st, hipStream_t s);
// The same launch also closing the iteration: the workgroup that finishes last advances the scheduler
// (sched_advance, no mirror check), which saves the one-thread launch behind it where an iteration
// is a handful of microsecond kernels.  Only for launches of few workgroups: average_can_advance.
bool average_can_advance(int K, long long P);
hipError_t launch_average_rows_advance(float *buf, int K, long long P, DevState *st, SchedParams sp, hipStream_t s);

hipError_t launch_broadcast_rows(float *dst, const float *src, int K, long long P, hipStream_t s);
hipError_t launch_fill_zero(float *dst, long long n, hipStream_t s);

// out[k*row_stride + i] = sigma * z for i < n, z ~ N(0,1) keyed (seed; i/4, stream, k, st->t)
hipError_t launch_fill_normal(float *out, long long row_stride, int K, long long n, float sigma,
                              uint32_t stream, uint64_t seed, const DevState *st, hipStream_t s);
hipError_t launch_noise_grad(float *g, int K, long long P, float sigma, uint64_t seed,
                             const DevState *st, hipStream_t s);

struct ModelDims {
    int K;
    long long P, B, d_in, d_hidden, d_out;
    int n_blocks;
    int n_heads;            // residual-MLP model: attention heads per block, 0 = none
    long long seq_len;      //   tokens per sequence (attention only)
    float data_sigma;
    uint64_t seed;
};

size_t linreg_workspace_bytes(const ModelDims &d);
hipError_t launch_linreg_grad(const ModelDims &d, const float *theta, float *g, const float *wstar,
                              void *ws, float *loss, const DevState *st, hipStream_t s);

size_t mlp2_workspace_bytes(const ModelDims &d);
hipError_t launch_mlp2_grad(const ModelDims &d, const float *theta, float *g, const float *means,
                            void *ws, float *loss, const DevState *st, hipStream_t s);

size_t resmlp_workspace_bytes(const ModelDims &d);
hipError_t launch_resmlp_grad(const ModelDims &d, const float *theta, float *g, const float *teacher,
                              void *ws, float *loss, const DevState *st, hipStream_t s);

}  // namespace qsr
