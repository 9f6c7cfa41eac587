// scheduler.hip -- device-side QSR scheduler (arXiv 2310.14423, Sec. 2, Eq. (2), and the round
// bookkeeping of Alg. 2).  Single-thread kernels: the work is O(1) per iteration, what matters
// is that the decision "average now?" and the next period H are taken on the device, so the
// host enqueues steps without ever reading device state.
#include "qsr_internal.h"

namespace qsr {

// Eq. (2): H = max{H_base, floor((alpha/eta_t)^2)} at the iteration t that starts a round.
//  - a round starting inside the warm-up looks at the first post-warm-up learning rate
//    ("Dealing with Learning Rate Warmup");
//  - the last round is cut so that training ends with a synchronization: H = T - t.
// Evaluated in double precision as one division and one multiplication (no pow, no fused
// operations), so that the integer result is reproducible bit for bit.  The same routine
// serves the schedules the paper compares with: a general integer power gamma (1: H ~ 1/eta,
// 3: the cubic rule of App. F) by repeated multiplication, constant H (gamma = 0), and the
// post-local schedule (H = 1 for rounds that start before a switching iteration) and the
// modified SWAP schedule of App. G (one last round from a switching iteration to T).
#pragma clang fp contract(off)
__device__ long long get_H(const SchedParams &sp, long long t)
{
    long long rem = sp.T - t;
    if (rem <= 0) return 0;
    if (sp.t_swap_start > 0 && t >= sp.t_swap_start) return rem;
    if (t < sp.t_local_start) return 1;
    if (sp.power == 0) return sp.H_base < rem ? sp.H_base : rem;
    long long te = t < sp.T_warm ? sp.T_warm : t;
    if (te >= sp.T) return rem;
    double e = sp.eta[te];
    if (!(e > 0.0)) return rem;
    double q = sp.alpha / e;
    double v = q;
    for (int i = 1; i < sp.power; ++i) v = v * q;
    if (!(v < (double)rem)) return rem;       // also catches inf / NaN
    long long H = (long long)floor(v);
    if (H < sp.H_base) H = sp.H_base;
    if (H > rem) H = rem;
    return H;
}

__global__ void sched_init_kernel(DevState *st, SchedParams sp)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    st->t = 0; st->s = 0; st->h = 0;
    st->H = get_H(sp, 0);
    st->do_sync = 0; st->pad = 0;
}

// resume: install a saved (t, s, h, H); log entries of earlier rounds are cleared
__global__ void sched_set_kernel(DevState *st, SchedParams sp, long long t, long long s, long long h,
                                 long long H)
{
    for (long long i = threadIdx.x; i < s; i += blockDim.x) { sp.log_t[i] = 0; sp.log_H[i] = 0; }
    if (threadIdx.x != 0) return;
    st->t = t; st->s = s; st->h = h; st->H = H;
    st->do_sync = 0; st->pad = 0;
}

// end of a local step (Alg. 2's inner loop counter)
__global__ void sched_tick_kernel(DevState *st)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    long long h = st->h + 1;
    st->t = st->t + 1;
    st->h = h;
    st->do_sync = (h == st->H) ? 1 : 0;
}

// after the averaging of round s: log it, open round s+1 (Alg. 2: t already advanced by H)
__global__ void sched_next_round_kernel(DevState *st, SchedParams sp)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    if (!st->do_sync) return;
    long long s = st->s, t = st->t;
    sp.log_t[s] = t;
    sp.log_H[s] = st->H;
    st->s = s + 1;
    st->h = 0;
    st->H = get_H(sp, t);
    st->do_sync = 0;
}

hipError_t launch_sched_init(DevState *st, SchedParams sp, hipStream_t s)
{
    sched_init_kernel<<<1, 64, 0, s>>>(st, sp);
    return hipGetLastError();
}
hipError_t launch_sched_set(DevState *st, SchedParams sp, long long t, long long s_, long long h, long long H,
                            hipStream_t s)
{
    sched_set_kernel<<<1, 256, 0, s>>>(st, sp, t, s_, h, H);
    return hipGetLastError();
}
hipError_t launch_sched_tick(DevState *st, hipStream_t s)
{
    sched_tick_kernel<<<1, 64, 0, s>>>(st);
    return hipGetLastError();
}
hipError_t launch_sched_next_round(DevState *st, SchedParams sp, hipStream_t s)
{
    sched_next_round_kernel<<<1, 64, 0, s>>>(st, sp);
    return hipGetLastError();
}

}  // namespace qsr
