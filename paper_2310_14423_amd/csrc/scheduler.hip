// scheduler.hip -- device-side QSR scheduler (arXiv 2310.14423, Sec. 2, Eq. (2), and the round
// bookkeeping of Alg. 2).  Single-thread kernels: the work is O(1) per iteration, what matters
// is that the decision "average now?" and the next period H are taken on the device, so the
// host enqueues steps without ever reading device state.
#include "qsr_internal.h"
#include "sched_dev.h"

namespace qsr {

__global__ void sched_init_kernel(DevState *st, SchedParams sp)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    st->t = 0; st->s = 0; st->h = 0;
    st->H = get_H(sp, 0);
    st->mismatch = 0; st->ticket = 0;
}

// resume: install a saved (t, s, h, H); log entries of earlier rounds are cleared
__global__ void sched_set_kernel(DevState *st, SchedParams sp, long long t, long long s, long long h,
                                 long long H)
{
    for (long long i = threadIdx.x; i < s; i += blockDim.x) { sp.log_t[i] = 0; sp.log_H[i] = 0; }
    if (threadIdx.x != 0) return;
    st->t = t; st->s = s; st->h = h; st->H = H;
    st->mismatch = 0; st->ticket = 0;
}

// the last launch of an iteration when no other kernel closes it
__global__ void sched_advance_kernel(DevState *st, SchedParams sp, int expect_sync)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    sched_advance(st, sp, expect_sync);
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
hipError_t launch_sched_advance(DevState *st, SchedParams sp, int expect_sync, hipStream_t s)
{
    sched_advance_kernel<<<1, 64, 0, s>>>(st, sp, expect_sync);
    return hipGetLastError();
}

}  // namespace qsr
