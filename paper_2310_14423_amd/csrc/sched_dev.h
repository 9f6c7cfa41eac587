// sched_dev.h -- the device-side QSR scheduler's routines (arXiv 2310.14423, Sec. 2, Eq. (2), and the
// round bookkeeping of Alg. 2), shared by the scheduler kernels and by the averaging kernel that can
// close an iteration itself.
#pragma once
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
__device__ __forceinline__ long long get_H(const SchedParams &sp, long long t)
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

// End of an iteration (Alg. 2's counters): t += 1, h += 1; if that was the round's H-th local step,
// whose averaging the kernels before this have done (they test h + 1 == H), the round is logged and
// round s + 1 opened with its period from Eq. (2) at the new t.  One thread.
__device__ __forceinline__ void sched_advance(DevState *st, const SchedParams &sp, int expect_sync)
{
    const long long t = st->t + 1, h = st->h + 1, s = st->s;
    const int sync = (h == st->H) ? 1 : 0;
    if (expect_sync >= 0 && expect_sync != sync) st->mismatch = 1;
    st->t = t;
    if (sync) {
        sp.log_t[s] = t;
        sp.log_H[s] = st->H;
        st->s = s + 1;
        st->h = 0;
        st->H = get_H(sp, t);
    } else {
        st->h = h;
    }
}

}  // namespace qsr
