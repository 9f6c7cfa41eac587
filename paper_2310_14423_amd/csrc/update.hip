// update.hip -- fused multi-replica OPT update (Alg. 2's "OPT" line of arXiv 2310.14423, for
// all K workers in one launch).  The K rows share eta_t and every scalar, so the [K][P] buffers
// are treated as one vector of K*P elements.  The kernels are HBM-bound (AdamW: 16 B read +
// 12 B written per element; SGD: 12 B + 8 B): 128-bit accesses, several independent loads in
// flight per lane, streaming (non-temporal) hints because nothing is re-read within a step.
// Launch shape, from a sweep on MI355X at K*P = 0.96e9: one-wavefront workgroups that each make
// a single trip (no grid-stride loop) over 2 x 64 float4 per array reached 5.85 TB/s, against
// 5.0-5.1 TB/s for 256-thread blocks in a capped persistent grid and 5.77 TB/s for a plain
// copy kernel; non-temporal loads and stores were each worth 3-5 %.
#include "opt_elem.h"
#include "sched_dev.h"
#include "philox.h"
#include "qsr_internal.h"

namespace qsr {

constexpr int UPD_THREADS = 64;
constexpr int UPD_UNROLL = 2;      // float4 per array per thread per trip

__device__ __forceinline__ float4 ldg_nt(const float4 *p) { return ld_nt4(p); }
__device__ __forceinline__ void stg_nt(float4 *p, float4 v) { st_nt4(p, v); }

// `fused_sync`: the context folds the averaging into the last local step of a round (see the
// *_sync kernels below), so the plain update leaves that step alone.
// CLIP: the launch has one grid row per worker (blockIdx.y), n4 and n are one worker's row, and
// the gradient is multiplied by that worker's clipping factor as it is read.
// NOISE (optimizer-only workloads): the gradient is not read but drawn here, g = sigma * N(0,1)
// from the same Philox counters and with the same arithmetic as fill_normal_kernel.  The separate
// fill is bound by its arithmetic (about 220 vector instructions per four normals), this kernel by
// HBM, and the draw hides completely behind the loads of theta, m and v (timed on MI355X at
// 16 x 60e6: 4.02 ms against 4.63 ms for the update that reads g plus 1.01 ms for the fill).
// One grid row per worker, like CLIP.  With `store` the draw is also written to the gradient
// buffer (4 B written in place of the 4 B read: 28 B per element as before, but the write-heavier
// mix runs at 5.5 TB/s instead of 5.8: 4.91 ms); without, the gradient never exists in HBM and
// the kernel moves 12 B read + 12 B written = 24 B per element.
struct NoiseDraw { float sigma; uint64_t seed; int store; };

// The scheduler's end-of-iteration step taken by the update kernel itself, on an iteration that
// does not end a round (the host's mirror says so; a disagreement is latched as a mismatch): the
// state is read from the copy every kernel of this iteration reads and the advanced state written
// to the other copy, which the next iteration's kernels are handed.  No kernel of this iteration
// reads that one, so no ordering between workgroups is needed, and the one-thread scheduler launch
// (4 us of dispatch latency, 3 % of a perceptron iteration) goes away.
__device__ __forceinline__ void tick_into(const DevState *st, DevState *st_next, const SchedParams &sp)
{
    DevState nx = *st;
    sched_advance(&nx, sp, 0);
    *st_next = nx;
}

template <bool CLIP, bool NOISE>
__global__ __launch_bounds__(UPD_THREADS) void update_adamw_kernel(
    float4 *__restrict__ theta, float4 *__restrict__ g, float4 *__restrict__ m,
    float4 *__restrict__ v, long long n4, long long n, const DevState *__restrict__ st,
    const StepScalars *__restrict__ sc, float c1, float c2, float eps, int fused_sync,
    const float *__restrict__ row_coef, NoiseDraw nd, DevState *__restrict__ st_next, SchedParams sp)
{
    if (st_next != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) tick_into(st, st_next, sp);
    if (fused_sync && st->h + 1 == st->H) return;
    float gs = 1.0f;
    if (CLIP || NOISE) {
        const long long off = (long long)blockIdx.y * n4;      // rows are 16-byte aligned here
        theta += off; g += off; m += off; v += off;
        if (CLIP) gs = row_coef[blockIdx.y];
    }
    const long long t = st->t;
    const StepScalars s = sc[t];
    const long long stride = (long long)gridDim.x * UPD_THREADS * UPD_UNROLL;
    long long base = (long long)blockIdx.x * UPD_THREADS * UPD_UNROLL + threadIdx.x;
    for (; base < n4; base += stride) {
        float4 a[UPD_UNROLL], b[UPD_UNROLL], c[UPD_UNROLL], d[UPD_UNROLL];
#pragma unroll
        for (int u = 0; u < UPD_UNROLL; ++u) {
            long long i = base + (long long)u * UPD_THREADS;
            if (i < n4) {
                a[u] = ldg_nt(theta + i); c[u] = ldg_nt(m + i); d[u] = ldg_nt(v + i);
                if (!NOISE) b[u] = ldg_nt(g + i);
            }
            if (CLIP) { b[u].x *= gs; b[u].y *= gs; b[u].z *= gs; b[u].w *= gs; }
        }
        if (NOISE) {
#pragma unroll
            for (int u = 0; u < UPD_UNROLL; ++u) {
                long long i = base + (long long)u * UPD_THREADS;
                if (i < n4) {
                    b[u] = normal4(nd.seed, STREAM_GRAD, blockIdx.y, (uint32_t)t, (uint32_t)i);
                    b[u].x *= nd.sigma; b[u].y *= nd.sigma; b[u].z *= nd.sigma; b[u].w *= nd.sigma;
                }
            }
            if (nd.store) {
#pragma unroll
                for (int u = 0; u < UPD_UNROLL; ++u) {
                    long long i = base + (long long)u * UPD_THREADS;
                    if (i < n4) stg_nt(g + i, b[u]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UPD_UNROLL; ++u) {
            long long i = base + (long long)u * UPD_THREADS;
            if (i < n4) {
                adamw_elem(a[u].x, b[u].x, c[u].x, d[u].x, s.x, s.y, s.z, c1, c2, eps);
                adamw_elem(a[u].y, b[u].y, c[u].y, d[u].y, s.x, s.y, s.z, c1, c2, eps);
                adamw_elem(a[u].z, b[u].z, c[u].z, d[u].z, s.x, s.y, s.z, c1, c2, eps);
                adamw_elem(a[u].w, b[u].w, c[u].w, d[u].w, s.x, s.y, s.z, c1, c2, eps);
                stg_nt(theta + i, a[u]); stg_nt(m + i, c[u]); stg_nt(v + i, d[u]);
            }
        }
    }
    // ragged tail (n not a multiple of 4): at most 3 elements, done by the first threads
    if (!CLIP && !NOISE && blockIdx.x == 0 && threadIdx.x < (int)(n - n4 * 4)) {
        long long i = n4 * 4 + threadIdx.x;
        float *th = (float *)theta, *mm = (float *)m, *vv = (float *)v;
        const float *gg = (const float *)g;
        float a = th[i], c = mm[i], d = vv[i];
        adamw_elem(a, gg[i], c, d, s.x, s.y, s.z, c1, c2, eps);
        th[i] = a; mm[i] = c; vv[i] = d;
    }
}

template <bool CLIP, bool NOISE>
__global__ __launch_bounds__(UPD_THREADS) void update_sgdm_kernel(
    float4 *__restrict__ theta, float4 *__restrict__ g, float4 *__restrict__ buf,
    long long n4, long long n, const DevState *__restrict__ st,
    const StepScalars *__restrict__ sc, float mu, float lambda, int fused_sync,
    const float *__restrict__ row_coef, NoiseDraw nd, DevState *__restrict__ st_next, SchedParams sp)
{
    if (st_next != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) tick_into(st, st_next, sp);
    if (fused_sync && st->h + 1 == st->H) return;
    float gs = 1.0f;
    if (CLIP || NOISE) {
        const long long off = (long long)blockIdx.y * n4;
        theta += off; g += off; buf += off;
        if (CLIP) gs = row_coef[blockIdx.y];
    }
    const long long t = st->t;
    const float eta = sc[t].x;
    const long long stride = (long long)gridDim.x * UPD_THREADS * UPD_UNROLL;
    long long base = (long long)blockIdx.x * UPD_THREADS * UPD_UNROLL + threadIdx.x;
    for (; base < n4; base += stride) {
        float4 a[UPD_UNROLL], b[UPD_UNROLL], c[UPD_UNROLL];
#pragma unroll
        for (int u = 0; u < UPD_UNROLL; ++u) {
            long long i = base + (long long)u * UPD_THREADS;
            if (i < n4) {
                a[u] = ldg_nt(theta + i); c[u] = ldg_nt(buf + i);
                if (!NOISE) b[u] = ldg_nt(g + i);
            }
            if (CLIP) { b[u].x *= gs; b[u].y *= gs; b[u].z *= gs; b[u].w *= gs; }
        }
        if (NOISE) {
#pragma unroll
            for (int u = 0; u < UPD_UNROLL; ++u) {
                long long i = base + (long long)u * UPD_THREADS;
                if (i < n4) {
                    b[u] = normal4(nd.seed, STREAM_GRAD, blockIdx.y, (uint32_t)t, (uint32_t)i);
                    b[u].x *= nd.sigma; b[u].y *= nd.sigma; b[u].z *= nd.sigma; b[u].w *= nd.sigma;
                }
            }
            if (nd.store) {
#pragma unroll
                for (int u = 0; u < UPD_UNROLL; ++u) {
                    long long i = base + (long long)u * UPD_THREADS;
                    if (i < n4) stg_nt(g + i, b[u]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UPD_UNROLL; ++u) {
            long long i = base + (long long)u * UPD_THREADS;
            if (i < n4) {
                sgdm_elem(a[u].x, b[u].x, c[u].x, eta, mu, lambda);
                sgdm_elem(a[u].y, b[u].y, c[u].y, eta, mu, lambda);
                sgdm_elem(a[u].z, b[u].z, c[u].z, eta, mu, lambda);
                sgdm_elem(a[u].w, b[u].w, c[u].w, eta, mu, lambda);
                stg_nt(theta + i, a[u]); stg_nt(buf + i, c[u]);
            }
        }
    }
    if (!CLIP && !NOISE && blockIdx.x == 0 && threadIdx.x < (int)(n - n4 * 4)) {
        long long i = n4 * 4 + threadIdx.x;
        float *th = (float *)theta, *bb = (float *)buf;
        const float *gg = (const float *)g;
        float a = th[i], c = bb[i];
        sgdm_elem(a, gg[i], c, eta, mu, lambda);
        th[i] = a; bb[i] = c;
    }
}

// One trip per workgroup; the kernels keep their stride loop so that any grid is correct, and
// the grid is only capped where it would overflow the launch limit.
static int update_grid(long long n4)
{
    long long per_block = (long long)UPD_THREADS * UPD_UNROLL;
    long long blocks = (n4 + per_block - 1) / per_block;
    const long long cap = 0x7FFFFFFFll;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

// ---------------------------------------------------------------------------------------------
// The last local step of a round and the averaging that follows it, in one pass (Alg. 2's OPT
// line for h = H-1 and its All-Reduce line): a lane owns four consecutive parameters, walks the
// K rows (ROWS of them in flight), updates each worker's state in place, adds the updated
// parameters up with the same error-free summation and in the same order as the averaging
// kernel, and writes the mean to all K rows.  AdamW then moves 16 B read + 8 B (m, v) + 4 B
// (mean) written = 28 B per replica-parameter on such a step instead of 28 + 8; SGD 12 + 8 = 20
// instead of 20 + 8.  Acts only when this step completes the round (decided on the device, like
// the averaging); results are bit-identical to update followed by average.
// ---------------------------------------------------------------------------------------------
constexpr int SYNC_ROWS = 4;
// 256 threads: these launches are skipped on the device in all but a handful of iterations, and a
// skipped launch then has four times fewer workgroups to retire than with one-wavefront blocks
constexpr int SYNC_THREADS = 256;

__global__ __launch_bounds__(SYNC_THREADS) void update_adamw_sync_kernel(
    float4 *__restrict__ theta, const float4 *__restrict__ g, float4 *__restrict__ m,
    float4 *__restrict__ v, int K, long long P4, const DevState *__restrict__ st,
    const StepScalars *__restrict__ sc, float c1, float c2, float eps, const float *__restrict__ row_coef)
{
    if (st->h + 1 != st->H) return;
    const StepScalars s = sc[st->t];
    const float fK = (float)K;
    const long long stride = (long long)gridDim.x * SYNC_THREADS;
    for (long long i = (long long)blockIdx.x * SYNC_THREADS + threadIdx.x; i < P4; i += stride) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f), cmp = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k0 = 0; k0 < K; k0 += SYNC_ROWS) {
            float4 a[SYNC_ROWS], b[SYNC_ROWS], c[SYNC_ROWS], d[SYNC_ROWS];
#pragma unroll
            for (int u = 0; u < SYNC_ROWS; ++u)
                if (k0 + u < K) {
                    const long long o = (long long)(k0 + u) * P4 + i;
                    a[u] = ldg_nt(theta + o); b[u] = ldg_nt(g + o); c[u] = ldg_nt(m + o); d[u] = ldg_nt(v + o);
                    if (row_coef != nullptr) { const float gs = row_coef[k0 + u]; b[u].x *= gs; b[u].y *= gs; b[u].z *= gs; b[u].w *= gs; }
                }
#pragma unroll
            for (int u = 0; u < SYNC_ROWS; ++u)
                if (k0 + u < K) {
                    const long long o = (long long)(k0 + u) * P4 + i;
                    adamw_elem(a[u].x, b[u].x, c[u].x, d[u].x, s.x, s.y, s.z, c1, c2, eps);
                    adamw_elem(a[u].y, b[u].y, c[u].y, d[u].y, s.x, s.y, s.z, c1, c2, eps);
                    adamw_elem(a[u].z, b[u].z, c[u].z, d[u].z, s.x, s.y, s.z, c1, c2, eps);
                    adamw_elem(a[u].w, b[u].w, c[u].w, d[u].w, s.x, s.y, s.z, c1, c2, eps);
                    stg_nt(m + o, c[u]); stg_nt(v + o, d[u]);
                    add_comp(acc.x, cmp.x, a[u].x); add_comp(acc.y, cmp.y, a[u].y);
                    add_comp(acc.z, cmp.z, a[u].z); add_comp(acc.w, cmp.w, a[u].w);
                }
        }
        const float4 mean = make_float4((acc.x + cmp.x) / fK, (acc.y + cmp.y) / fK,
                                        (acc.z + cmp.z) / fK, (acc.w + cmp.w) / fK);
        for (int k = 0; k < K; ++k) stg_nt(theta + (long long)k * P4 + i, mean);
    }
}

__global__ __launch_bounds__(SYNC_THREADS) void update_sgdm_sync_kernel(
    float4 *__restrict__ theta, const float4 *__restrict__ g, float4 *__restrict__ buf, int K,
    long long P4, const DevState *__restrict__ st, const StepScalars *__restrict__ sc, float mu,
    float lambda, const float *__restrict__ row_coef)
{
    if (st->h + 1 != st->H) return;
    const float eta = sc[st->t].x;
    const float fK = (float)K;
    const long long stride = (long long)gridDim.x * SYNC_THREADS;
    for (long long i = (long long)blockIdx.x * SYNC_THREADS + threadIdx.x; i < P4; i += stride) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f), cmp = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k0 = 0; k0 < K; k0 += SYNC_ROWS) {
            float4 a[SYNC_ROWS], b[SYNC_ROWS], c[SYNC_ROWS];
#pragma unroll
            for (int u = 0; u < SYNC_ROWS; ++u)
                if (k0 + u < K) {
                    const long long o = (long long)(k0 + u) * P4 + i;
                    a[u] = ldg_nt(theta + o); b[u] = ldg_nt(g + o); c[u] = ldg_nt(buf + o);
                    if (row_coef != nullptr) { const float gs = row_coef[k0 + u]; b[u].x *= gs; b[u].y *= gs; b[u].z *= gs; b[u].w *= gs; }
                }
#pragma unroll
            for (int u = 0; u < SYNC_ROWS; ++u)
                if (k0 + u < K) {
                    const long long o = (long long)(k0 + u) * P4 + i;
                    sgdm_elem(a[u].x, b[u].x, c[u].x, eta, mu, lambda);
                    sgdm_elem(a[u].y, b[u].y, c[u].y, eta, mu, lambda);
                    sgdm_elem(a[u].z, b[u].z, c[u].z, eta, mu, lambda);
                    sgdm_elem(a[u].w, b[u].w, c[u].w, eta, mu, lambda);
                    stg_nt(buf + o, c[u]);
                    add_comp(acc.x, cmp.x, a[u].x); add_comp(acc.y, cmp.y, a[u].y);
                    add_comp(acc.z, cmp.z, a[u].z); add_comp(acc.w, cmp.w, a[u].w);
                }
        }
        const float4 mean = make_float4((acc.x + cmp.x) / fK, (acc.y + cmp.y) / fK,
                                        (acc.z + cmp.z) / fK, (acc.w + cmp.w) / fK);
        for (int k = 0; k < K; ++k) stg_nt(theta + (long long)k * P4 + i, mean);
    }
}

// rows whose length is not a multiple of 4 are not 16-byte aligned: one element per lane
// (v == nullptr: SGD with momentum, m is its buffer, c1 = mu, c2 = lambda)
__global__ __launch_bounds__(SYNC_THREADS) void update_sync_scalar_kernel(
    float *__restrict__ theta, const float *__restrict__ g, float *__restrict__ m,
    float *__restrict__ v, int K, long long P, const DevState *__restrict__ st,
    const StepScalars *__restrict__ sc, float c1, float c2, float eps, const float *__restrict__ row_coef)
{
    if (st->h + 1 != st->H) return;
    const StepScalars s = sc[st->t];
    const float fK = (float)K;
    const long long stride = (long long)gridDim.x * SYNC_THREADS;
    for (long long i = (long long)blockIdx.x * SYNC_THREADS + threadIdx.x; i < P; i += stride) {
        float acc = 0.f, cmp = 0.f;
        for (int k = 0; k < K; ++k) {
            const long long o = (long long)k * P + i;
            float a = theta[o], c = m[o];
            const float gk = row_coef != nullptr ? g[o] * row_coef[k] : g[o];
            if (v != nullptr) {
                float d = v[o];
                adamw_elem(a, gk, c, d, s.x, s.y, s.z, c1, c2, eps);
                v[o] = d;
            } else {
                sgdm_elem(a, gk, c, s.x, c1, c2);
            }
            m[o] = c;
            add_comp(acc, cmp, a);
        }
        const float mean = (acc + cmp) / fK;
        for (int k = 0; k < K; ++k) theta[(long long)k * P + i] = mean;
    }
}

// clipped update of rows that are not 16-byte aligned (P not a multiple of 4): one element per
// lane, one grid row per worker (v == nullptr: SGD with momentum, c1 = mu, c2 = lambda)
__global__ __launch_bounds__(SYNC_THREADS) void update_clip_scalar_kernel(
    float *__restrict__ theta, const float *__restrict__ g, float *__restrict__ m,
    float *__restrict__ v, long long P, const DevState *__restrict__ st,
    const StepScalars *__restrict__ sc, float c1, float c2, float eps, int fused_sync,
    const float *__restrict__ row_coef)
{
    if (fused_sync && st->h + 1 == st->H) return;
    const StepScalars s = sc[st->t];
    const float gs = row_coef[blockIdx.y];
    const long long stride = (long long)gridDim.x * SYNC_THREADS;
    for (long long i = (long long)blockIdx.x * SYNC_THREADS + threadIdx.x; i < P; i += stride) {
        const long long o = (long long)blockIdx.y * P + i;
        float a = theta[o], c = m[o];
        if (v != nullptr) {
            float d = v[o];
            adamw_elem(a, g[o] * gs, c, d, s.x, s.y, s.z, c1, c2, eps);
            v[o] = d;
        } else {
            sgdm_elem(a, g[o] * gs, c, s.x, c1, c2);
        }
        theta[o] = a; m[o] = c;
    }
}

static int sync_grid(long long items)
{
    long long blocks = (items + SYNC_THREADS - 1) / SYNC_THREADS;
    const long long cap = 0x7FFFFFFFll;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

hipError_t launch_update_adamw_sync(float *theta, const float *g, float *m, float *v, int K, long long P,
                                    const DevState *st, const StepScalars *sc, float c1, float c2,
                                    float eps, const float *row_coef, hipStream_t s)
{
    if ((P & 3) == 0)
        update_adamw_sync_kernel<<<sync_grid(P / 4), SYNC_THREADS, 0, s>>>(
            (float4 *)theta, (const float4 *)g, (float4 *)m, (float4 *)v, K, P / 4, st, sc, c1, c2, eps, row_coef);
    else
        update_sync_scalar_kernel<<<sync_grid(P), SYNC_THREADS, 0, s>>>(theta, g, m, v, K, P, st, sc, c1, c2, eps,
                                                                        row_coef);
    return hipGetLastError();
}

hipError_t launch_update_sgdm_sync(float *theta, const float *g, float *buf, int K, long long P,
                                   const DevState *st, const StepScalars *sc, float mu, float lambda,
                                   const float *row_coef, hipStream_t s)
{
    if ((P & 3) == 0)
        update_sgdm_sync_kernel<<<sync_grid(P / 4), SYNC_THREADS, 0, s>>>(
            (float4 *)theta, (const float4 *)g, (float4 *)buf, K, P / 4, st, sc, mu, lambda, row_coef);
    else
        update_sync_scalar_kernel<<<sync_grid(P), SYNC_THREADS, 0, s>>>(theta, g, buf, nullptr, K, P, st, sc, mu,
                                                                        lambda, 0.f, row_coef);
    return hipGetLastError();
}

// row_coef != nullptr: clipped update, one grid row per worker
hipError_t launch_update_adamw(float *theta, float *g, float *m, float *v, int K, long long P,
                               const DevState *st, const StepScalars *sc, float c1, float c2,
                               float eps, bool fused_sync, const float *row_coef, hipStream_t s, DevState *st_next,
                               const SchedParams *sp)
{
    const SchedParams spv = sp ? *sp : SchedParams{};
    const int fs = fused_sync ? 1 : 0;
    const NoiseDraw none{0.f, 0, 0};
    if (row_coef == nullptr) {
        const long long n = (long long)K * P, n4 = n / 4;
        update_adamw_kernel<false, false><<<update_grid(n4), UPD_THREADS, 0, s>>>(
            (float4 *)theta, (float4 *)g, (float4 *)m, (float4 *)v, n4, n, st, sc, c1, c2, eps, fs, nullptr, none, st_next, spv);
    } else if ((P & 3) == 0) {
        update_adamw_kernel<true, false><<<dim3((unsigned)update_grid(P / 4), (unsigned)K), UPD_THREADS, 0, s>>>(
            (float4 *)theta, (float4 *)g, (float4 *)m, (float4 *)v, P / 4, P, st, sc, c1, c2, eps, fs, row_coef, none, st_next, spv);
    } else {
        update_clip_scalar_kernel<<<dim3((unsigned)sync_grid(P), (unsigned)K), SYNC_THREADS, 0, s>>>(
            theta, g, m, v, P, st, sc, c1, c2, eps, fs, row_coef);
    }
    return hipGetLastError();
}

hipError_t launch_update_sgdm(float *theta, float *g, float *buf, int K, long long P,
                              const DevState *st, const StepScalars *sc, float mu, float lambda,
                              bool fused_sync, const float *row_coef, hipStream_t s, DevState *st_next,
                              const SchedParams *sp)
{
    const SchedParams spv = sp ? *sp : SchedParams{};
    const int fs = fused_sync ? 1 : 0;
    const NoiseDraw none{0.f, 0, 0};
    if (row_coef == nullptr) {
        const long long n = (long long)K * P, n4 = n / 4;
        update_sgdm_kernel<false, false><<<update_grid(n4), UPD_THREADS, 0, s>>>(
            (float4 *)theta, (float4 *)g, (float4 *)buf, n4, n, st, sc, mu, lambda, fs, nullptr, none, st_next, spv);
    } else if ((P & 3) == 0) {
        update_sgdm_kernel<true, false><<<dim3((unsigned)update_grid(P / 4), (unsigned)K), UPD_THREADS, 0, s>>>(
            (float4 *)theta, (float4 *)g, (float4 *)buf, P / 4, P, st, sc, mu, lambda, fs, row_coef, none, st_next, spv);
    } else {
        update_clip_scalar_kernel<<<dim3((unsigned)sync_grid(P), (unsigned)K), SYNC_THREADS, 0, s>>>(
            theta, g, buf, nullptr, P, st, sc, mu, lambda, 0.f, fs, row_coef);
    }
    return hipGetLastError();
}

// The optimizer-only workloads' gradient g = sigma * N(0,1) drawn inside the update (P a multiple of 4)
hipError_t launch_update_adamw_noise(float *theta, float *g, float *m, float *v, int K, long long P,
                                     const DevState *st, const StepScalars *sc, float c1, float c2, float eps,
                                     float sigma, uint64_t seed, bool store_g, hipStream_t s, DevState *st_next,
                                     const SchedParams *sp)
{
    if ((P & 3) != 0) return hipErrorInvalidValue;
    const SchedParams spv = sp ? *sp : SchedParams{};
    update_adamw_kernel<false, true><<<dim3((unsigned)update_grid(P / 4), (unsigned)K), UPD_THREADS, 0, s>>>(
        (float4 *)theta, (float4 *)g, (float4 *)m, (float4 *)v, P / 4, P, st, sc, c1, c2, eps, 0, nullptr,
        NoiseDraw{sigma, seed, store_g ? 1 : 0}, st_next, spv);
    return hipGetLastError();
}

hipError_t launch_update_sgdm_noise(float *theta, float *g, float *buf, int K, long long P, const DevState *st,
                                    const StepScalars *sc, float mu, float lambda, float sigma, uint64_t seed,
                                    bool store_g, hipStream_t s, DevState *st_next, const SchedParams *sp)
{
    if ((P & 3) != 0) return hipErrorInvalidValue;
    const SchedParams spv = sp ? *sp : SchedParams{};
    update_sgdm_kernel<false, true><<<dim3((unsigned)update_grid(P / 4), (unsigned)K), UPD_THREADS, 0, s>>>(
        (float4 *)theta, (float4 *)g, (float4 *)buf, P / 4, P, st, sc, mu, lambda, 0, nullptr,
        NoiseDraw{sigma, seed, store_g ? 1 : 0}, st_next, spv);
    return hipGetLastError();
}

}  // namespace qsr
