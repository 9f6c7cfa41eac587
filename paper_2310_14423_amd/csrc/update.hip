// update.hip -- fused multi-replica OPT update (Alg. 2's "OPT" line of arXiv 2310.14423, for
// all K workers in one launch).  The K rows share eta_t and every scalar, so the [K][P] buffers
// are treated as one vector of K*P elements.  The kernels are HBM-bound (AdamW: 16 B read +
// 12 B written per element; SGD: 12 B + 8 B): 128-bit accesses, several independent loads in
// flight per lane, streaming (non-temporal) hints because nothing is re-read within a step.
// Launch shape, from a sweep on MI355X at K*P = 0.96e9: one-wavefront workgroups that each make
// a single trip (no grid-stride loop) over 2 x 64 float4 per array reached 5.85 TB/s, against
// 5.0-5.1 TB/s for 256-thread blocks in a capped persistent grid and 5.77 TB/s for a plain
// copy kernel; non-temporal loads and stores were each worth 3-5 %.
#include "qsr_internal.h"

namespace qsr {

constexpr int UPD_THREADS = 64;
constexpr int UPD_UNROLL = 2;      // float4 per array per thread per trip

__device__ __forceinline__ float4 ldg_nt(const float4 *p) { return ld_nt4(p); }
__device__ __forceinline__ void stg_nt(float4 *p, float4 v) { st_nt4(p, v); }

// AdamW (decoupled weight decay, bias-corrected), in the order
//   m <- m + (1-b1)(g - m) ; v <- v + (1-b2)(g^2 - v)
//   theta <- theta - [ eta*lambda*theta + (eta/bc1) * m / (sqrt(v)/sqrt(bc2) + eps) ]
// The moment updates are written as one rounding on top of the old moment, and the decay and
// the Adam step are added before they are subtracted from theta, so that each state variable
// takes one rounding per step (keeps thousands of fp32 steps within 1e-5 of exact arithmetic).
__device__ __forceinline__ void adamw_elem(float &th, float g, float &m, float &v, float etalam,
                                           float stepsz, float rsq_bc2, float c1, float c2,
                                           float eps)
{
    m = fmaf(c1, g - m, m);
    v = fmaf(c2, fmaf(g, g, -v), v);
    float denom = fmaf(sqrtf(v), rsq_bc2, eps);
    float upd = (stepsz * m) / denom;
    th = th - fmaf(etalam, th, upd);
}

__global__ __launch_bounds__(UPD_THREADS) void update_adamw_kernel(
    float4 *__restrict__ theta, const float4 *__restrict__ g, float4 *__restrict__ m,
    float4 *__restrict__ v, long long n4, long long n, const DevState *__restrict__ st,
    const StepScalars *__restrict__ sc, float c1, float c2, float eps)
{
    const StepScalars s = sc[st->t];
    const long long stride = (long long)gridDim.x * UPD_THREADS * UPD_UNROLL;
    long long base = (long long)blockIdx.x * UPD_THREADS * UPD_UNROLL + threadIdx.x;
    for (; base < n4; base += stride) {
        float4 a[UPD_UNROLL], b[UPD_UNROLL], c[UPD_UNROLL], d[UPD_UNROLL];
#pragma unroll
        for (int u = 0; u < UPD_UNROLL; ++u) {
            long long i = base + (long long)u * UPD_THREADS;
            if (i < n4) { a[u] = ldg_nt(theta + i); b[u] = ldg_nt(g + i); c[u] = ldg_nt(m + i); d[u] = ldg_nt(v + i); }
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
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - n4 * 4)) {
        long long i = n4 * 4 + threadIdx.x;
        float *th = (float *)theta, *mm = (float *)m, *vv = (float *)v;
        const float *gg = (const float *)g;
        float a = th[i], c = mm[i], d = vv[i];
        adamw_elem(a, gg[i], c, d, s.x, s.y, s.z, c1, c2, eps);
        th[i] = a; mm[i] = c; vv[i] = d;
    }
}

// SGD with heavy-ball momentum and coupled weight decay:
//   g' = g + lambda*theta ; buf <- mu*buf + g' ; theta <- theta - eta*buf
__device__ __forceinline__ void sgdm_elem(float &th, float g, float &buf, float eta, float mu,
                                          float lambda)
{
    float gp = fmaf(lambda, th, g);
    buf = fmaf(mu, buf, gp);
    th = fmaf(-eta, buf, th);
}

__global__ __launch_bounds__(UPD_THREADS) void update_sgdm_kernel(
    float4 *__restrict__ theta, const float4 *__restrict__ g, float4 *__restrict__ buf,
    long long n4, long long n, const DevState *__restrict__ st,
    const StepScalars *__restrict__ sc, float mu, float lambda)
{
    const float eta = sc[st->t].x;
    const long long stride = (long long)gridDim.x * UPD_THREADS * UPD_UNROLL;
    long long base = (long long)blockIdx.x * UPD_THREADS * UPD_UNROLL + threadIdx.x;
    for (; base < n4; base += stride) {
        float4 a[UPD_UNROLL], b[UPD_UNROLL], c[UPD_UNROLL];
#pragma unroll
        for (int u = 0; u < UPD_UNROLL; ++u) {
            long long i = base + (long long)u * UPD_THREADS;
            if (i < n4) { a[u] = ldg_nt(theta + i); b[u] = ldg_nt(g + i); c[u] = ldg_nt(buf + i); }
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
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - n4 * 4)) {
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

hipError_t launch_update_adamw(float *theta, const float *g, float *m, float *v, long long n,
                               const DevState *st, const StepScalars *sc, float c1, float c2,
                               float eps, hipStream_t s)
{
    long long n4 = n / 4;
    update_adamw_kernel<<<update_grid(n4), UPD_THREADS, 0, s>>>(
        (float4 *)theta, (const float4 *)g, (float4 *)m, (float4 *)v, n4, n, st, sc, c1, c2, eps);
    return hipGetLastError();
}

hipError_t launch_update_sgdm(float *theta, const float *g, float *buf, long long n,
                              const DevState *st, const StepScalars *sc, float mu, float lambda,
                              hipStream_t s)
{
    long long n4 = n / 4;
    update_sgdm_kernel<<<update_grid(n4), UPD_THREADS, 0, s>>>(
        (float4 *)theta, (const float4 *)g, (float4 *)buf, n4, n, st, sc, mu, lambda);
    return hipGetLastError();
}

}  // namespace qsr
