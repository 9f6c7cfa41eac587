// average.hip -- replica averaging: theta_k <- (1/K) sum_k theta_k for every worker k (the
// All-Reduce line of Alg. 2, arXiv 2310.14423), as a reduction over the K axis of the [K][P]
// buffer on one GPU.  HBM-bound: 4 B read + 4 B written per replica-parameter.  Each lane owns
// four consecutive parameters and walks the K rows with 128-bit loads, KU rows in flight at a
// time; a wavefront therefore reads 1 KiB contiguous from each row.  The sum runs over k in
// ascending order in fp32 with an error-free transformation of every addition (the rounding
// error of each partial sum is carried in a second accumulator), so the mean is accurate to
// about one rounding whatever K is, does not depend on the launch shape, all K rows receive the
// same bits, and averaging K identical rows returns that row when K is a power of two.
#include "opt_elem.h"
#include "qsr_internal.h"

namespace qsr {

constexpr int AVG_THREADS = 64;
constexpr int AVG_KU = 16;

// K <= KMAX: all K row loads of a column are issued before the first addition (fully unrolled,
// predicated on k < K), then K stores.  From a sweep on MI355X (K = 16 and 32, P = 60e6):
// one-wavefront workgroups making one trip each gave 5.7 TB/s (K = 16) and 5.5 TB/s (K = 32),
// 8-20 % above 256-thread blocks in a capped grid and above the chunked variant below.
// THREADS: 64 for the stand-alone entry point (fastest); the predicated in-run launch, which is
// skipped on the device in all but a handful of iterations, uses 256 so that a skipped launch
// has fewer workgroups to retire (0.013 ms instead of 0.05 ms at P = 60e6 with one trip each;
// the launcher caps the grid further) at the price of a few per cent on the launches that do average.
template <int KMAX, int THREADS>
__global__ __launch_bounds__(THREADS) void average_rows_full_kernel(
    float *__restrict__ buf, int K, long long P4, const DevState *__restrict__ st)
{
    if (st != nullptr && st->do_sync == 0) return;
    const float fK = (float)K;
    const long long stride = (long long)gridDim.x * THREADS;
    for (long long i = (long long)blockIdx.x * THREADS + threadIdx.x; i < P4; i += stride) {
        float4 *col = (float4 *)buf + i;
        float4 r[KMAX];
#pragma unroll
        for (int u = 0; u < KMAX; ++u)
            if (u < K) r[u] = ld_nt4(col + (long long)u * P4);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float4 cmp = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < KMAX; ++u)
            if (u < K) {
                add_comp(acc.x, cmp.x, r[u].x); add_comp(acc.y, cmp.y, r[u].y);
                add_comp(acc.z, cmp.z, r[u].z); add_comp(acc.w, cmp.w, r[u].w);
            }
        float4 mean = make_float4((acc.x + cmp.x) / fK, (acc.y + cmp.y) / fK,
                                  (acc.z + cmp.z) / fK, (acc.w + cmp.w) / fK);
#pragma unroll
        for (int u = 0; u < KMAX; ++u)
            if (u < K) st_nt4(col + (long long)u * P4, mean);
    }
}

// any K: AVG_KU rows in flight at a time
__global__ __launch_bounds__(AVG_THREADS) void average_rows_vec4_kernel(
    float *__restrict__ buf, int K, long long P4, const DevState *__restrict__ st)
{
    if (st != nullptr && st->do_sync == 0) return;
    const float fK = (float)K;
    const long long stride = (long long)gridDim.x * AVG_THREADS;
    for (long long i = (long long)blockIdx.x * AVG_THREADS + threadIdx.x; i < P4; i += stride) {
        float4 *col = (float4 *)buf + i;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float4 cmp = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k0 = 0; k0 < K; k0 += AVG_KU) {
            float4 r[AVG_KU];
#pragma unroll
            for (int u = 0; u < AVG_KU; ++u)
                if (k0 + u < K) r[u] = ld_nt4(col + (long long)(k0 + u) * P4);
#pragma unroll
            for (int u = 0; u < AVG_KU; ++u)
                if (k0 + u < K) {
                    add_comp(acc.x, cmp.x, r[u].x); add_comp(acc.y, cmp.y, r[u].y);
                    add_comp(acc.z, cmp.z, r[u].z); add_comp(acc.w, cmp.w, r[u].w);
                }
        }
        float4 mean = make_float4((acc.x + cmp.x) / fK, (acc.y + cmp.y) / fK,
                                  (acc.z + cmp.z) / fK, (acc.w + cmp.w) / fK);
        for (int k = 0; k < K; ++k) st_nt4(col + (long long)k * P4, mean);
    }
}

// rows whose length is not a multiple of 4 are not 16-byte aligned: one element per lane
__global__ __launch_bounds__(AVG_THREADS) void average_rows_scalar_kernel(
    float *__restrict__ buf, int K, long long P, const DevState *__restrict__ st)
{
    if (st != nullptr && st->do_sync == 0) return;
    const float fK = (float)K;
    const long long stride = (long long)gridDim.x * AVG_THREADS;
    for (long long i = (long long)blockIdx.x * AVG_THREADS + threadIdx.x; i < P; i += stride) {
        float acc = 0.f, cmp = 0.f;
        for (int k = 0; k < K; ++k) add_comp(acc, cmp, buf[(long long)k * P + i]);
        float mean = (acc + cmp) / fK;
        for (int k = 0; k < K; ++k) buf[(long long)k * P + i] = mean;
    }
}

static int avg_grid(long long items, int threads)
{
    long long blocks = (items + threads - 1) / threads;
    const long long cap = 0x7FFFFFFFll;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

hipError_t launch_average_rows(float *buf, int K, long long P, const DevState *st, hipStream_t s)
{
    if ((P & 3) == 0) {
        const long long P4 = P / 4;
        const int grid = avg_grid(P4, AVG_THREADS);
        // predicated in-run launches: a capped grid walked with a stride loop.  In a QSR run nearly
        // all of them are skipped on the device, and retiring 4096 workgroups costs 0.006 ms where
        // the 58 594 one-trip ones of P = 60e6 cost 0.016 ms; the few launches that do average run
        // 5 % slower for it
        const int grid256 = avg_grid(P4, 256) < 4096 ? avg_grid(P4, 256) : 4096;
        if (K <= 8) {
            if (st) average_rows_full_kernel<8, 256><<<grid256, 256, 0, s>>>(buf, K, P4, st);
            else average_rows_full_kernel<8, AVG_THREADS><<<grid, AVG_THREADS, 0, s>>>(buf, K, P4, st);
        } else if (K <= 32) {
            if (st) average_rows_full_kernel<32, 256><<<grid256, 256, 0, s>>>(buf, K, P4, st);
            else average_rows_full_kernel<32, AVG_THREADS><<<grid, AVG_THREADS, 0, s>>>(buf, K, P4, st);
        } else {
            average_rows_vec4_kernel<<<grid, AVG_THREADS, 0, s>>>(buf, K, P4, st);
        }
    } else {
        average_rows_scalar_kernel<<<avg_grid(P, AVG_THREADS), AVG_THREADS, 0, s>>>(buf, K, P, st);
    }
    return hipGetLastError();
}

// Alg. 2's initialisation theta_k <- theta_bar^(0): copy src [P] into each of the K rows
__global__ __launch_bounds__(256) void broadcast_rows_kernel(float *__restrict__ dst,
                                                             const float *__restrict__ src, int K,
                                                             long long P)
{
    const long long stride = (long long)gridDim.x * 256;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < P; i += stride) {
        float x = src[i];
        for (int k = 0; k < K; ++k) dst[(long long)k * P + i] = x;
    }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float *__restrict__ dst, long long n)
{
    const long long stride = (long long)gridDim.x * 256;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = 0.f;
}

hipError_t launch_broadcast_rows(float *dst, const float *src, int K, long long P, hipStream_t s)
{
    broadcast_rows_kernel<<<avg_grid(P, 256), 256, 0, s>>>(dst, src, K, P);
    return hipGetLastError();
}

hipError_t launch_fill_zero(float *dst, long long n, hipStream_t s)
{
    fill_zero_kernel<<<avg_grid(n, 256), 256, 0, s>>>(dst, n);
    return hipGetLastError();
}

}  // namespace qsr
