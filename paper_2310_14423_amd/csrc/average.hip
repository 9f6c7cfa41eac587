// average.hip -- replica averaging: theta_k <- (1/K) sum_k theta_k for every worker k (the
// All-Reduce line of Alg. 2, arXiv 2310.14423), as a reduction over the K axis of the [K][P]
// buffer on one GPU.  HBM-bound: 4 B read + 4 B written per replica-parameter.
//
// K <= 32: a workgroup owns a tile of columns and stages it in LDS as [K][columns]: its wavefronts
// split the K rows between them (wavefront w copies rows w, w + W, ... with 128-bit loads, 1 or
// 2 KiB contiguous from each), and after a barrier every lane adds up its columns from LDS and
// the wavefront writes the mean back to the rows it loaded.  Any K: each lane owns four
// consecutive parameters and walks the K rows in registers, 16 in flight at a time.
// Timed on MI355X (HBM3E, 8 TB/s), the other three state arrays of a run allocated beside it, three
// passes each:
//                                       K = 16, P = 60e6     K = 32, P = 350e6
//   rows in registers, 64 threads         5.68-5.81 TB/s       5.27-5.31
//   rows in registers, 256 threads        5.55-5.58            5.18-5.22
//   LDS tile, 8 wavefronts x 1 KiB        5.79-5.80            5.49-5.50
//   LDS tile, 2 wavefronts x 2 KiB        5.64-5.70            5.58-5.59
//   LDS tile, 4 wavefronts x 2 KiB        5.61-5.64            5.52
//   K split over the lanes of a
//   wavefront, partial sums combined
//   with shuffles                         5.05-5.06            5.12-5.13
// (a plain copy kernel reaches 5.77 TB/s on this chip).  At K = 16 the register and the LDS variants
// are equal within the spread of a pass; at K = 32 the LDS tile gains 5 % because a wavefront touches
// fewer rows with longer runs (32 row loads in flight per lane cost the register variant its
// occupancy).  The shuffle variant loses because a wavefront then reads only 256 B from each row.
// Chosen: 8 x 1 KiB up to K = 16, 2 x 2 KiB up to K = 32.
//
// In every variant the sum runs over k in ascending order in fp32 with an error-free
// transformation of every addition (the rounding error of each partial sum is carried in a
// second accumulator), so the mean is accurate to about one rounding whatever K is, does not
// depend on the launch shape, all K rows receive the same bits, and averaging K identical rows
// returns that row when K is a power of two.
#include "opt_elem.h"
#include "qsr_internal.h"
#include "sched_dev.h"

namespace qsr {

constexpr int AVG_THREADS = 64;
constexpr int AVG_KU = 16;

// LDS-staged tile: W wavefronts, RUN x 64 float4 columns (RUN KiB contiguous per row and wavefront)
template <int KMAX, int W, int RUN>
__device__ __forceinline__ void average_tile_body(float *__restrict__ buf, int K, long long P4, float4 *avg_tile)
{
    constexpr int TC = RUN * 64;
    constexpr int RPW = (KMAX + W - 1) / W;          // rows per wavefront
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long c0 = (long long)blockIdx.x * TC;
    float4 *base = (float4 *)buf;
    float4 r[RPW][RUN];
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
        const int k = w + j * W;
        if (k < K) {
#pragma unroll
            for (int u = 0; u < RUN; ++u) {
                const long long c = c0 + u * 64 + lane;
                if (c < P4) r[j][u] = ld_nt4(base + (long long)k * P4 + c);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
        const int k = w + j * W;
        if (k < K) {
#pragma unroll
            for (int u = 0; u < RUN; ++u) avg_tile[k * TC + u * 64 + lane] = r[j][u];
        }
    }
    __syncthreads();
    float4 mean[RUN];
#pragma unroll
    for (int u = 0; u < RUN; ++u) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float4 cmp = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k = 0; k < K; ++k) {
            const float4 v = avg_tile[k * TC + u * 64 + lane];
            add_comp(acc.x, cmp.x, v.x); add_comp(acc.y, cmp.y, v.y);
            add_comp(acc.z, cmp.z, v.z); add_comp(acc.w, cmp.w, v.w);
        }
        const float fK = (float)K;
        mean[u] = make_float4((acc.x + cmp.x) / fK, (acc.y + cmp.y) / fK,
                              (acc.z + cmp.z) / fK, (acc.w + cmp.w) / fK);
    }
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
        const int k = w + j * W;
        if (k < K) {
#pragma unroll
            for (int u = 0; u < RUN; ++u) {
                const long long c = c0 + u * 64 + lane;
                if (c < P4) st_nt4(base + (long long)k * P4 + c, mean[u]);
            }
        }
    }
}

// ADVANCE: the launch also closes the iteration.  Every workgroup reads the scheduler state when it
// starts and takes a ticket when it is done; the one that draws the last ticket knows that all
// others have read the state, and advances it.
template <int KMAX, int W, int RUN, bool ADVANCE>
__global__ __launch_bounds__(64 * W) void average_rows_tile_kernel(
    float *__restrict__ buf, int K, long long P4, const DevState *st, DevState *st_adv, SchedParams sp)
{
    extern __shared__ float4 avg_tile[];            // [K][RUN * 64]
    const bool act = st == nullptr || st->h + 1 == st->H;   // the step that completes a round
    if (ADVANCE) {
        if (act) average_tile_body<KMAX, W, RUN>(buf, K, P4, avg_tile);
        __syncthreads();
        if (threadIdx.x == 0) {
            __threadfence();
            if (atomicAdd(&st_adv->ticket, 1u) == gridDim.x - 1) {
                st_adv->ticket = 0;
                sched_advance(st_adv, sp, -1);
            }
        }
        return;
    }
    if (!act) return;
    average_tile_body<KMAX, W, RUN>(buf, K, P4, avg_tile);
}

// any K: AVG_KU rows in flight at a time
__global__ __launch_bounds__(AVG_THREADS) void average_rows_vec4_kernel(
    float *__restrict__ buf, int K, long long P4, const DevState *__restrict__ st)
{
    if (st != nullptr && st->h + 1 != st->H) return;
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

// rows whose length is not a multiple of 4 are not 16-byte aligned: two elements per lane where the
// length is even, else one; AVG_KU rows in flight at a time (one load per addition, as it was first
// written, ran the perceptron's 8 x 814 090 parameters in 17.7 us: every load waited for the one before)
template <int V>
__global__ __launch_bounds__(AVG_THREADS) void average_rows_narrow_kernel(
    float *__restrict__ buf, int K, long long P, const DevState *__restrict__ st)
{
    if (st != nullptr && st->h + 1 != st->H) return;
    const float fK = (float)K;
    const long long PV = P / V;
    const long long stride = (long long)gridDim.x * AVG_THREADS;
    for (long long i = (long long)blockIdx.x * AVG_THREADS + threadIdx.x; i < PV; i += stride) {
        float acc[V], cmp[V];
#pragma unroll
        for (int v = 0; v < V; ++v) { acc[v] = 0.f; cmp[v] = 0.f; }
        for (int k0 = 0; k0 < K; k0 += AVG_KU) {
            float r[AVG_KU][V];
#pragma unroll
            for (int u = 0; u < AVG_KU; ++u)
                if (k0 + u < K) {
                    const float *src = buf + (long long)(k0 + u) * P + i * V;
                    if (V == 2) { const float2 t = *(const float2 *)src; r[u][0] = t.x; r[u][V - 1] = t.y; }
                    else r[u][0] = *src;
                }
#pragma unroll
            for (int u = 0; u < AVG_KU; ++u)
                if (k0 + u < K) {
#pragma unroll
                    for (int v = 0; v < V; ++v) add_comp(acc[v], cmp[v], r[u][v]);
                }
        }
        float mean[V];
#pragma unroll
        for (int v = 0; v < V; ++v) mean[v] = (acc[v] + cmp[v]) / fK;
        for (int k = 0; k < K; ++k) {
            float *dst = buf + (long long)k * P + i * V;
            if (V == 2) *(float2 *)dst = make_float2(mean[0], mean[V - 1]);
            else *dst = mean[0];
        }
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

template <int KMAX, int W, int RUN, bool ADVANCE>
static hipError_t launch_tile(float *buf, int K, long long P4, const DevState *st, DevState *st_adv, SchedParams sp,
                              hipStream_t s)
{
    const size_t lds = (size_t)K * RUN * 64 * sizeof(float4);
    static bool raised = false;                       // above the default only for K = 32 x 2 KiB
    if (lds > 48 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void *)average_rows_tile_kernel<KMAX, W, RUN, ADVANCE>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, KMAX * RUN * 64 * (int)sizeof(float4));
        if (e != hipSuccess) return e;
        raised = true;
    }
    average_rows_tile_kernel<KMAX, W, RUN, ADVANCE><<<avg_grid(P4, RUN * 64), 64 * W, lds, s>>>(buf, K, P4, st, st_adv, sp);
    return hipGetLastError();
}

// st != nullptr: the launch acts only on the step that completes a round (h + 1 == H in the device's
// scheduler state, read before the scheduler advances)
hipError_t launch_average_rows(float *buf, int K, long long P, const DevState *st, hipStream_t s)
{
    if ((P & 3) == 0) {
        const long long P4 = P / 4;
        if (P4 > 0x7FFFFFFFll * 64) return hipErrorInvalidValue;
        if (K <= 16) return launch_tile<16, 8, 1, false>(buf, K, P4, st, nullptr, SchedParams{}, s);
        if (K <= 32) return launch_tile<32, 2, 2, false>(buf, K, P4, st, nullptr, SchedParams{}, s);
        average_rows_vec4_kernel<<<avg_grid(P4, AVG_THREADS), AVG_THREADS, 0, s>>>(buf, K, P4, st);
    } else {
        if ((P & 1) == 0) average_rows_narrow_kernel<2><<<avg_grid(P / 2, AVG_THREADS), AVG_THREADS, 0, s>>>(buf, K, P, st);
        else average_rows_narrow_kernel<1><<<avg_grid(P, AVG_THREADS), AVG_THREADS, 0, s>>>(buf, K, P, st);
    }
    return hipGetLastError();
}

// few workgroups (a ticket each), rows that the tile kernel takes
bool average_can_advance(int K, long long P)
{
    return (P & 3) == 0 && K <= 32 && P / 4 <= 64 * 64;
}

hipError_t launch_average_rows_advance(float *buf, int K, long long P, DevState *st, SchedParams sp, hipStream_t s)
{
    if (!average_can_advance(K, P)) return hipErrorInvalidValue;
    if (K <= 16) return launch_tile<16, 8, 1, true>(buf, K, P / 4, st, st, sp, s);
    return launch_tile<32, 2, 2, true>(buf, K, P / 4, st, st, sp, s);
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
