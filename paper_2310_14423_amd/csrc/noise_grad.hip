// noise_grad.hip -- bulk standard-normal fills from Philox4x32-10, keyed (seed; element/4,
// stream, worker k, iteration t).  With stream GRAD this is the local "gradient" of the
// optimizer-only workloads, g[k][p] = sigma * z, which stands in for Eq. (1) of arXiv 2310.14423
// where only the optimizer and averaging traffic is of interest; with stream X it draws the
// input features of the model workloads.
#include "philox.h"
#include "qsr_internal.h"

namespace qsr {

__global__ __launch_bounds__(64) void fill_normal_kernel(float *__restrict__ out, long long row_stride,
                                                          long long n, long long groups, float sigma,
                                                          uint32_t stream, uint64_t seed,
                                                          const DevState *__restrict__ st)
{
    const uint32_t t = (uint32_t)st->t;
    const uint32_t k = blockIdx.y;
    float *row = out + (long long)k * row_stride;
    const bool vec = ((n | row_stride) & 3) == 0;
    const long long stride = (long long)gridDim.x * 64;
    for (long long q = (long long)blockIdx.x * 64 + threadIdx.x; q < groups; q += stride) {
        float4 z = normal4(seed, stream, k, t, (uint32_t)q);
        z.x *= sigma; z.y *= sigma; z.z *= sigma; z.w *= sigma;
        long long p = q * 4;
        if (vec) {
            st_nt4((float4 *)(row + p), z);
        } else {
            row[p] = z.x;
            if (p + 1 < n) row[p + 1] = z.y;
            if (p + 2 < n) row[p + 2] = z.z;
            if (p + 3 < n) row[p + 3] = z.w;
        }
    }
}

hipError_t launch_fill_normal(float *out, long long row_stride, int K, long long n, float sigma,
                              uint32_t stream, uint64_t seed, const DevState *st, hipStream_t s)
{
    long long groups = (n + 3) / 4;
    long long bx = (groups + 63) / 64;            // one trip per one-wavefront workgroup
    if (bx > 0x7FFFFFFFll) bx = 0x7FFFFFFFll;
    dim3 grid((unsigned)bx, (unsigned)K);
    fill_normal_kernel<<<grid, 64, 0, s>>>(out, row_stride, n, groups, sigma, stream, seed, st);
    return hipGetLastError();
}

hipError_t launch_noise_grad(float *g, int K, long long P, float sigma, uint64_t seed,
                             const DevState *st, hipStream_t s)
{
    return launch_fill_normal(g, P, K, P, sigma, STREAM_GRAD, seed, st, s);
}

}  // namespace qsr
