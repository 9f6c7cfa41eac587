// grad_linreg.hip -- local gradient (Eq. (1) of arXiv 2310.14423) of the linear least-squares
// workload for all K workers: loss_k = 1/(2B) sum_i (x_i.w_k - y_i)^2 with fresh Gaussian
// inputs x_i and targets y_i = x_i.w* + sigma*noise per (worker, iteration).
//   1. X[k] <- N(0,1)                              (Philox, stream X: drawn by the kernel of step 2
//      itself when rows are whole groups of four draws, else by the bulk fill kernel)
//   2. r[k][i] = x_i.(w_k - w*) - sigma*eps_i      (one block per sample; the two inner
//      products are taken as one, which avoids cancellation when w_k is close to w*)
//   3. g[k][j] = (1/B) sum_i r[k][i] X[k][i][j];  loss[k] = 1/(2B) sum_i r^2
// The problem is tiny (K*B*d = 131072 inputs at the benchmark size): latency-bound, kept simple.
#include "philox.h"
#include "qsr_internal.h"

namespace qsr {

__device__ __forceinline__ float block_sum_256(float v, float *red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float s = red[0] + red[1] + red[2] + red[3];
    __syncthreads();
    return s;
}

// DRAW: the sample's inputs are drawn here (d a multiple of 4: the row is d/4 whole groups of the
// generator, the same counters and arithmetic as the fill kernel) and written to X for step 3.
template <bool DRAW>
__global__ __launch_bounds__(256) void linreg_residual_kernel(
    float *__restrict__ X, const float *__restrict__ theta, const float *__restrict__ wstar,
    float *__restrict__ r, long long B, long long d, float sigma, uint64_t seed,
    const DevState *__restrict__ st)
{
    __shared__ float red[4];
    const int k = blockIdx.y;
    const long long i = blockIdx.x;
    float *x = X + ((long long)k * B + i) * d;
    const float *w = theta + (long long)k * d;
    float acc = 0.f;
    if (DRAW) {
        const uint32_t t = (uint32_t)st->t;
        const long long q0 = i * (d >> 2);                       // first group of this row
        for (long long q = threadIdx.x; q < (d >> 2); q += 256) {
            const float4 z = normal4(seed, STREAM_X, (uint32_t)k, t, (uint32_t)(q0 + q));
            const long long j = q * 4;
            *(float4 *)(x + j) = z;
            const float4 wv = *(const float4 *)(w + j), ws = *(const float4 *)(wstar + j);
            acc = fmaf(z.x, wv.x - ws.x, acc); acc = fmaf(z.y, wv.y - ws.y, acc);
            acc = fmaf(z.z, wv.z - ws.z, acc); acc = fmaf(z.w, wv.w - ws.w, acc);
        }
    } else {
        for (long long j = threadIdx.x; j < d; j += 256) acc = fmaf(x[j], w[j] - wstar[j], acc);
    }
    float dot = block_sum_256(acc, red);
    if (threadIdx.x == 0) {
        float4 z = normal4(seed, STREAM_NOISE, (uint32_t)k, (uint32_t)st->t, (uint32_t)(i >> 2));
        float e = (i & 3) == 0 ? z.x : (i & 3) == 1 ? z.y : (i & 3) == 2 ? z.z : z.w;
        r[(long long)k * B + i] = dot - sigma * e;
    }
}

__global__ __launch_bounds__(256) void linreg_grad_kernel(
    const float *__restrict__ X, const float *__restrict__ r, float *__restrict__ g,
    float *__restrict__ loss, long long B, long long d)
{
    __shared__ float red[4];
    const int k = blockIdx.y;
    const long long j = (long long)blockIdx.x * 256 + threadIdx.x;
    const float *Xk = X + (long long)k * B * d;
    const float *rk = r + (long long)k * B;
    const float invB = 1.0f / (float)B;
    if (j < d) {
        // eight loads in flight at a time (the launch has too few wavefronts to hide the latency of
        // one load per addition); the additions stay in sample order
        float acc = 0.f;
        long long i = 0;
        for (; i + 8 <= B; i += 8) {
            float xv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) xv[u] = Xk[(i + u) * d + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = fmaf(rk[i + u], xv[u], acc);
        }
        for (; i < B; ++i) acc = fmaf(rk[i], Xk[i * d + j], acc);
        g[(long long)k * d + j] = acc * invB;
    }
    if (blockIdx.x == 0) {
        float a = 0.f;
        for (long long i = threadIdx.x; i < B; i += 256) a = fmaf(rk[i], rk[i], a);
        float s = block_sum_256(a, red);
        if (threadIdx.x == 0) loss[k] = 0.5f * s * invB;
    }
}

size_t linreg_workspace_bytes(const ModelDims &d)
{
    size_t x = (size_t)d.K * (size_t)d.B * (size_t)d.d_in * sizeof(float);
    size_t r = (size_t)d.K * (size_t)d.B * sizeof(float);
    return ((x + 255) & ~(size_t)255) + ((r + 255) & ~(size_t)255);
}

hipError_t launch_linreg_grad(const ModelDims &d, const float *theta, float *g, const float *wstar,
                              void *ws, float *loss, const DevState *st, hipStream_t s)
{
    float *X = (float *)ws;
    size_t xb = ((size_t)d.K * d.B * d.d_in * sizeof(float) + 255) & ~(size_t)255;
    float *r = (float *)((char *)ws + xb);
    hipError_t e;
    if ((d.d_in & 3) == 0) {
        linreg_residual_kernel<true><<<dim3((unsigned)d.B, (unsigned)d.K), 256, 0, s>>>(
            X, theta, wstar, r, d.B, d.d_in, d.data_sigma, d.seed, st);
    } else {
        e = launch_fill_normal(X, d.B * d.d_in, d.K, d.B * d.d_in, 1.0f, STREAM_X, d.seed, st, s);
        if (e != hipSuccess) return e;
        linreg_residual_kernel<false><<<dim3((unsigned)d.B, (unsigned)d.K), 256, 0, s>>>(
            X, theta, wstar, r, d.B, d.d_in, d.data_sigma, d.seed, st);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    linreg_grad_kernel<<<dim3((unsigned)((d.d_in + 255) / 256), (unsigned)d.K), 256, 0, s>>>(
        X, r, g, loss, d.B, d.d_in);
    return hipGetLastError();
}

}  // namespace qsr
