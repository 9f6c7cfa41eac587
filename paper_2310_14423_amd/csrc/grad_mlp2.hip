// grad_mlp2.hip -- local gradient (Eq. (1) of arXiv 2310.14423) of the two-layer perceptron
// workload for all K workers in batched launches.  Parameters of one worker are packed as
// W1 [d_in][d_hidden], b1 [d_hidden], W2 [d_hidden][d_out], b2 [d_out]; the gradient uses the
// same packing.  hidden = relu(x W1 + b1); logits = hidden W2 + b2; loss = mean softmax
// cross-entropy.  Inputs: label_i uniform over the classes, x_i = mean[label_i] + sigma*N(0,I),
// drawn per (worker, iteration) from Philox4x32-10.
#include "philox.h"
#include "qsr_internal.h"
#include "sgemm.h"

namespace qsr {

struct Mlp2Ws {
    float *X, *hid, *dhid, *logit;
    double *logit64;       // the logits before the softmax, in double precision (at most 16 classes)
    int *label;
};

static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

static Mlp2Ws carve(const ModelDims &d, void *ws, size_t *total)
{
    char *p = (char *)ws;
    size_t off = 0;
    Mlp2Ws w;
    size_t K = (size_t)d.K, B = (size_t)d.B;
    w.X = (float *)(p + off);     off += up256(K * B * d.d_in * sizeof(float));
    w.hid = (float *)(p + off);   off += up256(K * B * d.d_hidden * sizeof(float));
    w.dhid = (float *)(p + off);  off += up256(K * B * d.d_hidden * sizeof(float));
    w.logit = (float *)(p + off); off += up256(K * B * d.d_out * sizeof(float));
    w.logit64 = (double *)(p + off); off += up256(K * B * d.d_out * sizeof(double));
    w.label = (int *)(p + off);   off += up256(K * B * sizeof(int));
    if (total) *total = off;
    return w;
}

size_t mlp2_workspace_bytes(const ModelDims &d)
{
    size_t total = 0;
    carve(d, nullptr, &total);
    return total;
}

// Sample() in one pass: label c_i uniform over the classes, x_i = mu_{c_i} + sigma z.  One thread
// per group of four consecutive elements of a worker's [B][d_in] batch (the group is the Philox
// counter of the normal draws); the label of a row comes from word i % 4 of the label stream's
// group i / 4 and is recomputed by every thread that needs it, which is cheaper than a kernel of
// its own; the thread that holds a row's first element also stores the label for the loss.
__global__ __launch_bounds__(64) void mlp2_sample_kernel(float *__restrict__ X, int *__restrict__ label,
                                                         const float *__restrict__ means, long long B,
                                                         long long d_in, uint32_t classes, float sigma,
                                                         uint64_t seed, const DevState *__restrict__ st)
{
    const uint32_t t = (uint32_t)st->t;
    const uint32_t k = blockIdx.y;
    const long long n = B * d_in, groups = (n + 3) / 4;
    float *x = X + (long long)k * n;
    int *lab = label + (long long)k * B;
    auto label_of = [&](long long i) {
        const U4 r = draw4(seed, STREAM_LABEL, k, t, (uint32_t)(i >> 2));
        const uint32_t w = (i & 3) == 0 ? r.x : (i & 3) == 1 ? r.y : (i & 3) == 2 ? r.z : r.w;
        return (int)index_from_word(w, classes);
    };
    const long long stride = (long long)gridDim.x * 64;
    for (long long q = (long long)blockIdx.x * 64 + threadIdx.x; q < groups; q += stride) {
        const float4 z4 = normal4(seed, STREAM_X, k, t, (uint32_t)q);
        const float z[4] = {z4.x, z4.y, z4.z, z4.w};
        const long long p = q * 4;
        long long i = p / d_in, j = p - i * d_in;
        int c = label_of(i);
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (p + e < n) {
                if (j == 0) lab[i] = c;
                v[e] = z[e] * sigma + means[(long long)c * d_in + j];
                if (++j == d_in) {
                    j = 0; ++i;
                    if (e < 3 && p + e + 1 < n) c = label_of(i);
                }
            }
        }
        if ((n & 3) == 0) {
            *(float4 *)(x + p) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (p + e < n) x[p + e] = v[e];
        }
    }
}

// per sample: logits -> (softmax - onehot)/B; per worker: mean cross-entropy and, for at most
// CMAX classes, the output bias gradient (the column sums of the new array), which would otherwise
// be a launch of its own.  One block per worker, samples strided over its threads (d_out is small).
// ZT = double: the logits come in double precision and the maximum is subtracted in double before
// anything is rounded to fp32.  At the workload's step size the logits grow into the hundreds within
// a few iterations, where one fp32 ulp of a logit (6e-5 at 600) is the relative error of the
// probability computed from it; the difference to the largest logit is small and rounds harmlessly.
template <int CMAX, typename ZT>
__global__ __launch_bounds__(256) void mlp2_softmax_ce_kernel(const ZT *zin, float *dlogit,   // may alias
                                                              const int *__restrict__ label,
                                                              float *__restrict__ loss,
                                                              float *__restrict__ gbias, long long sG,
                                                              long long B, int C)
{
    __shared__ float red[4][CMAX + 1];
    const int k = blockIdx.x;
    const float invB = 1.0f / (float)B;
    float lsum = 0.f;
    float cs[CMAX > 0 ? CMAX : 1];
#pragma unroll
    for (int o = 0; o < CMAX; ++o) cs[o] = 0.f;
    for (long long i = threadIdx.x; i < B; i += 256) {
        const ZT *z = zin + ((long long)k * B + i) * C;
        float *dz_out = dlogit + ((long long)k * B + i) * C;
        const int y = label[(long long)k * B + i];
        ZT mx = z[0];
        for (int o = 1; o < C; ++o) mx = z[o] > mx ? z[o] : mx;
        float se = 0.f;
        for (int o = 0; o < C; ++o) se += expf((float)(z[o] - mx));
        lsum += logf(se) - (float)(z[y] - mx);
        const float inv = 1.0f / se;
        if (CMAX > 0) {
#pragma unroll
            for (int o = 0; o < CMAX; ++o)
                if (o < C) {
                    const float dz = (expf((float)(z[o] - mx)) * inv - (o == y ? 1.f : 0.f)) * invB;
                    dz_out[o] = dz;
                    cs[o] += dz;
                }
        } else {
            // also in place (ZT = float, dlogit = zin): an entry is read before it is overwritten
            for (int o = 0; o < C; ++o) dz_out[o] = (expf((float)(z[o] - mx)) * inv - (o == y ? 1.f : 0.f)) * invB;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lsum += __shfl_down(lsum, o, 64);
#pragma unroll
    for (int c = 0; c < CMAX; ++c)
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) cs[c] += __shfl_down(cs[c], o, 64);
    if ((threadIdx.x & 63) == 0) {
        red[threadIdx.x >> 6][CMAX] = lsum;
#pragma unroll
        for (int c = 0; c < CMAX; ++c) red[threadIdx.x >> 6][c] = cs[c];
    }
    __syncthreads();
    if (threadIdx.x == 0) loss[k] = (red[0][CMAX] + red[1][CMAX] + red[2][CMAX] + red[3][CMAX]) * invB;
    if (CMAX > 0 && (int)threadIdx.x < C)
        gbias[(long long)k * sG + threadIdx.x] = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

// out[k][j] = sum_i A[k][i][j]   (bias gradients).  One thread per column, rows added in ascending
// order; eight loads are in flight at a time, since the launch has too few wavefronts to hide the
// latency of one load per addition.
__global__ __launch_bounds__(256) void colsum_kernel(const float *__restrict__ A,
                                                     float *__restrict__ out, long long rows,
                                                     long long cols, long long sA, long long sOut)
{
    const int k = blockIdx.y;
    const long long j = (long long)blockIdx.x * 256 + threadIdx.x;
    if (j >= cols) return;
    const float *a = A + (long long)k * sA + j;
    float acc = 0.f;
    long long i = 0;
    for (; i + 8 <= rows; i += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = a[(i + u) * cols];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
    }
    for (; i < rows; ++i) acc += a[i * cols];
    out[(long long)k * sOut + j] = acc;
}

// C[k][i][0..N) = A[k][i][:] B[k] + bias[k] for an output of at most NMAX columns (the class
// logits), products and sums in double precision, result stored in double (see the loss kernel):
// one wavefront per row i, lanes strided over the contraction index, butterfly sum over the lanes
// (a fixed order).  The 64x64-tile kernel would run this shape on M/64 workgroups per worker with
// Kd/16 dependent steps each.
template <int NMAX>
__global__ __launch_bounds__(256) void skinny_bias_kernel(const float *__restrict__ A, long long sA,
                                                          const float *__restrict__ Bm, long long sB,
                                                          const float *__restrict__ bias, long long sBias,
                                                          double *__restrict__ C, long long sC,
                                                          int M, int N, int Kd)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long k = blockIdx.y;
    if (row >= M) return;                                   // whole wavefronts leave together
    const float *a = A + k * sA + (long long)row * Kd;
    const float *b = Bm + k * sB;
    double acc[NMAX];
#pragma unroll
    for (int n = 0; n < NMAX; ++n) acc[n] = 0.0;
    // four steps of the contraction are loaded before their products are added (in the same
    // ascending order): a launch of one wavefront per SIMD hides no load latency by itself
    for (int kk0 = lane; kk0 < Kd; kk0 += 256) {
        float av[4], bv[4][NMAX];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int kk = kk0 + 64 * u;
            const bool in = kk < Kd;
            av[u] = in ? a[kk] : 0.f;
            const float *br = b + (long long)(in ? kk : 0) * N;
#pragma unroll
            for (int n = 0; n < NMAX; ++n) bv[u][n] = n < N ? br[n] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (kk0 + 64 * u < Kd) {
#pragma unroll
                for (int n = 0; n < NMAX; ++n) acc[n] = fma((double)av[u], (double)bv[u][n], acc[n]);
            }
    }
    // Sum over the 64 lanes, NMAX = 16 columns at once: at each of the first four exchange steps a
    // lane keeps half of its columns and hands the other half to its partner (which keeps those), so
    // the values to exchange halve from step to step (8 + 4 + 2 + 1 exchanges, then two plain steps on
    // the one value left: 17 instead of 16 x 6).  Lane l ends up with the sum of column
    // 8 (l/32 % 2) + 4 (l/16 % 2) + 2 (l/8 % 2) + l/4 % 2.  A fixed order.
    static_assert(NMAX == 16, "the exchange pattern is written for 16 columns");
    double v8[8], v4[4], v2[2];
    {
        const bool up = (lane & 32) != 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const double keep = up ? acc[j + 8] : acc[j], send = up ? acc[j] : acc[j + 8];
            v8[j] = keep + __shfl_xor(send, 32, 64);
        }
    }
    {
        const bool up = (lane & 16) != 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const double keep = up ? v8[j + 4] : v8[j], send = up ? v8[j] : v8[j + 4];
            v4[j] = keep + __shfl_xor(send, 16, 64);
        }
    }
    {
        const bool up = (lane & 8) != 0;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const double keep = up ? v4[j + 2] : v4[j], send = up ? v4[j] : v4[j + 2];
            v2[j] = keep + __shfl_xor(send, 8, 64);
        }
    }
    double mine;
    {
        const bool up = (lane & 4) != 0;
        const double keep = up ? v2[1] : v2[0], send = up ? v2[0] : v2[1];
        mine = keep + __shfl_xor(send, 4, 64);
    }
    mine += __shfl_xor(mine, 2, 64);
    mine += __shfl_xor(mine, 1, 64);
    const int col = ((lane >> 5) & 1) * 8 + ((lane >> 4) & 1) * 4 + ((lane >> 3) & 1) * 2 + ((lane >> 2) & 1);
    if ((lane & 3) == 0 && col < N) C[k * sC + (long long)row * N + col] = mine + (double)bias[k * sBias + col];
}

hipError_t launch_mlp2_grad(const ModelDims &d, const float *theta, float *g, const float *means,
                            void *ws, float *loss, const DevState *st, hipStream_t s)
{
    const long long B = d.B, di = d.d_in, dh = d.d_hidden, dz = d.d_out, P = d.P;
    const int K = d.K;
    Mlp2Ws w = carve(d, ws, nullptr);
    const long long oW1 = 0, ob1 = di * dh, oW2 = ob1 + dh, ob2 = oW2 + dh * dz;
    hipError_t e;

    // Sample(): labels and inputs
    {
        long long bx = ((B * di + 3) / 4 + 63) / 64;
        if (bx > 0x7FFFFFFFll) bx = 0x7FFFFFFFll;
        mlp2_sample_kernel<<<dim3((unsigned)bx, (unsigned)K), 64, 0, s>>>(w.X, w.label, means, B, di, (uint32_t)dz,
                                                                        (float)d.data_sigma, d.seed, st);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    // forward
    GemmArgs a{};
    a.A = w.X; a.lda = di; a.sA = B * di;
    a.B = theta + oW1; a.ldb = dh; a.sB = P;
    a.C = w.hid; a.ldc = dh; a.sC = B * dh;
    a.M = (int)B; a.N = (int)dh; a.Kd = (int)di; a.bias = theta + ob1; a.sBias = P;
    if ((e = launch_sgemm<false, false, EPI_BIAS_RELU, true>(a, K, s)) != hipSuccess) return e;   // double accumulation

    a = GemmArgs{};
    a.A = w.hid; a.lda = dh; a.sA = B * dh;
    a.B = theta + oW2; a.ldb = dz; a.sB = P;
    a.C = w.logit; a.ldc = dz; a.sC = B * dz;
    a.M = (int)B; a.N = (int)dz; a.Kd = (int)dh; a.bias = theta + ob2; a.sBias = P;
    if (dz <= 16) {
        skinny_bias_kernel<16><<<dim3((unsigned)((B + 3) / 4), (unsigned)K), 256, 0, s>>>(
            w.hid, B * dh, theta + oW2, P, theta + ob2, P, w.logit64, B * dz, (int)B, (int)dz, (int)dh);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    } else if ((e = launch_sgemm<false, false, EPI_BIAS>(a, K, s)) != hipSuccess) return e;

    const bool bias_grad_in_loss = dz <= 16;
    if (bias_grad_in_loss)
        mlp2_softmax_ce_kernel<16, double><<<K, 256, 0, s>>>(w.logit64, w.logit, w.label, loss, g + ob2, P, B, (int)dz);
    else
        mlp2_softmax_ce_kernel<0, float><<<K, 256, 0, s>>>(w.logit, w.logit, w.label, loss, nullptr, 0, B, (int)dz);
    if ((e = hipGetLastError()) != hipSuccess) return e;

    // backward; w.logit now holds d loss / d logits
    a = GemmArgs{};                                        // gW2 = hid^T dlogits
    a.A = w.hid; a.lda = dh; a.sA = B * dh;
    a.B = w.logit; a.ldb = dz; a.sB = B * dz;
    a.C = g + oW2; a.ldc = dz; a.sC = P;
    a.M = (int)dh; a.N = (int)dz; a.Kd = (int)B;
    if ((e = launch_sgemm<true, false, EPI_NONE>(a, K, s)) != hipSuccess) return e;
    if (!bias_grad_in_loss) {
        colsum_kernel<<<dim3((unsigned)((dz + 255) / 256), (unsigned)K), 256, 0, s>>>(
            w.logit, g + ob2, B, dz, B * dz, P);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }

    a = GemmArgs{};                                        // dhid = (dlogits W2^T) * [hid > 0]
    a.A = w.logit; a.lda = dz; a.sA = B * dz;
    a.B = theta + oW2; a.ldb = dz; a.sB = P;
    a.C = w.dhid; a.ldc = dh; a.sC = B * dh;
    a.M = (int)B; a.N = (int)dh; a.Kd = (int)dz; a.aux = w.hid;
    if ((e = launch_sgemm<false, true, EPI_MASK_POS>(a, K, s)) != hipSuccess) return e;

    a = GemmArgs{};                                        // gW1 = X^T dhid
    a.A = w.X; a.lda = di; a.sA = B * di;
    a.B = w.dhid; a.ldb = dh; a.sB = B * dh;
    a.C = g + oW1; a.ldc = dh; a.sC = P;
    a.M = (int)di; a.N = (int)dh; a.Kd = (int)B;
    if ((e = launch_sgemm<true, false, EPI_NONE>(a, K, s)) != hipSuccess) return e;
    colsum_kernel<<<dim3((unsigned)((dh + 255) / 256), (unsigned)K), 256, 0, s>>>(
        w.dhid, g + ob1, B, dh, B * dh, P);
    return hipGetLastError();
}

}  // namespace qsr
