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
    float *part;           // [K][tiles of 16 rows][17]: column sums of dlogit and the summed loss of a tile
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
    w.part = (float *)(p + off);  off += up256(K * ((B + 15) / 16) * 17 * sizeof(float));
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

// More than 16 classes: per sample, logits -> (softmax - onehot)/B in place; per worker, the mean
// cross-entropy.  One block per worker, samples strided over its threads.
__global__ __launch_bounds__(256) void mlp2_softmax_ce_kernel(float *__restrict__ z_dz,
                                                              const int *__restrict__ label,
                                                              float *__restrict__ loss, long long B, int C)
{
    __shared__ float red[4];
    const int k = blockIdx.x;
    const float invB = 1.0f / (float)B;
    float lsum = 0.f;
    for (long long i = threadIdx.x; i < B; i += 256) {
        float *z = z_dz + ((long long)k * B + i) * C;
        const int y = label[(long long)k * B + i];
        float mx = z[0];
        for (int o = 1; o < C; ++o) mx = fmaxf(mx, z[o]);
        float se = 0.f;
        for (int o = 0; o < C; ++o) se += expf(z[o] - mx);
        lsum += logf(se) - (z[y] - mx);
        const float inv = 1.0f / se;
        for (int o = 0; o < C; ++o) z[o] = (expf(z[o] - mx) * inv - (o == y ? 1.f : 0.f)) * invB;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lsum += __shfl_down(lsum, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = lsum;
    __syncthreads();
    if (threadIdx.x == 0) loss[k] = (red[0] + red[1] + red[2] + red[3]) * invB;
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

// Output layer forward and loss for at most 16 classes, one workgroup per 16 samples of a worker:
// logits = hid W2 + b2 with products and sums in double precision on the fp64 matrix cores (one
// 16x16x4 instruction covers 16 samples x 16 classes x 4 hidden units; the eight wavefronts take an
// eighth of the hidden units each and wavefront 0 adds the eight partial results in order), then
// the softmax of each row across the 16 lanes that hold it: the maximum is subtracted in double
// before anything is rounded to fp32.  At the workload's step size the logits grow into the hundreds
// within a few iterations, where one fp32 ulp of a logit (6e-5 at 600) would be the relative error
// of the probability computed from it; the difference to the largest logit is small and rounds
// harmlessly.  Written: dlogit = (softmax - onehot)/B, and per tile the column sums of dlogit and
// the summed cross-entropy (mlp2_out_bwd_kernel adds the tiles up).
__global__ __launch_bounds__(512) void mlp2_logits_ce_kernel(const float *__restrict__ hid,
                                                             const float *__restrict__ theta, long long P,
                                                             long long oW2, long long ob2,
                                                             const int *__restrict__ label,
                                                             float *__restrict__ dlogit,
                                                             float *__restrict__ part,
                                                             int B, int dh, int C)
{
    __shared__ double dpart[7][4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r = lane & 15, q = lane >> 4;
    const int k = blockIdx.y, row0 = blockIdx.x * 16;
    const float *A = hid + (long long)k * B * dh;
    const float *W = theta + (long long)k * P + oW2;
    const bool vec = (dh & 3) == 0 && (((unsigned long long)A) & 15) == 0;
    const int ng = (dh + 15) / 16, ngw = (ng + 7) / 8;
    const int g0 = w * ngw, g1 = min(ng, g0 + ngw);
    const int arow = row0 + r;

    // lane l supplies A[row l%16][k l/16] and B[k l/16][column l%16] of an instruction; a float4 of a
    // row of hid along k feeds four instructions, with the matching four rows of W2
    struct Frag { float a[4], b[4]; };
    auto gload = [&](int g, Frag &f) {
        const int kk = g * 16 + 4 * q;
        const float *ar = A + (long long)arow * dh + kk;
        if (arow < B && vec && kk + 3 < dh) {
            const float4 v = *(const float4 *)ar;
            f.a[0] = v.x; f.a[1] = v.y; f.a[2] = v.z; f.a[3] = v.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) f.a[j] = (arow < B && kk + j < dh) ? ar[j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) f.b[j] = (r < C && kk + j < dh) ? W[(long long)(kk + j) * C + r] : 0.f;
    };
    f64x4_t acc;
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = 0.0;
    constexpr int PF = 4;
    Frag fr[PF];
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (g0 + u < g1) gload(g0 + u, fr[u]);
    for (int gb = g0; gb < g1; gb += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int g = gb + u;                   // uniform over the wavefront
            if (g < g1) {
                const Frag f = fr[u];
                if (g + PF < g1) gload(g + PF, fr[u]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64((double)f.a[j], (double)f.b[j], acc, 0, 0, 0);
            }
        }
    }
    if (w > 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e) dpart[w - 1][e][lane] = acc[e];
    }
    __syncthreads();
    if (w > 0) return;
#pragma unroll
    for (int g = 0; g < 7; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += dpart[g][e][lane];

    // accumulator element e of lane l is the logit of sample row0 + 4e + l/16, class l%16
    const bool cin = r < C;
    const double bias = cin ? (double)theta[(long long)k * P + ob2 + r] : 0.0;
    const float invB = 1.0f / (float)B;
    float cs = 0.f, ls = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int row = row0 + 4 * e + q;
        const bool rin = row < B;
        const double z = cin ? acc[e] + bias : -1.7e308;
        double mx = z;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) { const double t = __shfl_xor(mx, o, 64); mx = t > mx ? t : mx; }
        const float zs = cin ? (float)(z - mx) : 0.f;
        const float ex = cin ? expf(zs) : 0.f;
        float se = ex;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) se += __shfl_xor(se, o, 64);
        const int y = rin ? label[(long long)k * B + row] : -1;
        float zy = r == y ? zs : 0.f;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) zy += __shfl_xor(zy, o, 64);
        const float dz = (ex * (1.0f / se) - (r == y ? 1.f : 0.f)) * invB;
        if (rin && cin) {
            dlogit[((long long)k * B + row) * C + r] = dz;
            cs += dz;
        }
        if (rin) ls += logf(se) - zy;
    }
    cs += __shfl_xor(cs, 16, 64); cs += __shfl_xor(cs, 32, 64);
    ls += __shfl_xor(ls, 16, 64); ls += __shfl_xor(ls, 32, 64);
    float *pt = part + ((long long)k * gridDim.x + blockIdx.x) * 17;
    if (lane < 16) pt[lane] = cs;
    if (lane == 0) pt[16] = ls;
}

// Output layer backward for at most 16 classes, one workgroup per 64 hidden units of a worker:
// gW2[j][c] = sum_i hid[i][j] dlogit[i][c], dhid[i][j] = [hid[i][j] > 0] sum_c dlogit[i][c] W2[j][c],
// gb1[j] = sum_i dhid[i][j]; a thread owns a hidden unit and every eighth sample (its loads of hid go
// out eight at a time before the first is used), the eight partial sums are added in
// order through LDS.  The first workgroup of a worker also adds up the tiles of
// mlp2_logits_ce_kernel: gb2 and the mean cross-entropy.  (These were three launches of the tiled
// GEMM and a column-sum kernel, 5 to 9 us each whatever they did.)
__global__ __launch_bounds__(512) void mlp2_out_bwd_kernel(const float *__restrict__ hid,
                                                           const float *__restrict__ dlogit,
                                                           const float *__restrict__ theta,
                                                           float *__restrict__ dhid, float *__restrict__ g,
                                                           long long P, long long oW2, long long ob1, long long ob2,
                                                           const float *__restrict__ part, int tiles,
                                                           float *__restrict__ loss, int B, int dh, int C)
{
    __shared__ __attribute__((aligned(16))) float dl_s[128][16];
    __shared__ float red[8][64][17];
    const int tid = threadIdx.x, tj = tid & 63, ti = tid >> 6;
    const int k = blockIdx.y, j0 = blockIdx.x * 64, j = j0 + tj;
    const bool jin = j < dh;
    float w2[16], gw[16], cs = 0.f;
#pragma unroll
    for (int c = 0; c < 16; ++c) {
        w2[c] = (jin && c < C) ? theta[(long long)k * P + oW2 + (long long)j * C + c] : 0.f;
        gw[c] = 0.f;
    }
    const float *hk = hid + (long long)k * B * dh;
    float *dk = dhid + (long long)k * B * dh;
    for (int i0 = 0; i0 < B; i0 += 128) {
        __syncthreads();
        for (int idx = tid; idx < 128 * 16; idx += 512) {
            const int rr = idx >> 4, c = idx & 15;
            dl_s[rr][c] = (i0 + rr < B && c < C) ? dlogit[((long long)k * B + i0 + rr) * C + c] : 0.f;
        }
        __syncthreads();
#pragma unroll 1
        for (int half = 0; half < 2; ++half) {
            float hv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + ti + 8 * (half * 8 + u);
                hv[u] = (jin && i < B) ? hk[(long long)i * dh + j] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int rr = ti + 8 * (half * 8 + u), i = i0 + rr;
                const float4 *dl4 = (const float4 *)dl_s[rr];
                const float4 x0 = dl4[0], x1 = dl4[1], x2 = dl4[2], x3 = dl4[3];
                const float dl[16] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w,
                                      x2.x, x2.y, x2.z, x2.w, x3.x, x3.y, x3.z, x3.w};
                float d = 0.f;
#pragma unroll
                for (int c = 0; c < 16; ++c) d = fmaf(dl[c], w2[c], d);
                d = hv[u] > 0.f ? d : 0.f;
                if (jin && i < B) dk[(long long)i * dh + j] = d;
                cs += d;
#pragma unroll
                for (int c = 0; c < 16; ++c) gw[c] = fmaf(hv[u], dl[c], gw[c]);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < 16; ++c) red[ti][tj][c] = gw[c];
    red[ti][tj][16] = cs;
    __syncthreads();
    float *gk = g + (long long)k * P;
    for (int idx = tid; idx < 64 * 17; idx += 512) {
        const int jj = idx / 17, c = idx - jj * 17;
        float v = red[0][jj][c];
#pragma unroll
        for (int t = 1; t < 8; ++t) v += red[t][jj][c];
        if (j0 + jj < dh) {
            if (c == 16) gk[ob1 + j0 + jj] = v;
            else if (c < C) gk[oW2 + (long long)(j0 + jj) * C + c] = v;
        }
    }
    if (blockIdx.x == 0 && tid < 17) {
        float v = 0.f;
        for (int t = 0; t < tiles; ++t) v += part[((long long)k * tiles + t) * 17 + tid];
        if (tid == 16) loss[k] = v * (1.0f / (float)B);
        else if (tid < C) gk[ob2 + tid] = v;
    }
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
    if ((e = launch_dgemm_nn<EPI_BIAS_RELU>(a, K, s)) != hipSuccess) return e;   // double accumulation

    if (dz <= 16) {
        // logits, softmax and loss in one launch; gW2, dhid, gb1 (and the sums that finish gb2 and
        // the loss) in a second
        const int tiles = (int)((B + 15) / 16);
        mlp2_logits_ce_kernel<<<dim3((unsigned)tiles, (unsigned)K), 512, 0, s>>>(
            w.hid, theta, P, oW2, ob2, w.label, w.logit, w.part, (int)B, (int)dh, (int)dz);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        mlp2_out_bwd_kernel<<<dim3((unsigned)((dh + 63) / 64), (unsigned)K), 512, 0, s>>>(
            w.hid, w.logit, theta, w.dhid, g, P, oW2, ob1, ob2, w.part, tiles, loss, (int)B, (int)dh, (int)dz);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    } else {
        a = GemmArgs{};
        a.A = w.hid; a.lda = dh; a.sA = B * dh;
        a.B = theta + oW2; a.ldb = dz; a.sB = P;
        a.C = w.logit; a.ldc = dz; a.sC = B * dz;
        a.M = (int)B; a.N = (int)dz; a.Kd = (int)dh; a.bias = theta + ob2; a.sBias = P;
        if ((e = launch_dgemm_nn<EPI_BIAS>(a, K, s)) != hipSuccess) return e;
        mlp2_softmax_ce_kernel<<<K, 256, 0, s>>>(w.logit, w.label, loss, B, (int)dz);
        if ((e = hipGetLastError()) != hipSuccess) return e;

        // backward; w.logit now holds d loss / d logits
        a = GemmArgs{};                                        // gW2 = hid^T dlogits
        a.A = w.hid; a.lda = dh; a.sA = B * dh;
        a.B = w.logit; a.ldb = dz; a.sB = B * dz;
        a.C = g + oW2; a.ldc = dz; a.sC = P;
        a.M = (int)dh; a.N = (int)dz; a.Kd = (int)B;
        if ((e = launch_sgemm<true, false, EPI_NONE>(a, K, s)) != hipSuccess) return e;
        colsum_kernel<<<dim3((unsigned)((dz + 255) / 256), (unsigned)K), 256, 0, s>>>(
            w.logit, g + ob2, B, dz, B * dz, P);
        if ((e = hipGetLastError()) != hipSuccess) return e;

        a = GemmArgs{};                                        // dhid = (dlogits W2^T) * [hid > 0]
        a.A = w.logit; a.lda = dz; a.sA = B * dz;
        a.B = theta + oW2; a.ldb = dz; a.sB = P;
        a.C = w.dhid; a.ldc = dh; a.sC = B * dh;
        a.M = (int)B; a.N = (int)dh; a.Kd = (int)dz; a.aux = w.hid;
        if ((e = launch_sgemm<false, true, EPI_MASK_POS>(a, K, s)) != hipSuccess) return e;
        colsum_kernel<<<dim3((unsigned)((dh + 255) / 256), (unsigned)K), 256, 0, s>>>(
            w.dhid, g + ob1, B, dh, B * dh, P);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }

    a = GemmArgs{};                                        // gW1 = X^T dhid
    a.A = w.X; a.lda = di; a.sA = B * di;
    a.B = w.dhid; a.ldb = dh; a.sB = B * dh;
    a.C = g + oW1; a.ldc = dh; a.sC = P;
    a.M = (int)di; a.N = (int)dh; a.Kd = (int)B;
    return launch_sgemm<true, false, EPI_NONE>(a, K, s);
}

}  // namespace qsr
