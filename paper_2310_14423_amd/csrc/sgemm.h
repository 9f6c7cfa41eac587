// sgemm.h -- batched single-precision GEMM on the vector ALUs, LDS-tiled, for the small fp32
// model workload (two-layer perceptron).  C[b] = op(A[b]) * op(B[b]) with optional epilogue;
// one launch covers all K workers (blockIdx.z).  64x64 output tile, 16-deep k-slabs, 256
// threads, 4x4 outputs per thread, global loads three slabs ahead in registers.  Every global
// access is bounds-checked, so any M, N, Kd is accepted.  fp32 accumulation in a fixed order: deterministic.
#pragma once
#include <hip/hip_runtime.h>

namespace qsr {

enum { EPI_NONE = 0, EPI_BIAS_RELU = 1, EPI_BIAS = 2, EPI_MASK_POS = 3 };

struct GemmArgs {
    const float *A, *B;
    float *C;
    int M, N, Kd;
    long long lda, ldb, ldc;
    long long sA, sB, sC;      // per-batch strides (elements)
    const float *bias;         // [N], per-batch stride sBias
    long long sBias;
    const float *aux;          // EPI_MASK_POS: same layout as C; C = aux > 0 ? acc : 0
};

template <bool TA, bool TB, int EPI>
__global__ __launch_bounds__(256) void sgemm_kernel(GemmArgs a)
{
    constexpr int TM = 64, TN = 64, TK = 16, PAD = 4;
    __shared__ float As[TK][TM + PAD];
    __shared__ float Bs[TK][TN + PAD];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    const long long bz = blockIdx.z;
    const float *A = a.A + bz * a.sA;
    const float *B = a.B + bz * a.sB;
    float acc[4][4] = {};

    // Global loads run PF slabs ahead of the multiplication, in registers: these problems have few
    // workgroups per compute unit (the batch is 128 rows), so a slab's load latency is not hidden
    // by other wavefronts and, unprefetched, every one of the Kd/16 steps paid it in full
    // (timed on MI355X, 128 x 784 x 1024, 8 workers: 178 us per launch without, 98 us with).
    // The order of the additions into acc is unchanged.
    constexpr int PF = 3;
    float ra[PF][4], rb[PF][4];
    auto gload = [&](int k0, float (&xa)[4], float (&xb)[4]) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int kk, m;
            if (TA) { m = tid & 63; kk = (tid >> 6) + 4 * r; }
            else    { kk = tid & 15; m = (tid >> 4) + 16 * r; }
            int gm = m0 + m, gk = k0 + kk;
            float v = 0.f;
            if (gm < a.M && gk < a.Kd) v = TA ? A[(long long)gk * a.lda + gm] : A[(long long)gm * a.lda + gk];
            xa[r] = v;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int kk, n;
            if (TB) { kk = tid & 15; n = (tid >> 4) + 16 * r; }
            else    { n = tid & 63; kk = (tid >> 6) + 4 * r; }
            int gn = n0 + n, gk = k0 + kk;
            float v = 0.f;
            if (gn < a.N && gk < a.Kd) v = TB ? B[(long long)gn * a.ldb + gk] : B[(long long)gk * a.ldb + gn];
            xb[r] = v;
        }
    };
    auto sstore = [&](const float (&xa)[4], const float (&xb)[4]) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (TA) As[(tid >> 6) + 4 * r][tid & 63] = xa[r];
            else    As[tid & 15][(tid >> 4) + 16 * r] = xa[r];
            if (TB) Bs[tid & 15][(tid >> 4) + 16 * r] = xb[r];
            else    Bs[(tid >> 6) + 4 * r][tid & 63] = xb[r];
        }
    };
    const int nslab = (a.Kd + TK - 1) / TK;
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (u < nslab) gload(u * TK, ra[u], rb[u]);
    for (int s0 = 0; s0 < nslab; s0 += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int sl = s0 + u;                  // uniform over the workgroup
            if (sl < nslab) {
                sstore(ra[u], rb[u]);
                if (sl + PF < nslab) gload((sl + PF) * TK, ra[u], rb[u]);
                __syncthreads();
#pragma unroll
                for (int kk = 0; kk < TK; ++kk) {
                    float4 av = *(const float4 *)&As[kk][ty * 4];
                    float4 bv = *(const float4 *)&Bs[kk][tx * 4];
                    float ar[4] = {av.x, av.y, av.z, av.w};
                    float br[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(ar[i], br[j], acc[i][j]);
                }
                __syncthreads();
            }
        }
    }

    float *C = a.C + bz * a.sC;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int gm = m0 + ty * 4 + i;
        if (gm >= a.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int gn = n0 + tx * 4 + j;
            if (gn >= a.N) continue;
            float v = acc[i][j];
            if (EPI == EPI_BIAS_RELU || EPI == EPI_BIAS) v += a.bias[bz * a.sBias + gn];
            if (EPI == EPI_BIAS_RELU) v = v > 0.f ? v : 0.f;
            if (EPI == EPI_MASK_POS) v = a.aux[bz * a.sC + (long long)gm * a.ldc + gn] > 0.f ? v : 0.f;
            C[(long long)gm * a.ldc + gn] = v;
        }
    }
}

template <bool TA, bool TB, int EPI>
inline hipError_t launch_sgemm(const GemmArgs &a, int batch, hipStream_t s)
{
    dim3 grid((unsigned)((a.N + 63) / 64), (unsigned)((a.M + 63) / 64), (unsigned)batch);
    sgemm_kernel<TA, TB, EPI><<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace qsr
