// sgemm.h -- batched single-precision GEMM, LDS-tiled, for the small fp32 model workload
// (two-layer perceptron).  C[b] = op(A[b]) * op(B[b]) with optional epilogue; one launch covers
// all K workers (blockIdx.z).  64x64 output tile, 16-deep k-slabs, four wavefronts, each a 32x32
// block on the fp32 matrix cores (v_mfma_f32_32x32x2_f32: fp32 operands, fp32 accumulation, two
// k per instruction), global loads three slabs ahead in registers.  A long contraction is cut in
// two halves that two such groups of four wavefronts in one workgroup run side by side (KSPLIT =
// 2; the halves are added through LDS at the end).  Every global access is bounds-checked, so
// any M, N, Kd is accepted.  Fixed order: deterministic.
// F64: the same operands (fp32 in memory and LDS) multiplied and accumulated in double precision on
// the fp64 matrix cores (v_mfma_f64_16x16x4_f64, four 16x16 blocks per wavefront): products of fp32
// values are exact in double, so the result is the exact sum rounded once.  Used for the hidden
// layer's pre-activations, whose rounding errors the output layer and the softmax amplify by two to
// three orders of magnitude once the logits have grown into the hundreds.
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

typedef double f64x4_t __attribute__((ext_vector_type(4)));

template <bool TA, bool TB, int EPI, int KSPLIT, bool F64 = false>
__global__ __launch_bounds__(256 * KSPLIT) void sgemm_kernel(GemmArgs a)
{
    constexpr int TM = 64, TN = 64, TK = 16, PAD = 32;   // rows k and k+1 of a slab 32 banks apart
    __shared__ float As_all[KSPLIT][TK][TM + PAD];
    __shared__ float Bs_all[KSPLIT][TK][TN + PAD];
    // The workgroup is KSPLIT groups of 256 threads; group grp contracts over its own run of
    // slabs with its own LDS slabs.  With one workgroup of four wavefronts per compute unit (the
    // batch is 128 rows) every slab's load -> LDS -> barrier -> MFMA chain ran unhidden; a second
    // group per SIMD fills part of those gaps (hidden layer forward, 8 x 128 x 784 x 1024: 46 -> 37 us).
    const int grp = threadIdx.x >> 8, tid = threadIdx.x & 255;
    float (*As)[TM + PAD] = As_all[grp];
    float (*Bs)[TN + PAD] = Bs_all[grp];
    const int lane = tid & 63, wm = tid >> 7, wn = (tid >> 6) & 1;   // wavefront (wm, wn) owns a 32x32 block
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    const long long bz = blockIdx.z;
    const float *A = a.A + bz * a.sA;
    const float *B = a.B + bz * a.sB;
    typedef float f32x16_t __attribute__((ext_vector_type(16)));
    f32x16_t acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    f64x4_t dacc[2][2];                              // F64: 16x16 block (bi, bj) of the wavefront's 32x32
#pragma unroll
    for (int e = 0; e < 4; ++e) { dacc[0][0][e] = 0.0; dacc[0][1][e] = 0.0; dacc[1][0][e] = 0.0; dacc[1][1][e] = 0.0; }

    // Global loads run PF slabs ahead of the multiplication, in registers: these problems have few
    // workgroups per compute unit (the batch is 128 rows), so a slab's load latency is not hidden
    // by other wavefronts and, unprefetched, every one of the Kd/16 steps paid it in full
    // (timed on MI355X, 128 x 784 x 1024, 8 workers, with the products still on the vector ALUs:
    // 178 us per launch without, 98 us with; 46 us with the products on the matrix cores.  Six
    // slabs ahead or 32-deep slabs timed the same to slower).
    constexpr int PF = 3;
    constexpr int R = TK / 4;                       // elements of each operand per thread and slab
    float ra[PF][R], rb[PF][R];
    auto gload = [&](int k0, float (&xa)[R], float (&xb)[R]) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            int kk, m;
            if (TA) { m = tid & 63; kk = (tid >> 6) + 4 * r; }
            else    { kk = tid % TK; m = tid / TK + (256 / TK) * r; }
            int gm = m0 + m, gk = k0 + kk;
            float v = 0.f;
            if (gm < a.M && gk < a.Kd) v = TA ? A[(long long)gk * a.lda + gm] : A[(long long)gm * a.lda + gk];
            xa[r] = v;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            int kk, n;
            if (TB) { kk = tid % TK; n = tid / TK + (256 / TK) * r; }
            else    { n = tid & 63; kk = (tid >> 6) + 4 * r; }
            int gn = n0 + n, gk = k0 + kk;
            float v = 0.f;
            if (gn < a.N && gk < a.Kd) v = TB ? B[(long long)gn * a.ldb + gk] : B[(long long)gk * a.ldb + gn];
            xb[r] = v;
        }
    };
    auto sstore = [&](const float (&xa)[R], const float (&xb)[R]) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (TA) As[(tid >> 6) + 4 * r][tid & 63] = xa[r];
            else    As[tid % TK][tid / TK + (256 / TK) * r] = xa[r];
            if (TB) Bs[tid % TK][tid / TK + (256 / TK) * r] = xb[r];
            else    Bs[(tid >> 6) + 4 * r][tid & 63] = xb[r];
        }
    };
    // every group runs the same number of slabs (the barriers are the workgroup's); slabs past
    // Kd load zeros
    const int nslab = ((a.Kd + TK - 1) / TK + KSPLIT - 1) / KSPLIT;
    const int kbase = grp * nslab * TK;
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (u < nslab) gload(kbase + u * TK, ra[u], rb[u]);
    for (int s0 = 0; s0 < nslab; s0 += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int sl = s0 + u;                  // uniform over the workgroup
            if (sl < nslab) {
                sstore(ra[u], rb[u]);
                if (sl + PF < nslab) gload(kbase + (sl + PF) * TK, ra[u], rb[u]);
                __syncthreads();
                if constexpr (F64) {
                    // lane l supplies A[row l%16][k l/16] and B[k l/16][column l%16] of the instruction
#pragma unroll
                    for (int kk = 0; kk < TK; kk += 4) {
                        const int kr = kk + (lane >> 4), c = lane & 15;
                        const double a0 = (double)As[kr][wm * 32 + c], a1 = (double)As[kr][wm * 32 + 16 + c];
                        const double b0 = (double)Bs[kr][wn * 32 + c], b1 = (double)Bs[kr][wn * 32 + 16 + c];
                        dacc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, dacc[0][0], 0, 0, 0);
                        dacc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, dacc[0][1], 0, 0, 0);
                        dacc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, dacc[1][0], 0, 0, 0);
                        dacc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, dacc[1][1], 0, 0, 0);
                    }
                } else {
                    // lane l supplies A[row l%32][k l/32] and B[k l/32][column l%32] of the instruction
#pragma unroll
                    for (int kk = 0; kk < TK; kk += 2) {
                        const float av = As[kk + (lane >> 5)][wm * 32 + (lane & 31)];
                        const float bv = Bs[kk + (lane >> 5)][wn * 32 + (lane & 31)];
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc, 0, 0, 0);
                    }
                }
                __syncthreads();
            }
        }
    }

    float *C = a.C + bz * a.sC;
    if constexpr (F64) {
        if constexpr (KSPLIT > 1) {   // the other groups' partial sums, added in group order
            __shared__ double dpart[KSPLIT - 1][4][16][64];
            if (grp > 0) {
#pragma unroll
                for (int i = 0; i < 16; ++i) dpart[grp - 1][tid >> 6][i][lane] = dacc[i >> 3][(i >> 2) & 1][i & 3];
            }
            __syncthreads();
            if (grp > 0) return;
#pragma unroll
            for (int g = 0; g < KSPLIT - 1; ++g)
#pragma unroll
                for (int i = 0; i < 16; ++i) dacc[i >> 3][(i >> 2) & 1][i & 3] += dpart[g][tid >> 6][i][lane];
        }
        // accumulator element e of lane l is C[4*e + l/16][l%16] of its 16x16 block
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int bj = 0; bj < 2; ++bj)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int gm = m0 + wm * 32 + bi * 16 + 4 * e + (lane >> 4);
                    const int gn = n0 + wn * 32 + bj * 16 + (lane & 15);
                    if (gm >= a.M || gn >= a.N) continue;
                    double v = dacc[bi][bj][e];
                    if (EPI == EPI_BIAS_RELU || EPI == EPI_BIAS) v += (double)a.bias[bz * a.sBias + gn];
                    if (EPI == EPI_BIAS_RELU) v = v > 0.0 ? v : 0.0;
                    if (EPI == EPI_MASK_POS) v = a.aux[bz * a.sC + (long long)gm * a.ldc + gn] > 0.f ? v : 0.0;
                    C[(long long)gm * a.ldc + gn] = (float)v;
                }
    } else {
    if constexpr (KSPLIT > 1) {       // the other groups' partial sums, added in group order
        __shared__ float part[KSPLIT - 1][4][16][64];
        if (grp > 0) {
#pragma unroll
            for (int i = 0; i < 16; ++i) part[grp - 1][tid >> 6][i][lane] = acc[i];
        }
        __syncthreads();
        if (grp > 0) return;
#pragma unroll
        for (int g = 0; g < KSPLIT - 1; ++g)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] += part[g][tid >> 6][i][lane];
    }

    // accumulator element i of lane l is C[(i/4)*8 + (l/32)*4 + i%4][l%32] of the wavefront's block
    const int gn = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int gm = m0 + wm * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
        if (gm >= a.M || gn >= a.N) continue;
        float v = acc[i];
        if (EPI == EPI_BIAS_RELU || EPI == EPI_BIAS) v += a.bias[bz * a.sBias + gn];
        if (EPI == EPI_BIAS_RELU) v = v > 0.f ? v : 0.f;
        if (EPI == EPI_MASK_POS) v = a.aux[bz * a.sC + (long long)gm * a.ldc + gn] > 0.f ? v : 0.f;
        C[(long long)gm * a.ldc + gn] = v;
    }
    }
}

template <bool TA, bool TB, int EPI, bool F64 = false>
inline hipError_t launch_sgemm(const GemmArgs &a, int batch, hipStream_t s)
{
    dim3 grid((unsigned)((a.N + 63) / 64), (unsigned)((a.M + 63) / 64), (unsigned)batch);
    if (a.Kd >= 256) sgemm_kernel<TA, TB, EPI, 2, F64><<<grid, 512, 0, s>>>(a);
    else sgemm_kernel<TA, TB, EPI, 1, F64><<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace qsr
