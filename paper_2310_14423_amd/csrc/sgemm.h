// sgemm.h -- batched single-precision GEMM, LDS-tiled, for the small fp32 model workload
// (two-layer perceptron).  C[b] = op(A[b]) * op(B[b]) with optional epilogue; one launch covers
// all K workers (blockIdx.z).  64x64 output tile, 16-deep k-slabs, four wavefronts, each a 32x32
// block on the fp32 matrix cores (v_mfma_f32_32x32x2_f32: fp32 operands, fp32 accumulation, two
// k per instruction), global loads three slabs ahead in registers.  A long contraction is cut in
// two halves that two such groups of four wavefronts in one workgroup run side by side (KSPLIT =
// 2; the halves are added through LDS at the end).  Every global access is bounds-checked, so
// any M, N, Kd is accepted.  Fixed order: deterministic.
// dgemm_nn_kernel: fp32 operands (row-major, not transposed) multiplied and accumulated in double
// precision on the fp64 matrix cores (v_mfma_f64_16x16x4_f64): products of fp32 values are exact in
// double, so the result is the exact sum rounded once.  Used for the hidden layer's
// pre-activations, whose rounding errors the output layer and the softmax amplify by two to three
// orders of magnitude once the logits have grown into the hundreds.
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

template <bool TA, bool TB, int EPI, int KSPLIT>
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

    // Global loads run PF slabs ahead of the multiplication, in registers: these problems have few
    // workgroups per compute unit (the batch is 128 rows), so a slab's load latency is not hidden
    // by other wavefronts and, unprefetched, every one of the Kd/16 steps paid it in full
    // (timed on MI355X, 128 x 784 x 1024, 8 workers, with the products still on the vector ALUs:
    // 178 us per launch without, 98 us with; 46 us with the products on the matrix cores.  Six
    // slabs ahead or 32-deep slabs timed the same to slower; 64-deep slabs one ahead, for the weight
    // gradient whose contraction is 128 long: 29.5 against 27.4 us; 64 x 256 tiles with four wavefronts
    // of 64 x 64 side by side, one fragment read per instruction: 30.4 us).
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
                    // lane l supplies A[row l%32][k l/32] and B[k l/32][column l%32] of the instruction
#pragma unroll
                for (int kk = 0; kk < TK; kk += 2) {
                    const float av = As[kk + (lane >> 5)][wm * 32 + (lane & 31)];
                    const float bv = Bs[kk + (lane >> 5)][wn * 32 + (lane & 31)];
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc, 0, 0, 0);
                }
                __syncthreads();
            }
        }
    }

    float *C = a.C + bz * a.sC;
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

template <bool TA, bool TB, int EPI>
inline hipError_t launch_sgemm(const GemmArgs &a, int batch, hipStream_t s)
{
    dim3 grid((unsigned)((a.N + 63) / 64), (unsigned)((a.M + 63) / 64), (unsigned)batch);
    if (a.Kd >= 256) sgemm_kernel<TA, TB, EPI, 2><<<grid, 512, 0, s>>>(a);
    else sgemm_kernel<TA, TB, EPI, 1><<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}

// C = epilogue(A B) in double precision, A [M][Kd] and B [Kd][N] fp32 and row-major, C fp32.
// 64x64 output tile per workgroup, four wavefronts of a 32x32 block each (2 x 2 instructions of
// 16x16x4), KSPLIT such groups side by side on their shares of the contraction, added through LDS at
// the end.  No LDS in the main loop and no barrier: a lane's share of an instruction's operands,
// A[row l%16][k l/16] and B[k l/16][column l%16], comes straight from global memory (a float4 of A
// along k feeds four instructions in a row, the matching four rows of B one element each; the
// order of k inside a group of 16 is a permutation, the same for both operands).  The LDS-tiled
// form above ran 8 x 128 x 784 x 1024 in 50.5 us with two groups; this one 52.2 us with two and
// 46.7 us with four (35 TFLOP/s; the instruction's measured issue rate is 47).
template <int EPI, int KSPLIT>
__global__ __launch_bounds__(256 * KSPLIT) void dgemm_nn_kernel(GemmArgs a)
{
    constexpr int PF = 3;
    const int grp = threadIdx.x >> 8, tid = threadIdx.x & 255;
    const int lane = tid & 63, wm = tid >> 7, wn = (tid >> 6) & 1;
    const int r = lane & 15, q = lane >> 4;
    const int m0 = blockIdx.y * 64 + wm * 32, n0 = blockIdx.x * 64 + wn * 32;
    const long long bz = blockIdx.z;
    const float *A = a.A + bz * a.sA;
    const float *B = a.B + bz * a.sB;
    const bool vecA = (a.lda & 3) == 0 && (((unsigned long long)A) & 15) == 0;
    const int ng = (a.Kd + 15) / 16, ngg = (ng + KSPLIT - 1) / KSPLIT;
    const int g0 = grp * ngg, g1 = min(ng, g0 + ngg);

    // Guarded loads: the compiler turns each into a short branch with a wait behind it, so the
    // PF groups "ahead" are in fact waited for where they are loaded, and the wavefronts of the
    // KSPLIT groups hide each other's latency.  Timed at 8 x 128 x 784 x 1024 (KSPLIT = 4): 46.7 us
    // this way; 56.6 us with clamped addresses and selects, 73.3 us with unconditional clamped loads
    // and the masks applied at the point of use (loads truly in flight three groups ahead; 62.0 us two
    // groups ahead, without register spills).
    struct Frag { float a[2][4]; float b[2][4]; };
    auto gload = [&](int g, Frag &f) {
        const int k = g * 16 + 4 * q;
#pragma unroll
        for (int bi = 0; bi < 2; ++bi) {
            const int gm = m0 + bi * 16 + r;
            const float *ar = A + (long long)gm * a.lda + k;
            if (gm < a.M && vecA && k + 3 < a.Kd) {
                const float4 v = *(const float4 *)ar;
                f.a[bi][0] = v.x; f.a[bi][1] = v.y; f.a[bi][2] = v.z; f.a[bi][3] = v.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) f.a[bi][j] = (gm < a.M && k + j < a.Kd) ? ar[j] : 0.f;
            }
        }
#pragma unroll
        for (int bj = 0; bj < 2; ++bj) {
            const int gn = n0 + bj * 16 + r;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                f.b[bj][j] = (gn < a.N && k + j < a.Kd) ? B[(long long)(k + j) * a.ldb + gn] : 0.f;
        }
    };
    f64x4_t dacc[2][2];                              // 16x16 block (bi, bj) of the wavefront's 32x32
#pragma unroll
    for (int e = 0; e < 4; ++e) { dacc[0][0][e] = 0.0; dacc[0][1][e] = 0.0; dacc[1][0][e] = 0.0; dacc[1][1][e] = 0.0; }
    auto multiply = [&](const Frag &f) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const double a0 = (double)f.a[0][j], a1 = (double)f.a[1][j];
            const double b0 = (double)f.b[0][j], b1 = (double)f.b[1][j];
            dacc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, dacc[0][0], 0, 0, 0);
            dacc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, dacc[0][1], 0, 0, 0);
            dacc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, dacc[1][0], 0, 0, 0);
            dacc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, dacc[1][1], 0, 0, 0);
        }
    };
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
                multiply(f);
            }
        }
    }

    float *C = a.C + bz * a.sC;
    if constexpr (KSPLIT > 1) {       // the groups' partial sums, added pairwise in a fixed order
        __shared__ double dpart[KSPLIT / 2][4][16][64];
#pragma unroll
        for (int stride = KSPLIT / 2; stride >= 1; stride >>= 1) {
            if (grp >= stride && grp < 2 * stride) {
#pragma unroll
                for (int i = 0; i < 16; ++i) dpart[grp - stride][tid >> 6][i][lane] = dacc[i >> 3][(i >> 2) & 1][i & 3];
            }
            __syncthreads();
            if (grp < stride) {
#pragma unroll
                for (int i = 0; i < 16; ++i) dacc[i >> 3][(i >> 2) & 1][i & 3] += dpart[grp][tid >> 6][i][lane];
            }
            __syncthreads();
        }
        if (grp > 0) return;
    }
    // accumulator element e of lane l is C[4*e + l/16][l%16] of its 16x16 block
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int gm = m0 + bi * 16 + 4 * e + q;
                const int gn = n0 + bj * 16 + r;
                if (gm >= a.M || gn >= a.N) continue;
                double v = dacc[bi][bj][e];
                if (EPI == EPI_BIAS_RELU || EPI == EPI_BIAS) v += (double)a.bias[bz * a.sBias + gn];
                if (EPI == EPI_BIAS_RELU) v = v > 0.0 ? v : 0.0;
                C[(long long)gm * a.ldc + gn] = (float)v;
            }
}

template <int EPI>
inline hipError_t launch_dgemm_nn(const GemmArgs &a, int batch, hipStream_t s)
{
    dim3 grid((unsigned)((a.N + 63) / 64), (unsigned)((a.M + 63) / 64), (unsigned)batch);
    // measured issue rate of the fp64 matrix instruction on MI355X: 33 TFLOP/s with one wavefront per
    // SIMD, 44 with two, 47 with four (registers only, four independent accumulators each)
    if (a.Kd >= 512) dgemm_nn_kernel<EPI, 4><<<grid, 1024, 0, s>>>(a);
    else if (a.Kd >= 128) dgemm_nn_kernel<EPI, 2><<<grid, 512, 0, s>>>(a);
    else dgemm_nn_kernel<EPI, 1><<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace qsr
