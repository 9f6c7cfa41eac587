// grad_resmlp.hip -- local gradient (Eq. (1) of arXiv 2310.14423) of the residual-MLP workload
// for all K workers, batched over the workers in every launch.  The workload has the MLP
// sub-block shapes of the paper's ViT-B (Sec. 4; width d, hidden width dh, L blocks):
//
//   x_0 = tokens [M][d] ~ N(0,1);  y = x_0 W_T / sqrt(d)
//   u_l = LayerNorm(x_l; gamma_l, beta_l);  h_l = u_l W1_l + b1_l;  a_l = gelu_erf(h_l)
//   x_l+1 = x_l + a_l W2_l + b2_l;  loss = 1/(2 M d) sum (x_L - y)^2
//
// The six GEMMs per block (2 forward, 2 data-gradient, 2 weight-gradient) run on the bf16
// matrix cores with fp32 accumulation (gemm_bf16.h); the residual stream, LayerNorm statistics,
// loss and all gradients stay fp32.  The forward and data-gradient GEMMs are brought to the
// K-contiguous "NT" form by keeping bf16 copies of the weights in both orientations; the
// weight-gradient GEMMs reduce over the token axis and read the same bf16 activations as they are
// ("TN" form, LDS transpose reads), so no transposed activation copies exist.  The bf16 weights
// and the bf16 activations that GEMM epilogues and the LayerNorm forward pass produce (LayerNorm
// output, GELU output and derivative, the gradient of the hidden layer) are stored in 32-row x
// 32-column blocks (gemm_bf16.h), written that way by their producers, so that the slab copies of
// the GEMMs read consecutive memory.  The bf16 copy of the residual gradient stays row-major (the
// LayerNorm backward pass that writes it lost more on 64-byte store pieces than its two GEMMs
// gained), and so does what the attention core reads and writes.
// Per-block parameter packing: gamma[d], beta[d], W1[d][dh], b1[dh], W2[dh][d], b2[d].
//
// With n_heads > 0 each block first runs the attention half of a ViT encoder block,
//   u = LayerNorm(x_l; gamma_a, beta_a);  q|k|v = u Wqkv + bqkv;
//   o = softmax(q k^T / sqrt(64)) v per head and sequence;  x_l' = x_l + o Wo + bo,
// its parameters gamma_a[d], beta_a[d], Wqkv[d][3d], bqkv[3d], Wo[d][d], bo[d] packed in front of
// the block's six arrays above: four more GEMMs forward/data-gradient and two weight-gradient
// GEMMs of the same kinds, and the attention core of attention.h.
#include "attention.h"
#include "gemm_bf16.h"
#include "gemm_pp.h"
#include "qsr_internal.h"

namespace qsr {

static inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

constexpr float LN_EPS = 1e-5f;
constexpr int WGRAD_SPLIT = 4;          // most ranges a weight gradient's token reduction is cut into
constexpr int LN_ROWS_PER_WAVE = 16;     // least token rows per wavefront of the LayerNorm backward pass

struct ResWs {
    // per-replica strides are the element counts of one replica's array
    // "sub" counts residual sub-blocks: L without attention, 2L with (attention, MLP, attention, ...)
    float *X;      long long sX;       // [sub+1][M][d]
    float *MU, *RSTD; long long sStat; // [sub][M]
    bf16_t *H;     long long sH;       // [L][M][dh]  gelu'(pre-activation)
    bf16_t *U;     long long sU;       // [sub][M][d] LayerNorm output
    bf16_t *A;     long long sA;       // [L][M][dh]  GELU output
    float *Y;      long long sY;       // [M][d]
    float *DX;     long long sDX;      // [M][d]
    bf16_t *DXb;   long long sDXb;     // [M][d]
    bf16_t *DH;    long long sDH;      // [M][dh]
    float *DU;     long long sDU;      // [M][d]
    bf16_t *W1b, *W1Tb, *W2b, *W2Tb; long long sW; // [L][blocked d x dh or dh x d] each
    long long mdB, mdhB;               // elements of one blocked [M][d] / [M][dh] activation
    long long wB[2];                   // elements of one blocked [d][dh] / [dh][d] weight
    bf16_t *WTt;                       // [d][d], shared: teacher map transposed
    float *PART;   long long sPART;    // [2][wave_rows][d] partial dgamma, dbeta
    float *LPART;  long long sLPART;   // loss partials
    bf16_t *ZERO;                      // 256 bytes of zeros (stand-in rows of ragged GEMM slabs)
    float *SPLITK, *SPLITKB;           // [K][WGRAD_SPLIT][largest weight matrix], [K][WGRAD_SPLIT][widest bias]
    // attention sub-blocks only
    bf16_t *QKV;   long long sQKV;     // [L][M][3d]
    bf16_t *O;     long long sO;       // [L][M][d]   attention output before the projection
    float *LSE;    long long sLSE;     // [L][heads][M]
    bf16_t *DO;    long long sDO;      // [M][d]
    bf16_t *DQKV;  long long sDQKV;    // [M][3d]
    bf16_t *Wqb, *WqTb; long long sWq; // [L][d*3d] each
    bf16_t *Wob, *WoTb; long long sWo; // [L][d*d] each
};

static ResWs carve(const ModelDims &dm, void *ws, size_t *total)
{
    const long long K = dm.K, M = dm.B, d = dm.d_in, dh = dm.d_hidden, L = dm.n_blocks;
    const long long heads = dm.n_heads, sub = heads > 0 ? 2 * L : L;
    char *p = (char *)ws;
    size_t off = 0;
    ResWs w;
    // Per-worker arrays are laid out [K][stride].  The natural strides of the benchmark size are
    // exact multiples of 512 KiB, which puts the 8 workers' arrays in phase with every power-of-two
    // interleaving of the memory channels: XCDs that sweep one worker each, at the same relative
    // offsets and the same time, would all sit on the same channels.  8448 extra bytes per worker
    // take them out of phase.
    auto padded = [&](long long n, size_t elt) { return (long long)(up256((size_t)n * elt) + 8448) / (long long)elt; };
    auto take = [&](long long per_replica, size_t elt, long long copies) {
        void *r = p + off;
        off += up256((size_t)per_replica * elt * (size_t)copies);
        return r;
    };
    // blocked arrays: token rows padded to a multiple of 256, weight rows likewise
    w.mdB = blk_elems(M, d); w.mdhB = blk_elems(M, dh);
    w.wB[0] = blk_elems(d, dh); w.wB[1] = blk_elems(dh, d);
    const long long wmax = w.wB[0] > w.wB[1] ? w.wB[0] : w.wB[1];
    w.sX = padded((sub + 1) * M * d, 4); w.X = (float *)take(w.sX, 4, K);
    w.sStat = padded(sub * M, 4);        w.MU = (float *)take(w.sStat, 4, K); w.RSTD = (float *)take(w.sStat, 4, K);
    w.sH = padded(L * w.mdhB, 2);        w.H = (bf16_t *)take(w.sH, 2, K);
    w.sU = padded(sub * w.mdB, 2);       w.U = (bf16_t *)take(w.sU, 2, K);
    w.sA = padded(L * w.mdhB, 2);        w.A = (bf16_t *)take(w.sA, 2, K);
    w.sY = padded(M * d, 4);             w.Y = (float *)take(w.sY, 4, K);
    w.sDX = padded(M * d, 4);            w.DX = (float *)take(w.sDX, 4, K);
    w.sDXb = padded(M * d, 2);           w.DXb = (bf16_t *)take(w.sDXb, 2, K);
    w.sDH = padded(w.mdhB, 2);           w.DH = (bf16_t *)take(w.sDH, 2, K);
    w.sDU = padded(w.mdB > M * d ? w.mdB : M * d, 4); w.DU = (float *)take(w.sDU, 4, K);
    w.sW = padded(L * wmax, 2);
    w.W1b = (bf16_t *)take(w.sW, 2, K);  w.W1Tb = (bf16_t *)take(w.sW, 2, K);
    w.W2b = (bf16_t *)take(w.sW, 2, K);  w.W2Tb = (bf16_t *)take(w.sW, 2, K);
    w.WTt = (bf16_t *)take(blk_elems(d, d), 2, 1);
    const long long wave_rows = (M + LN_ROWS_PER_WAVE - 1) / LN_ROWS_PER_WAVE;
    w.sPART = padded(2 * wave_rows * d, 4); w.PART = (float *)take(w.sPART, 4, K);
    w.sLPART = padded((M * d + 1023) / 1024, 4); w.LPART = (float *)take(w.sLPART, 4, K);
    w.ZERO = (bf16_t *)take(128, 2, 1);
    {
        const long long widest = heads > 0 && 3 * d > dh ? 3 * d : dh;
        w.SPLITK = (float *)take(K * WGRAD_SPLIT * d * widest, 4, 1);
        w.SPLITKB = (float *)take(K * WGRAD_SPLIT * widest, 4, 1);
    }
    w.QKV = w.O = w.DO = w.DQKV = w.Wqb = w.WqTb = w.Wob = w.WoTb = nullptr; w.LSE = nullptr;
    w.sQKV = w.sO = w.sLSE = w.sDO = w.sDQKV = w.sWq = w.sWo = 0;
    if (heads > 0) {
        w.sQKV = padded(L * M * 3 * d, 2);   w.QKV = (bf16_t *)take(w.sQKV, 2, K);
        w.sO = padded(L * M * d, 2);         w.O = (bf16_t *)take(w.sO, 2, K);
        w.sLSE = padded(L * heads * M, 4);   w.LSE = (float *)take(w.sLSE, 4, K);
        w.sDO = padded(M * d, 2);            w.DO = (bf16_t *)take(w.sDO, 2, K);
        w.sDQKV = padded(M * 3 * d, 2);      w.DQKV = (bf16_t *)take(w.sDQKV, 2, K);
        const long long wq = blk_elems(3 * d, d) > blk_elems(d, 3 * d) ? blk_elems(3 * d, d) : blk_elems(d, 3 * d);
        w.sWq = padded(L * wq, 2);                           // blocked [d][3d] and [3d][d]
        w.Wqb = (bf16_t *)take(w.sWq, 2, K); w.WqTb = (bf16_t *)take(w.sWq, 2, K);
        w.sWo = padded(L * blk_elems(d, d), 2);
        w.Wob = (bf16_t *)take(w.sWo, 2, K); w.WoTb = (bf16_t *)take(w.sWo, 2, K);
    }
    if (total) *total = off;
    return w;
}

size_t resmlp_workspace_bytes(const ModelDims &d)
{
    size_t total = 0;
    carve(d, nullptr, &total);
    return total;
}

// ---------------------------------------------------------------------------------------------
// layout / conversion kernels
// ---------------------------------------------------------------------------------------------

// in [R][C] (row stride ld_in) -> out [R][C] bf16 (optional) and outT [C][R] bf16, both in the
// blocked layout of gemm_bf16.h (R and C multiples of 32), 64x64 tiles through LDS.  Batch index
// blockIdx.z = z * n_inner + l: z with the element strides s_in, s_out, s_t (workers), l with the
// strides l_in (input) and l_out, l_t (the blocks of the model), so that one launch converts a weight
// of all blocks.
template <class TIn>
__global__ __launch_bounds__(256) void cvt_transpose_kernel(const TIn *__restrict__ in, long long ld_in,
                                                            long long s_in, long long l_in, bf16_t *__restrict__ out,
                                                            long long s_out, long long l_out, bf16_t *__restrict__ outT,
                                                            long long s_t, long long l_t, int R, int C, int n_inner)
{
    __shared__ bf16_t tile[64][66];
    const int z = blockIdx.z / n_inner, l = blockIdx.z - z * n_inner;
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    in += (long long)z * s_in + (long long)l * l_in;
    for (int r = ty; r < 64; r += 4) {
        bf16_t v = (bf16_t)0.0f;
        if (r0 + r < R && c0 + tx < C) {
            v = (bf16_t)in[(long long)(r0 + r) * ld_in + c0 + tx];
            if (out) out[(long long)z * s_out + (long long)l * l_out + blk_off(r0 + r, c0 + tx, C)] = v;
        }
        tile[r][tx] = v;
    }
    __syncthreads();
    if (outT) {
        for (int c = ty; c < 64; c += 4)
            if (c0 + c < C && r0 + tx < R)
                outT[(long long)z * s_t + (long long)l * l_t + blk_off(c0 + c, r0 + tx, R)] = tile[tx][c];
    }
}

template <class TIn>
static hipError_t launch_cvt_transpose(const TIn *in, long long ld_in, long long s_in, long long l_in, bf16_t *out,
                                       long long s_out, bf16_t *outT, long long s_t,
                                       int R, int C, int batch, int n_inner, hipStream_t s)
{
    if ((long long)batch * n_inner > 65535 || R % 32 != 0 || C % 32 != 0) return hipErrorInvalidValue;
    dim3 grid((unsigned)((C + 63) / 64), (unsigned)((R + 63) / 64), (unsigned)(batch * n_inner));
    cvt_transpose_kernel<TIn><<<grid, 256, 0, s>>>(in, ld_in, s_in, l_in, out, s_out, blk_elems(R, C), outT, s_t,
                                                   blk_elems(C, R), R, C, n_inner);
    return hipGetLastError();
}

// out[z] = bf16(in[z]) for a row-major [rows][d] fp32 array, written in the blocked layout; four
// elements per lane and trip (d a multiple of 4); blockIdx.y = worker
__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float *__restrict__ in, long long s_in,
                                                          bf16_t *__restrict__ out, long long s_out,
                                                          long long n4, int d)
{
    const float4 *src = (const float4 *)(in + (long long)blockIdx.y * s_in);
    bf16_t *dst = out + (long long)blockIdx.y * s_out;
    const long long stride = (long long)gridDim.x * 256;
    const int d4 = d >> 2;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        const float4 v = src[i];
        const bf16x4 b = {(bf16_t)v.x, (bf16_t)v.y, (bf16_t)v.z, (bf16_t)v.w};
        const long long row = i / d4;
        *(bf16x4 *)(dst + blk_off(row, (i - row * d4) * 4, d)) = b;
    }
}

// ---------------------------------------------------------------------------------------------
// LayerNorm
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// One wavefront per token row, the row held in registers as VPL float4 per lane (d <= 256 VPL,
// d a multiple of 32): statistics in fp32, output u = gamma*xhat + beta in bf16 (64-bit stores) in
// the blocked layout.
template <int VPL>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const float *__restrict__ X, long long sX,
                                                     const float *__restrict__ theta, long long sTh,
                                                     long long off_gamma, bf16_t *__restrict__ U,
                                                     long long sU, float *__restrict__ MU,
                                                     float *__restrict__ RSTD, long long sStat, int M, int d)
{
    const int z = blockIdx.y;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= M) return;
    const float *x = X + (long long)z * sX + (long long)row * d;
    const float *gam = theta + (long long)z * sTh + off_gamma, *bet = gam + d;
    float4 xv[VPL];
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < VPL; ++c) {
        const int j = (lane + c * 64) * 4;
        xv[c] = j < d ? *(const float4 *)(x + j) : make_float4(0.f, 0.f, 0.f, 0.f);
        s += (xv[c].x + xv[c].y) + (xv[c].z + xv[c].w);
    }
    const float mean = wave_sum(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int c = 0; c < VPL; ++c) {
        const int j = (lane + c * 64) * 4;
        if (j < d) {
            float a = xv[c].x - mean, b = xv[c].y - mean, e = xv[c].z - mean, f = xv[c].w - mean;
            q = fmaf(a, a, q); q = fmaf(b, b, q); q = fmaf(e, e, q); q = fmaf(f, f, q);
        }
    }
    const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + LN_EPS);
    bf16_t *u = U + (long long)z * sU;                  // blocked [M][d]
#pragma unroll
    for (int c = 0; c < VPL; ++c) {
        const int j = (lane + c * 64) * 4;
        if (j < d) {
            const float4 gv = *(const float4 *)(gam + j), bv = *(const float4 *)(bet + j);
            bf16x4 o = {(bf16_t)fmaf(gv.x, (xv[c].x - mean) * rstd, bv.x), (bf16_t)fmaf(gv.y, (xv[c].y - mean) * rstd, bv.y),
                        (bf16_t)fmaf(gv.z, (xv[c].z - mean) * rstd, bv.z), (bf16_t)fmaf(gv.w, (xv[c].w - mean) * rstd, bv.w)};
            *(bf16x4 *)(u + blk_off(row, j, d)) = o;
        }
    }
    if (lane == 0) { MU[(long long)z * sStat + row] = mean; RSTD[(long long)z * sStat + row] = rstd; }
}

__device__ __forceinline__ float4 load4f(const float *p) { return *(const float4 *)p; }
__device__ __forceinline__ float4 load4f(const bf16_t *p)
{
    const bf16x4 v = *(const bf16x4 *)p;
    return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
}

// Backward of LayerNorm plus the residual path, one wavefront per rows_per_wave token rows,
// VPL float4 per lane:
//   dn = du*gamma; dx_out = dx_in + rstd*(dn - mean(dn) - xhat*mean(dn*xhat))
// dx_out may be dx_in (each element is read and then written by the same lane): the launcher does
// that, so the update of dx is one stream of addresses instead of two.
// and per-wavefront partial sums of dgamma = sum_m du*xhat, dbeta = sum_m du (reduced by
// colsum_final_kernel).
template <int VPL, typename TDU>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const TDU *__restrict__ DU, long long sDU,
                                                     const float *__restrict__ X, long long sX,
                                                     const float *__restrict__ MU,
                                                     const float *__restrict__ RSTD, long long sStat,
                                                     const float *__restrict__ theta, long long sTh,
                                                     long long off_gamma, const float *DXin,
                                                     float *DXout, long long sDX,
                                                     bf16_t *__restrict__ DXb, long long sDXb,
                                                     float *__restrict__ PART, long long sPART,
                                                     int wave_rows, int rows_per_wave, int M, int d)
{
    const int z = blockIdx.y;
    const int wr = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (wr >= wave_rows) return;
    const float *gam = theta + (long long)z * sTh + off_gamma;
    float g[VPL][4], dg[VPL][4], db[VPL][4];
#pragma unroll
    for (int c = 0; c < VPL; ++c) {
        const int j = (lane + c * 64) * 4;
        const float4 gv = j < d ? *(const float4 *)(gam + j) : make_float4(0.f, 0.f, 0.f, 0.f);
        g[c][0] = gv.x; g[c][1] = gv.y; g[c][2] = gv.z; g[c][3] = gv.w;
#pragma unroll
        for (int e = 0; e < 4; ++e) { dg[c][e] = 0.f; db[c][e] = 0.f; }
    }
    const int r_end = min(M, (wr + 1) * rows_per_wave);
    for (int row = wr * rows_per_wave; row < r_end; ++row) {
        const long long o = (long long)row * d;
        const float mean = MU[(long long)z * sStat + row], rstd = RSTD[(long long)z * sStat + row];
        float xh[VPL][4], dn[VPL][4];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int c = 0; c < VPL; ++c) {
            const int j = (lane + c * 64) * 4;
            float4 duv = make_float4(0.f, 0.f, 0.f, 0.f), xv = make_float4(mean, mean, mean, mean);
            if (j < d) {
                duv = load4f(DU + (long long)z * sDU + o + j);     // row-major in either type: no GEMM reads it
                xv = *(const float4 *)(X + (long long)z * sX + o + j);
            }
            const float du[4] = {duv.x, duv.y, duv.z, duv.w}, xx[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                xh[c][e] = (xx[e] - mean) * rstd;
                dn[c][e] = du[e] * g[c][e];
                s1 += dn[c][e]; s2 = fmaf(dn[c][e], xh[c][e], s2);
                dg[c][e] = fmaf(du[e], xh[c][e], dg[c][e]); db[c][e] += du[e];
            }
        }
        const float m1 = wave_sum(s1) / (float)d, m2 = wave_sum(s2) / (float)d;
#pragma unroll
        for (int c = 0; c < VPL; ++c) {
            const int j = (lane + c * 64) * 4;
            if (j < d) {
                const float4 di = *(const float4 *)(DXin + (long long)z * sDX + o + j);
                float4 v;
                v.x = di.x + rstd * (dn[c][0] - m1 - xh[c][0] * m2);
                v.y = di.y + rstd * (dn[c][1] - m1 - xh[c][1] * m2);
                v.z = di.z + rstd * (dn[c][2] - m1 - xh[c][2] * m2);
                v.w = di.w + rstd * (dn[c][3] - m1 - xh[c][3] * m2);
                *(float4 *)(DXout + (long long)z * sDX + o + j) = v;
                bf16x4 b = {(bf16_t)v.x, (bf16_t)v.y, (bf16_t)v.z, (bf16_t)v.w};
                *(bf16x4 *)(DXb + (long long)z * sDXb + o + j) = b;
            }
        }
    }
    float *pg = PART + (long long)z * sPART + (long long)wr * d;
    float *pb = PART + (long long)z * sPART + ((long long)wave_rows + wr) * d;
#pragma unroll
    for (int c = 0; c < VPL; ++c) {
        const int j = (lane + c * 64) * 4;
        if (j < d) {
            *(float4 *)(pg + j) = make_float4(dg[c][0], dg[c][1], dg[c][2], dg[c][3]);
            *(float4 *)(pb + j) = make_float4(db[c][0], db[c][1], db[c][2], db[c][3]);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// column sums: final stage of the LayerNorm parameter gradients
// ---------------------------------------------------------------------------------------------
// out[z][j] = sum_c PART[z][c][j].  A workgroup owns 64 columns; its 4 wavefronts each sum a
// contiguous quarter of the chunks in ascending order and the four partial sums are added in
// wavefront order (fixed order: deterministic).
__global__ __launch_bounds__(256) void colsum_final_kernel(const float *__restrict__ PART, long long sPART,
                                                           float *__restrict__ out, long long sOut,
                                                           int chunks, int cols)
{
    // blockIdx.z selects the partial array (0: dgamma, 1: dbeta); the results are adjacent
    __shared__ float red[4][64];
    const int z = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = blockIdx.x * 64 + lane;
    const float *p = PART + (long long)z * sPART + (long long)blockIdx.z * chunks * cols;
    out += (long long)blockIdx.z * cols;
    const int per = (chunks + 3) / 4;
    const int c0 = wave * per, c1 = min(chunks, c0 + per);
    // 8 independent partial sums per lane (rows c0+u, c0+u+8, ...), so that 8 loads are in flight;
    // combined in a fixed order
    float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (j < cols) {
        int c = c0;
        for (; c + 8 <= c1; c += 8) {
            float r[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) r[u] = p[(long long)(c + u) * cols + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) a8[u] += r[u];
        }
        for (int u = 0; c < c1; ++c, ++u) a8[u] += p[(long long)c * cols + j];
    }
    const float acc = ((a8[0] + a8[1]) + (a8[2] + a8[3])) + ((a8[4] + a8[5]) + (a8[6] + a8[7]));
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && j < cols)
        out[(long long)z * sOut + j] = ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
}

// ---------------------------------------------------------------------------------------------
// loss
// ---------------------------------------------------------------------------------------------
// r = x_L - y; dx = r/(M d) (fp32 and bf16); per-block partial sums of r^2
__global__ __launch_bounds__(256) void loss_kernel(const float *__restrict__ XL, long long sX,
                                                   const float *__restrict__ Y, long long sY,
                                                   float *__restrict__ DX, long long sDX,
                                                   bf16_t *__restrict__ DXb, long long sDXb,
                                                   float *__restrict__ LPART, long long sLPART,
                                                   long long n, float inv)
{
    __shared__ float red[4];
    const int z = blockIdx.y;
    float acc = 0.f;
    const long long base = (long long)blockIdx.x * 1024;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        long long i = base + u * 256 + threadIdx.x;
        if (i < n) {
            float r = XL[(long long)z * sX + i] - Y[(long long)z * sY + i];
            acc = fmaf(r, r, acc);
            float g = r * inv;
            DX[(long long)z * sDX + i] = g;
            DXb[(long long)z * sDXb + i] = (bf16_t)g;
        }
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) LPART[(long long)z * sLPART + blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(256) void loss_final_kernel(const float *__restrict__ LPART, long long sLPART,
                                                         int nparts, float scale, float *__restrict__ loss)
{
    __shared__ float red[4];
    const int z = blockIdx.x;
    float acc = 0.f;
    for (int i = threadIdx.x; i < nparts; i += 256) acc += LPART[(long long)z * sLPART + i];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) loss[z] = (red[0] + red[1] + red[2] + red[3]) * scale;
}

// ---------------------------------------------------------------------------------------------
// GEMM epilogues
// ---------------------------------------------------------------------------------------------
// Phi(h) and phi(h) of the standard normal, for GELU(h) = h Phi(h) and its derivative
// Phi(h) + h phi(h).  erf by the rational-times-Gaussian formula 7.1.26 of Abramowitz & Stegun
// (|error| <= 1.5e-7, far below the bf16 rounding of the outputs); its exp(-x^2) with
// x = |h|/sqrt(2) is exactly the Gaussian factor phi needs, so one exponential serves both.
// Written to be cheap on the vector ALU (this runs in GEMM epilogues over 3e8 elements per
// launch): x is never formed (its scale is folded into the constants), the factors 1/2 and t of
// the tail are folded into the polynomial, the exponential is one exp2 of h*h times a constant,
// and the reflection for h < 0 is a sign copy.
__device__ __forceinline__ void gelu_parts(float h, float &cdf, float &pdf)
{
    // t = 1 / (1 + p x), p x = (0.3275911 / sqrt(2)) |h|
    const float t = __builtin_amdgcn_rcpf(fmaf(0.23164189f, fabsf(h), 1.0f));
    // exp(-x^2) = exp(-h^2/2) = 2^(h*h * (-log2(e)/2))
    const float ex = __builtin_amdgcn_exp2f(h * h * -0.72134752f);
    // (1 - erf(x))/2 = ex * t * (a1/2 + t (a2/2 + t (a3/2 + t (a4/2 + t a5/2))))
    float q = fmaf(0.5307027145f, t, -0.7265760135f);
    q = fmaf(q, t, 0.7107068705f);
    q = fmaf(q, t, -0.142248368f);
    q = fmaf(q, t, 0.127414796f);
    const float half_tail = q * t * ex;
    // Phi(h) = 1/2 + sign(h) (1/2 - half_tail)
    cdf = 0.5f + copysignf(0.5f - half_tail, h);
    pdf = 0.3989422804014327f * ex;
}

__device__ __forceinline__ bf16x4 pack4(float a, float b, float c, float d)
{
    bf16x4 r = {(bf16_t)a, (bf16_t)b, (bf16_t)c, (bf16_t)d};
    return r;
}

struct EpiScaleF32 {             // C = scale * acc
    float *C; long long ldc, sC; float scale;
    typedef NoAux Aux;
    __device__ Aux pre(int, int, int) const { return Aux{}; }
    __device__ void operator()(int z, int m, int n, const float (&v)[4], const Aux &) const
    {
        st_nt4((float4 *)(C + (long long)z * sC + (long long)m * ldc + n),
               make_float4(v[0] * scale, v[1] * scale, v[2] * scale, v[3] * scale));
    }
};
template <bool BLK>
struct EpiBf16 {                 // C = bf16(acc), row-major or blocked
    bf16_t *C; long long ldc, sC;
    typedef NoAux Aux;
    __device__ Aux pre(int, int, int) const { return Aux{}; }
    __device__ void operator()(int z, int m, int n, const float (&v)[4], const Aux &) const
    {
        const long long o = BLK ? blk_off(m, n, ldc) : (long long)m * ldc + n;
        *(bf16x4 *)(C + (long long)z * sC + o) = pack4(v[0], v[1], v[2], v[3]);
    }
};
struct EpiBiasBf16 {             // C = bf16(acc + bias)
    const float *bias; long long sBias; bf16_t *C; long long ldc, sC;
    typedef NoAux Aux;
    __device__ Aux pre(int, int, int) const { return Aux{}; }
    __device__ void operator()(int z, int m, int n, const float (&v)[4], const Aux &) const
    {
        const float4 b = *(const float4 *)(bias + (long long)z * sBias + n);
        *(bf16x4 *)(C + (long long)z * sC + (long long)m * ldc + n) = pack4(v[0] + b.x, v[1] + b.y, v[2] + b.z, v[3] + b.w);
    }
};
struct EpiBiasGelu {             // h = acc + b1; H = bf16(gelu'(h)); A = bf16(gelu(h)), both blocked
    // The backward pass needs h only through gelu'(h) = Phi(h) + h phi(h), and both factors are at
    // hand here: storing the derivative instead of h costs two instructions per element now and
    // saves the whole GELU evaluation in the data-gradient epilogue.
    const float *bias; long long sBias; bf16_t *H; long long sH; bf16_t *A; long long sA; long long ld;
    typedef NoAux Aux;
    __device__ Aux pre(int, int, int) const { return Aux{}; }
    __device__ void operator()(int z, int m, int n, const float (&v)[4], const Aux &) const
    {
        const float4 b = *(const float4 *)(bias + (long long)z * sBias + n);
        const float h[4] = {v[0] + b.x, v[1] + b.y, v[2] + b.z, v[3] + b.w};
        float a[4], dg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float c, pdf;
            gelu_parts(h[i], c, pdf);
            a[i] = h[i] * c;
            dg[i] = fmaf(h[i], pdf, c);
        }
        const long long o = blk_off(m, n, ld);
        __builtin_nontemporal_store(pack4(dg[0], dg[1], dg[2], dg[3]), (bf16x4 *)(H + (long long)z * sH + o));
        __builtin_nontemporal_store(pack4(a[0], a[1], a[2], a[3]), (bf16x4 *)(A + (long long)z * sA + o));
    }
};
struct EpiBiasResidual {         // x_out = x_in + acc + b2
    const float *bias; long long sBias; const float *Xin; float *Xout; long long sX; long long ld;
    typedef float4 Aux;
    __device__ Aux pre(int z, int m, int n) const
    {
        return *(const float4 *)(Xin + (long long)z * sX + (long long)m * ld + n);
    }
    __device__ void operator()(int z, int m, int n, const float (&v)[4], const Aux &x) const
    {
        const long long o = (long long)z * sX + (long long)m * ld + n;
        const float4 b = *(const float4 *)(bias + (long long)z * sBias + n);
        st_nt4((float4 *)(Xout + o), make_float4(x.x + v[0] + b.x, x.y + v[1] + b.y, x.z + v[2] + b.z, x.w + v[3] + b.w));
    }
};
struct EpiGeluBwd {              // dh = acc * gelu'(h), H holding gelu'(h) from the forward pass; both blocked
    const bf16_t *H; long long sH; bf16_t *DH; long long sDH; long long ld;
    typedef bf16x4 Aux;
    __device__ Aux pre(int z, int m, int n) const
    {
        return *(const bf16x4 *)(H + (long long)z * sH + blk_off(m, n, ld));
    }
    __device__ void operator()(int z, int m, int n, const float (&v)[4], const Aux &hb) const
    {
        float r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = v[i] * (float)hb[i];
        __builtin_nontemporal_store(pack4(r[0], r[1], r[2], r[3]), (bf16x4 *)(DH + (long long)z * sDH + blk_off(m, n, ld)));
    }
};

// Tile shapes (BM, BN, BK, wavefronts in M, wavefronts in N), from timing the GEMM shapes of the
// benchmark size (tokens x width x hidden = 12608 x 768 x 3072, batch 8) on MI355X:
// 256x256x64 tiles with 8 wavefronts are fastest where the token axis is M (fwd, dgrad: 4800 or
// 1200 workgroups), also for the two GEMMs with the heavy GELU epilogues (128x256x32 tiles, two
// workgroups per CU so that one's epilogue could overlap the other's main loop, timed the same to
// 4 % slower: they fetch 1.5 times the bytes from L2, which is what bounds the main loop).
// The same tile on 4 wavefronts of 128x128 (2, 2: a third fewer LDS fragment reads per
// instruction, the 256 accumulator registers in the AGPRs, one wavefront per SIMD) compiles
// without spills and is 8 - 17 % slower (500 against 461 us, 872 against 744 with the GELU
// epilogue): with one wavefront per SIMD nothing covers its own waits.
// The weight gradients (768 x 3072 outputs per worker, reduction over the tokens) go to the
// persistent two-group kernel of gemm_pp.h, whose 192x384 tiles make exactly 256 workgroups for 8
// workers.
#define QSR_GEMM_BIG 256, 256, 64, 2, 4

// NT: the plain tiled kernel.  The persistent form (one workgroup per CU, a ring of four 32-deep
// stages copied as one stream across tile boundaries, two wavefront groups a phase apart), on the
// blocked operands and in place in the iteration: 441 against 461 us for the plain K = 3072 GEMM,
// but 855 against 744 and 813 against 635 us for the two K = 768 GEMMs with epilogue traffic (a
// workgroup that goes on to its next tile must first see its epilogue's stores complete, where a
// fresh workgroup starts at once, and its two groups take their epilogues one after the other).  TN: the persistent two-group kernel where the problem allows it.
// BLKA: the activation operand is blocked (the weights always are)
template <bool BLKA, class Epi>
static hipError_t gemm_nt(const GemmNT &p, const Epi &epi, int batch, hipStream_t s)
{
    return launch_gemm_nt<QSR_GEMM_BIG, BLKA>(p, epi, batch, s);
}
template <bool BLKA, bool BLKB, class Epi>
static hipError_t gemm_tn(const GemmNT &p, const Epi &epi, int batch, hipStream_t s)
{
    // widths are multiples of 64 and a block of zeros stands in for ragged token counts, so every
    // weight gradient of this model qualifies
    if (!gemm_pp_tn_supports(p)) return hipErrorInvalidValue;
    return launch_gemm_pp_tn<BLKA, BLKB>(p, epi, batch, s);
}

#define TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return e_; } while (0)

// out[z][i] = part[z][0][i] + part[z][1][i] + ... (ascending: a fixed order), i < n, n a multiple of 4
__global__ __launch_bounds__(256) void splitk_sum_kernel(const float *__restrict__ part, long long n, int split,
                                                         float *__restrict__ out, long long sOut)
{
    const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= n) return;
    const int z = blockIdx.y;
    const float *p = part + (long long)z * split * n + i;
    float4 a = *(const float4 *)p;
    for (int s = 1; s < split; ++s) {
        const float4 b = *(const float4 *)(p + (long long)s * n);
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    *(float4 *)(out + (long long)z * sOut + i) = a;
}

// Weight gradient dW[z] = A[z]^T B[z] (p.M x p.N, rows contiguous, per-worker stride sOut) with the
// bias gradient (column sums of B) as a by-product.  A gradient with few tiles for the chip's
// persistent workgroups has its token reduction cut into up to WGRAD_SPLIT ranges, whose partial
// results are added up afterwards (the 768 x 768 output projection of 8 workers is 64 tiles of
// 192 x 384 for 256 compute units: 0.37 ms as one range each, as long as a gradient four times
// its size).
template <bool BLKA, bool BLKB>
static hipError_t wgrad(GemmNT p, float *dW, float *db, long long sOut, const ResWs &w, int batch, hipStream_t s)
{
    p.zeros = w.ZERO;
    const int tiles = ((p.M + 191) / 192) * ((p.N + 383) / 384) * batch;
    const int cus = gemm_pp_cu_count();
    int split = tiles * 2 <= cus ? (cus / tiles < WGRAD_SPLIT ? cus / tiles : WGRAD_SPLIT) : 1;
    const int k_chunk = ((p.K + split - 1) / split + 31) / 32 * 32;
    split = (p.K + k_chunk - 1) / k_chunk;
    if (split <= 1) {
        p.colsum_B = db; p.s_colsum = sOut;
        EpiScaleF32 epi{dW, p.N, sOut, 1.0f};
        return gemm_tn<BLKA, BLKB>(p, epi, batch, s);
    }
    const long long MN = (long long)p.M * p.N;
    p.split = split; p.k_chunk = k_chunk;
    p.colsum_B = w.SPLITKB; p.s_colsum = p.N;
    EpiScaleF32 epi{w.SPLITK, p.N, MN, 1.0f};
    TRY((gemm_tn<BLKA, BLKB>(p, epi, batch, s)));
    splitk_sum_kernel<<<dim3((unsigned)((MN / 4 + 255) / 256), (unsigned)batch), 256, 0, s>>>(w.SPLITK, MN, split, dW, sOut);
    TRY(hipGetLastError());
    splitk_sum_kernel<<<dim3((unsigned)((p.N / 4 + 255) / 256), (unsigned)batch), 256, 0, s>>>(w.SPLITKB, p.N, split, db, sOut);
    return hipGetLastError();
}

hipError_t launch_resmlp_grad(const ModelDims &dm, const float *theta, float *g, const float *teacher,
                              void *ws, float *loss, const DevState *st, hipStream_t s)
{
    const int K = dm.K, M = (int)dm.B, d = (int)dm.d_in, dh = (int)dm.d_hidden, L = dm.n_blocks;
    const int heads = dm.n_heads, S = (int)dm.seq_len;
    const int nsub = heads > 0 ? 2 : 1;           // residual sub-blocks per block
    const long long P = dm.P;
    const long long dd = (long long)d * d;
    const long long per_attn = heads > 0 ? 2LL * d + 3 * dd + 3LL * d + dd + d : 0;
    const long long per_block = per_attn + 2LL * d + (long long)d * dh + dh + (long long)dh * d + d;
    if (heads > 0 && !attn_supports(d, heads, S, M)) return hipErrorInvalidValue;
    ResWs w = carve(dm, ws, nullptr);
    const long long Md = (long long)M * d;            // a row-major [M][d] array (fp32 state and its relatives)
    const long long MdB = w.mdB, MdhB = w.mdhB;       // a blocked [M][d] / [M][dh] bf16 array
    // Rows per wavefront of the LayerNorm backward pass: enough that all wavefronts of the launch
    // are resident at once (a launch of 1.5 times the chip's wavefront slots runs as one full wave of
    // workgroups and a half-empty one).  Resident wavefronts per CU follow from the kernel's registers.
    const int vpl_ln = (d + 255) / 256;
    const int ln_slots = gemm_pp_cu_count() * (vpl_ln <= 1 ? 28 : vpl_ln == 2 ? 20 : vpl_ln == 3 ? 16 : 12);
    int rows_per_wave = (int)(((long long)K * M + ln_slots - 1) / ln_slots);
    if (rows_per_wave < LN_ROWS_PER_WAVE) rows_per_wave = LN_ROWS_PER_WAVE;
    const int wave_rows = (M + rows_per_wave - 1) / rows_per_wave;

    AttnArgs att{};
    if (heads > 0) {
        att.sQKV = w.sQKV; att.sO = w.sO; att.sLSE = w.sLSE; att.DO = w.DO; att.sDO = w.sDO;
        att.DQKV = w.DQKV; att.sDQKV = w.sDQKV;
        att.M = M; att.d = d; att.S = S; att.nb = (S + 31) / 32;
        att.scale = 1.0f / sqrtf((float)ATT_DK);
        att.c2 = 1.4426950408889634f * att.scale;
    }

    // LayerNorm of residual state number `sub` with the parameters at off_gamma
    auto ln_fwd = [&](int sub, long long off_gamma) -> hipError_t {
        dim3 grid((unsigned)((M + 3) / 4), (unsigned)K);
#define LN_FWD(VPL) ln_fwd_kernel<VPL><<<grid, 256, 0, s>>>(w.X + (long long)sub * Md, w.sX, theta, P, off_gamma, \
                        w.U + (long long)sub * MdB, w.sU, w.MU + (long long)sub * M, w.RSTD + (long long)sub * M, w.sStat, M, d)
        const int vpl = (d + 255) / 256;
        if (vpl <= 1) LN_FWD(1); else if (vpl <= 2) LN_FWD(2); else if (vpl <= 3) LN_FWD(3); else LN_FWD(4);
#undef LN_FWD
        return hipGetLastError();
    };
    // The gradient with respect to a LayerNorm's output comes out of a bf16 GEMM.  In the MLP-only
    // model it is stored in bf16, like the activations (2 B instead of 4 written by the GEMM and
    // read by the pass below: 2-3 % of an iteration at the benchmark size).  With attention
    // sub-blocks it stays in fp32: the query-weight gradients, sums of small softmax-gradient
    // terms, sit at the tested error bound already, and this one more rounding (in the MLP
    // sub-block alone) moved an entry past it.  The buffer is the same.
    const bool du16 = heads == 0;
    bf16_t *const DU16 = (bf16_t *)w.DU;
    const long long sDU16 = 2 * w.sDU;
    // its backward pass plus the residual path: DX (d loss / d state sub+1) and DU -> DX in place
    // (d loss / d state sub, also in bf16), and the LayerNorm parameter gradients
    auto ln_bwd = [&](int sub, long long off_gamma) -> hipError_t {
        dim3 grid((unsigned)((wave_rows + 3) / 4), (unsigned)K);
#define LN_BWD_ARGS w.X + (long long)sub * Md, w.sX, w.MU + (long long)sub * M, w.RSTD + (long long)sub * M, w.sStat, theta, P, off_gamma, \
                    w.DX, w.DX, w.sDX, w.DXb, w.sDXb, w.PART, w.sPART, wave_rows, rows_per_wave, M, d
#define LN_BWD(VPL) do { if (du16) ln_bwd_kernel<VPL, bf16_t><<<grid, 256, 0, s>>>(DU16, sDU16, LN_BWD_ARGS); \
                         else ln_bwd_kernel<VPL, float><<<grid, 256, 0, s>>>(w.DU, w.sDU, LN_BWD_ARGS); } while (0)
        const int vpl = (d + 255) / 256;
        if (vpl <= 1) LN_BWD(1); else if (vpl <= 2) LN_BWD(2); else if (vpl <= 3) LN_BWD(3); else LN_BWD(4);
#undef LN_BWD
#undef LN_BWD_ARGS
        TRY(hipGetLastError());
        colsum_final_kernel<<<dim3((unsigned)((d + 63) / 64), (unsigned)K, 2), 256, 0, s>>>(
            w.PART, w.sPART, g + off_gamma, P, wave_rows, d);
        return hipGetLastError();
    };

    TRY(launch_fill_zero((float *)w.ZERO, 64, s));
    // bf16 copies of the weights in both orientations (the master weights changed last step): one
    // launch per kind of weight, over all blocks and workers
    {
        const long long oW1 = per_attn + 2LL * d, oW2 = oW1 + (long long)d * dh + dh;
        TRY(launch_cvt_transpose<float>(theta + oW1, dh, P, per_block, w.W1b, w.sW, w.W1Tb, w.sW, d, dh, K, L, s));
        TRY(launch_cvt_transpose<float>(theta + oW2, d, P, per_block, w.W2b, w.sW, w.W2Tb, w.sW, dh, d, K, L, s));
        if (heads > 0) {
            const long long oWq = 2LL * d, oWo = oWq + 3 * dd + 3LL * d;
            TRY(launch_cvt_transpose<float>(theta + oWq, 3LL * d, P, per_block, w.Wqb, w.sWq, w.WqTb, w.sWq, d, 3 * d, K, L, s));
            TRY(launch_cvt_transpose<float>(theta + oWo, d, P, per_block, w.Wob, w.sWo, w.WoTb, w.sWo, d, d, K, L, s));
        }
    }
    TRY(launch_cvt_transpose<float>(teacher, d, 0, 0, nullptr, 0, w.WTt, 0, d, d, 1, 1, s));
    // elements of one block's blocked weight copies: as stored ([rows][cols]) and transposed
    const long long wW1 = w.wB[0], wW1T = w.wB[1], wW2 = w.wB[1], wW2T = w.wB[0];
    const long long wWq = blk_elems(d, 3 * d), wWqT = blk_elems(3 * d, d), wWo = blk_elems(d, d);

    // Sample(): tokens x_0 (fp32 in X[0], bf16 in U), teacher targets y = x_0 W_T / sqrt(d)
    TRY(launch_fill_normal(w.X, w.sX, K, Md, 1.0f, STREAM_X, dm.seed, st, s));
    {
        long long blocks = (Md / 4 + 255) / 256; if (blocks > 65535) blocks = 65535;   // d is a multiple of 64
        f32_to_bf16_kernel<<<dim3((unsigned)blocks, (unsigned)K), 256, 0, s>>>(w.X, w.sX, w.U, w.sU, Md / 4, d);
        TRY(hipGetLastError());
    }
    {
        GemmNT p{w.U, w.WTt, M, d, d, d, d, w.sU, 0};
        EpiScaleF32 epi{w.Y, d, w.sY, 1.0f / sqrtf((float)d)};
        TRY(gemm_nt<true>(p, epi, K, s));
    }

    // forward
    for (int l = 0; l < L; ++l) {
        int sub = nsub * l;
        if (heads > 0) {
            const long long oga = l * per_block, obq = oga + 2LL * d + 3 * dd, obo = obq + 3LL * d + dd;
            bf16_t *QKVl = w.QKV + (long long)l * M * 3 * d, *Ol = w.O + (long long)l * Md;
            TRY(ln_fwd(sub, oga));
            {
                GemmNT p{w.U + (long long)sub * MdB, w.WqTb + l * wWqT, M, 3 * d, d, d, d, w.sU, w.sWq};
                EpiBiasBf16 epi{theta + obq, P, QKVl, 3LL * d, w.sQKV};
                TRY(gemm_nt<true>(p, epi, K, s));
            }
            att.QKV = QKVl; att.O = Ol; att.LSE = w.LSE + (long long)l * heads * M;
            TRY(launch_attn_fwd(att, heads, K, s));
            {
                GemmNT p{Ol, w.WoTb + l * wWo, M, d, d, d, d, w.sO, w.sWo};
                EpiBiasResidual epi{theta + obo, P, w.X + (long long)sub * Md, w.X + (long long)(sub + 1) * Md, w.sX, d};
                TRY(gemm_nt<false>(p, epi, K, s));
            }
            ++sub;
        }
        const long long og = l * per_block + per_attn, ob1 = og + 2LL * d + (long long)d * dh,
                        ob2 = ob1 + dh + (long long)dh * d;
        const float *Xl = w.X + (long long)sub * Md;
        float *Xn = w.X + (long long)(sub + 1) * Md;
        bf16_t *Ul = w.U + (long long)sub * MdB, *Al = w.A + (long long)l * MdhB;
        TRY(ln_fwd(sub, og));
        {
            GemmNT p{Ul, w.W1Tb + l * wW1T, M, dh, d, d, d, w.sU, w.sW};
            EpiBiasGelu epi{theta + ob1, P, w.H + (long long)l * MdhB, w.sH, Al, w.sA, dh};
            TRY(gemm_nt<true>(p, epi, K, s));
        }
        {
            GemmNT p{Al, w.W2Tb + l * wW2T, M, d, dh, dh, dh, w.sA, w.sW};
            EpiBiasResidual epi{theta + ob2, P, Xl, Xn, w.sX, d};
            TRY(gemm_nt<true>(p, epi, K, s));
        }
    }

    // loss and d loss / d x_L
    {
        const int nparts = (int)((Md + 1023) / 1024);
        const float inv = 1.0f / ((float)M * (float)d);
        loss_kernel<<<dim3((unsigned)nparts, (unsigned)K), 256, 0, s>>>(
            w.X + (long long)(nsub * L) * Md, w.sX, w.Y, w.sY, w.DX, w.sDX, w.DXb, w.sDXb, w.LPART, w.sLPART, Md, inv);
        TRY(hipGetLastError());
        loss_final_kernel<<<K, 256, 0, s>>>(w.LPART, w.sLPART, nparts, 0.5f * inv, loss);
        TRY(hipGetLastError());
    }

    // backward; DX (and its bf16 copy DXb) holds d loss / d (output of the sub-block at hand)
    for (int l = L - 1; l >= 0; --l) {
        int sub = nsub * l + nsub - 1;
        const long long og = l * per_block + per_attn, oW1 = og + 2LL * d, ob1 = oW1 + (long long)d * dh,
                        oW2 = ob1 + dh, ob2 = oW2 + (long long)dh * d;
        // W2 and b2:  dW2 = a^T dx, db2 = column sums of dx (by-product of the same GEMM)
        {
            GemmNT p{w.A + (long long)l * MdhB, w.DXb, dh, d, M, dh, d, w.sA, w.sDXb};
            TRY((wgrad<true, false>(p, g + oW2, g + ob2, P, w, K, s)));
        }
        // dh = (dx W2^T) * gelu'(h)
        {
            GemmNT p{w.DXb, w.W2b + l * wW2, M, dh, d, d, d, w.sDXb, w.sW};
            EpiGeluBwd epi{w.H + (long long)l * MdhB, w.sH, w.DH, w.sDH, dh};
            TRY(gemm_nt<false>(p, epi, K, s));
        }
        // W1 and b1:  dW1 = u^T dh, db1 = column sums of dh
        {
            GemmNT p{w.U + (long long)sub * MdB, w.DH, d, dh, M, d, dh, w.sU, w.sDH};
            TRY((wgrad<true, true>(p, g + oW1, g + ob1, P, w, K, s)));
        }
        // du = dh W1^T, then LayerNorm backward + residual
        {
            GemmNT p{w.DH, w.W1b + l * wW1, M, d, dh, dh, dh, w.sDH, w.sW};
            if (du16) {
                EpiBf16<false> epi{DU16, d, sDU16};
                TRY(gemm_nt<true>(p, epi, K, s));
            } else {
                EpiScaleF32 epi{w.DU, d, w.sDU, 1.0f};
                TRY(gemm_nt<true>(p, epi, K, s));
            }
        }
        TRY(ln_bwd(sub, og));
        if (heads > 0) {
            --sub;
            const long long oga = l * per_block, oWq = oga + 2LL * d, obq = oWq + 3 * dd, oWo = obq + 3LL * d,
                            obo = oWo + dd;
            bf16_t *QKVl = w.QKV + (long long)l * M * 3 * d, *Ol = w.O + (long long)l * Md;
            // Wo and bo:  dWo = o^T dx, dbo = column sums of dx
            {
                GemmNT p{Ol, w.DXb, d, d, M, d, d, w.sO, w.sDXb};
                TRY((wgrad<false, false>(p, g + oWo, g + obo, P, w, K, s)));
            }
            // do = dx Wo^T
            {
                GemmNT p{w.DXb, w.Wob + l * wWo, M, d, d, d, d, w.sDXb, w.sWo};
                EpiBf16<false> epi{w.DO, d, w.sDO};
                TRY(gemm_nt<false>(p, epi, K, s));
            }
            att.QKV = QKVl; att.O = Ol; att.LSE = w.LSE + (long long)l * heads * M;
            TRY(launch_attn_bwd(att, heads, K, s));
            // Wqkv and bqkv:  dWqkv = u^T dqkv, dbqkv = column sums of dqkv
            {
                GemmNT p{w.U + (long long)sub * MdB, w.DQKV, d, 3 * d, M, d, 3LL * d, w.sU, w.sDQKV};
                TRY((wgrad<true, false>(p, g + oWq, g + obq, P, w, K, s)));
            }
            // du = dqkv Wqkv^T, then LayerNorm backward + residual
            {
                GemmNT p{w.DQKV, w.Wqb + l * wWq, M, d, 3 * d, 3LL * d, 3LL * d, w.sDQKV, w.sWq};
                EpiScaleF32 epi{w.DU, d, w.sDU, 1.0f};
                TRY(gemm_nt<false>(p, epi, K, s));
            }
            TRY(ln_bwd(sub, oga));
        }
    }
    return hipSuccess;
}

}  // namespace qsr
