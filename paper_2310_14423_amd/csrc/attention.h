// attention.h -- the core of multi-head self-attention, o = softmax(q k^T / sqrt(dk)) v within each
// sequence, forward and backward, on the gfx950 bf16 matrix cores (the attention half of the ViT-B
// encoder block that Sec. 4 / App. C.2 of arXiv 2310.14423 trains: heads of width 64, sequences of
// 196-197 tokens).  The projections around it are ordinary GEMMs (gemm_bf16.h, gemm_pp.h).
//
// One workgroup per (sequence, head, worker); sequences are short, so a whole head's K and V (or
// Q and dO) tiles sit in LDS and each wavefront owns one block of 32 tokens.  Everything is
// computed in the transposed sense, S^T = K Q^T, so that a lane owns one query (the column l%32
// of v_mfma_f32_32x32x16_bf16's result) and the keys run over its 16 accumulator registers:
//   * the softmax statistics of a query are reductions over a lane's own registers plus one
//     exchange with lane l^32;
//   * the probabilities are, as they lie in the registers, the B operand of the next product
//     (O^T = V^T P^T): accumulator registers 8c..8c+7 of a lane are eight key indices of one
//     16-wide contraction step.  Which eight is a fixed permutation (keys 16c + 8(j/4) + 4(l/32) +
//     j%4 for slot j), and a contraction may run in any order as long as both operands use the
//     same one: the A operand is read from a transposed [feature][token] copy in LDS at exactly
//     those token indices (two 8-byte reads).  No probability ever passes through LDS.
// The backward pass recomputes the probabilities from the saved log-sum-exp (base 2) of each query
// and splits in two kernels by what is summed over: dK, dV (a wavefront owns 32 keys and walks the
// query blocks, lanes = keys, S itself rather than S^T) and dQ (a wavefront owns 32 queries and
// walks the key blocks, lanes = queries).
//
// Limits: head width 64, sequence length <= 224 (7 blocks of 32; the last block may be ragged:
// rows beyond the sequence are zero in LDS and masked in the probabilities).
#pragma once
#include <hip/hip_runtime.h>
#include "gemm_bf16.h"

namespace qsr {

constexpr int ATT_DK = 64;                    // head width
constexpr int ATT_MAXB = 7;                   // 32-token blocks per sequence
constexpr int ATT_ROWS = ATT_MAXB * 32;
constexpr int ATT_LDR = ATT_DK + 8;           // row stride (bf16) of a [token][feature] tile in LDS
constexpr int ATT_LDT = ATT_ROWS + 8;         // row stride (bf16) of a [feature][token] tile in LDS

struct AttnArgs {
    const bf16_t *QKV; long long sQKV;        // [M][3d] per worker: q | k | v, head h in columns h*64..
    bf16_t *O; long long sO;                  // [M][d]  attention output, heads side by side
    float *LSE; long long sLSE;               // [heads][M]  log2(sum_j 2^(c2 q.k_j)) per query
    const bf16_t *DO; long long sDO;          // [M][d]  d loss / d o
    bf16_t *DQKV; long long sDQKV;            // [M][3d] d loss / d (q | k | v)
    int M, d, S, nb;                          // tokens per worker, width, sequence length, ceil(S/32)
    float c2;                                 // log2(e) / sqrt(dk)
    float scale;                              // 1 / sqrt(dk)
};

__device__ __forceinline__ bf16x8 att_zero8()
{
    bf16x8 z;
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = (bf16_t)0.0f;
    return z;
}

// eight consecutive accumulator registers as one MFMA operand (the k-slot permutation above)
__device__ __forceinline__ bf16x8 att_pack8(const float (&v)[16], int c)
{
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = (bf16_t)v[8 * c + j];
    return r;
}

// A operand from a [feature][token] tile: feature row, tokens t0..t0+3 and t0+8..t0+11
__device__ __forceinline__ bf16x8 att_read_t(const bf16_t *tile, int row, int t0)
{
    const bf16x4 lo = *(const bf16x4 *)(tile + row * ATT_LDT + t0);
    const bf16x4 hi = *(const bf16x4 *)(tile + row * ATT_LDT + t0 + 8);
    bf16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return r;
}

// Forward: O and the log-sum-exp per query.  blockDim.x = 64 * nb, wavefront w owns queries 32w..
__global__ __launch_bounds__(64 * ATT_MAXB) void attn_fwd_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(16))) bf16_t Ks[ATT_ROWS * ATT_LDR];
    __shared__ __attribute__((aligned(16))) bf16_t Vt[ATT_DK * ATT_LDT];
    const int seq = blockIdx.x, head = blockIdx.y, z = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, l32 = lane & 31;
    const int S = a.S, nb = a.nb;
    const long long ld = 3LL * a.d;
    const bf16_t *base = a.QKV + (long long)z * a.sQKV + (long long)seq * S * ld + head * ATT_DK;

    for (int it = tid; it < nb * 256; it += nb * 64) {
        const int t = it >> 3, pc = it & 7;
        bf16x8 kv = att_zero8(), vv = att_zero8();
        if (t < S) {
            kv = *(const bf16x8 *)(base + (long long)t * ld + a.d + pc * 8);
            vv = *(const bf16x8 *)(base + (long long)t * ld + 2 * a.d + pc * 8);
        }
        *(bf16x8 *)(Ks + t * ATT_LDR + pc * 8) = kv;
#pragma unroll
        for (int e = 0; e < 8; ++e) Vt[(pc * 8 + e) * ATT_LDT + t] = vv[e];
    }
    const int q = wave * 32 + l32;
    const int qrow = min(q, S - 1);
    bf16x8 qf[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) qf[c] = *(const bf16x8 *)(base + (long long)qrow * ld + c * 16 + hf * 8);
    __syncthreads();

    // scores, transposed: st[kb][i] = q . k_key, key = 32 kb + 8 (i/4) + 4 hf + i%4
    float st[ATT_MAXB][16];
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < ATT_MAXB; ++kb) {
        if (kb < nb) {
            f32x16 acc;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bf16x8 kf = *(const bf16x8 *)(Ks + (kb * 32 + l32) * ATT_LDR + c * 16 + hf * 8);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], acc, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = kb * 32 + (i >> 2) * 8 + hf * 4 + (i & 3);
                const float v = key < S ? acc[i] * a.c2 : -INFINITY;
                st[kb][i] = v;
                mx = fmaxf(mx, v);
            }
        }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float sum = 0.f;
#pragma unroll
    for (int kb = 0; kb < ATT_MAXB; ++kb) {
        if (kb < nb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(st[kb][i] - mx);
                st[kb][i] = p;
                sum += p;
            }
        }
    }
    sum += __shfl_xor(sum, 32, 64);

    // O^T = V^T P^T
    f32x16 ot[2];
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int e = 0; e < 16; ++e) ot[fb][e] = 0.f;
#pragma unroll
    for (int kb = 0; kb < ATT_MAXB; ++kb) {
        if (kb < nb) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const bf16x8 pb = att_pack8(st[kb], c);
#pragma unroll
                for (int fb = 0; fb < 2; ++fb) {
                    const bf16x8 vf = att_read_t(Vt, fb * 32 + l32, kb * 32 + 16 * c + hf * 4);
                    ot[fb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb, ot[fb], 0, 0, 0);
                }
            }
        }
    }
    if (q < S) {
        const float inv = 1.0f / sum;
        const long long tok = (long long)seq * S + q;
        bf16_t *o = a.O + (long long)z * a.sO + tok * a.d + head * ATT_DK;
#pragma unroll
        for (int fb = 0; fb < 2; ++fb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 r = {(bf16_t)(ot[fb][4 * g] * inv), (bf16_t)(ot[fb][4 * g + 1] * inv),
                            (bf16_t)(ot[fb][4 * g + 2] * inv), (bf16_t)(ot[fb][4 * g + 3] * inv)};
                *(bf16x4 *)(o + fb * 32 + g * 8 + hf * 4) = r;
            }
        if (hf == 0) a.LSE[(long long)z * a.sLSE + (long long)head * a.M + tok] = mx + log2f(sum);
    }
}

constexpr size_t ATT_BWD_KV_SMEM = (size_t)(2 * ATT_ROWS * ATT_LDR + 2 * ATT_DK * ATT_LDT) * sizeof(bf16_t) + 2 * ATT_ROWS * sizeof(float);
constexpr size_t ATT_BWD_Q_SMEM = (size_t)(2 * ATT_ROWS * ATT_LDR + ATT_DK * ATT_LDT) * sizeof(bf16_t);

// Backward, dK and dV: wavefront w owns keys 32w.. (lanes = keys) and walks the query blocks.
//   P = 2^(c2 S - lse),  dV = P^T dO,  dP = dO V^T,  D = rowsum(dO o),  dS = P (dP - D),
//   dK = dS^T Q / sqrt(dk)
__global__ __launch_bounds__(64 * ATT_MAXB) void attn_bwd_kv_kernel(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char att_smem[];
    bf16_t *Qs = (bf16_t *)att_smem;
    bf16_t *dOs = Qs + ATT_ROWS * ATT_LDR;
    bf16_t *Qt = dOs + ATT_ROWS * ATT_LDR;
    bf16_t *dOt = Qt + ATT_DK * ATT_LDT;
    float *Ds = (float *)(dOt + ATT_DK * ATT_LDT);
    float *Ls = Ds + ATT_ROWS;
    const int seq = blockIdx.x, head = blockIdx.y, z = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, l32 = lane & 31;
    const int S = a.S, nb = a.nb;
    const long long ld = 3LL * a.d, tok0 = (long long)seq * S;
    const bf16_t *base = a.QKV + (long long)z * a.sQKV + tok0 * ld + head * ATT_DK;
    const bf16_t *dob = a.DO + (long long)z * a.sDO + tok0 * a.d + head * ATT_DK;
    const bf16_t *ob = a.O + (long long)z * a.sO + tok0 * a.d + head * ATT_DK;
    const float *lse = a.LSE + (long long)z * a.sLSE + (long long)head * a.M + tok0;

    // every thread makes the same number of trips (nb*256 items, nb*64 threads), and the eight
    // pieces of a token row are eight adjacent lanes: D is finished with three exchanges
    for (int it = tid; it < nb * 256; it += nb * 64) {
        const int t = it >> 3, pc = it & 7;
        bf16x8 qv = att_zero8(), dv = att_zero8(), ov = att_zero8();
        if (t < S) {
            qv = *(const bf16x8 *)(base + (long long)t * ld + pc * 8);
            dv = *(const bf16x8 *)(dob + (long long)t * a.d + pc * 8);
            ov = *(const bf16x8 *)(ob + (long long)t * a.d + pc * 8);
        }
        *(bf16x8 *)(Qs + t * ATT_LDR + pc * 8) = qv;
        *(bf16x8 *)(dOs + t * ATT_LDR + pc * 8) = dv;
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            Qt[(pc * 8 + e) * ATT_LDT + t] = qv[e];
            dOt[(pc * 8 + e) * ATT_LDT + t] = dv[e];
            dot = fmaf((float)dv[e], (float)ov[e], dot);
        }
        dot += __shfl_xor(dot, 1, 64);
        dot += __shfl_xor(dot, 2, 64);
        dot += __shfl_xor(dot, 4, 64);
        if (pc == 0) {
            Ds[t] = dot;
            Ls[t] = t < S ? lse[t] : 0.f;
        }
    }
    const int key = wave * 32 + l32;
    const int krow = min(key, S - 1);
    bf16x8 kf[4], vf[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        kf[c] = *(const bf16x8 *)(base + (long long)krow * ld + a.d + c * 16 + hf * 8);
        vf[c] = *(const bf16x8 *)(base + (long long)krow * ld + 2 * a.d + c * 16 + hf * 8);
    }
    __syncthreads();

    f32x16 dvt[2], dkt[2];
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int e = 0; e < 16; ++e) { dvt[fb][e] = 0.f; dkt[fb][e] = 0.f; }

    for (int qb = 0; qb < nb; ++qb) {
        f32x16 sacc, dpacc;
#pragma unroll
        for (int e = 0; e < 16; ++e) { sacc[e] = 0.f; dpacc[e] = 0.f; }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bf16x8 qa = *(const bf16x8 *)(Qs + (qb * 32 + l32) * ATT_LDR + c * 16 + hf * 8);
            const bf16x8 da = *(const bf16x8 *)(dOs + (qb * 32 + l32) * ATT_LDR + c * 16 + hf * 8);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[c], sacc, 0, 0, 0);
            dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da, vf[c], dpacc, 0, 0, 0);
        }
        // rows of the result = queries 32 qb + 8 (i/4) + 4 hf + i%4, column = this lane's key
        float p[16], ds[16];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int q0 = qb * 32 + g * 8 + hf * 4;
            const float4 l4 = *(const float4 *)(Ls + q0), d4 = *(const float4 *)(Ds + q0);
            const float lq[4] = {l4.x, l4.y, l4.z, l4.w}, dq[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = 4 * g + r;
                const bool valid = key < S && q0 + r < S;
                const float pv = valid ? __builtin_amdgcn_exp2f(fmaf(sacc[i], a.c2, -lq[r])) : 0.f;
                p[i] = pv;
                ds[i] = pv * (dpacc[i] - dq[r]);
            }
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bf16x8 pb = att_pack8(p, c), sb = att_pack8(ds, c);
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) {
                const bf16x8 dot_ = att_read_t(dOt, fb * 32 + l32, qb * 32 + 16 * c + hf * 4);
                const bf16x8 qt_ = att_read_t(Qt, fb * 32 + l32, qb * 32 + 16 * c + hf * 4);
                dvt[fb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dot_, pb, dvt[fb], 0, 0, 0);
                dkt[fb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt_, sb, dkt[fb], 0, 0, 0);
            }
        }
    }
    if (key < S) {
        bf16_t *dst = a.DQKV + (long long)z * a.sDQKV + (tok0 + key) * ld + head * ATT_DK;
#pragma unroll
        for (int fb = 0; fb < 2; ++fb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int f = fb * 32 + g * 8 + hf * 4;
                bf16x4 rk = {(bf16_t)(dkt[fb][4 * g] * a.scale), (bf16_t)(dkt[fb][4 * g + 1] * a.scale),
                             (bf16_t)(dkt[fb][4 * g + 2] * a.scale), (bf16_t)(dkt[fb][4 * g + 3] * a.scale)};
                bf16x4 rv = {(bf16_t)dvt[fb][4 * g], (bf16_t)dvt[fb][4 * g + 1], (bf16_t)dvt[fb][4 * g + 2],
                             (bf16_t)dvt[fb][4 * g + 3]};
                *(bf16x4 *)(dst + a.d + f) = rk;
                *(bf16x4 *)(dst + 2 * a.d + f) = rv;
            }
    }
}

// Backward, dQ: wavefront w owns queries 32w.. (lanes = queries) and walks the key blocks.
//   dQ = dS K / sqrt(dk), computed as dQ^T = K^T dS^T with dS^T in the registers
__global__ __launch_bounds__(64 * ATT_MAXB) void attn_bwd_q_kernel(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char att_smem[];
    bf16_t *Ks = (bf16_t *)att_smem;
    bf16_t *Vs = Ks + ATT_ROWS * ATT_LDR;
    bf16_t *Kt = Vs + ATT_ROWS * ATT_LDR;
    const int seq = blockIdx.x, head = blockIdx.y, z = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, l32 = lane & 31;
    const int S = a.S, nb = a.nb;
    const long long ld = 3LL * a.d, tok0 = (long long)seq * S;
    const bf16_t *base = a.QKV + (long long)z * a.sQKV + tok0 * ld + head * ATT_DK;
    const bf16_t *dob = a.DO + (long long)z * a.sDO + tok0 * a.d + head * ATT_DK;
    const bf16_t *ob = a.O + (long long)z * a.sO + tok0 * a.d + head * ATT_DK;

    for (int it = tid; it < nb * 256; it += nb * 64) {
        const int t = it >> 3, pc = it & 7;
        bf16x8 kv = att_zero8(), vv = att_zero8();
        if (t < S) {
            kv = *(const bf16x8 *)(base + (long long)t * ld + a.d + pc * 8);
            vv = *(const bf16x8 *)(base + (long long)t * ld + 2 * a.d + pc * 8);
        }
        *(bf16x8 *)(Ks + t * ATT_LDR + pc * 8) = kv;
        *(bf16x8 *)(Vs + t * ATT_LDR + pc * 8) = vv;
#pragma unroll
        for (int e = 0; e < 8; ++e) Kt[(pc * 8 + e) * ATT_LDT + t] = kv[e];
    }
    const int q = wave * 32 + l32;
    const int qrow = min(q, S - 1);
    bf16x8 qf[4], dof[4];
    float dot = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        qf[c] = *(const bf16x8 *)(base + (long long)qrow * ld + c * 16 + hf * 8);
        dof[c] = *(const bf16x8 *)(dob + (long long)qrow * a.d + c * 16 + hf * 8);
        const bf16x8 ov = *(const bf16x8 *)(ob + (long long)qrow * a.d + c * 16 + hf * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) dot = fmaf((float)dof[c][e], (float)ov[e], dot);
    }
    const float D = dot + __shfl_xor(dot, 32, 64);
    const float L = a.LSE[(long long)z * a.sLSE + (long long)head * a.M + tok0 + qrow];
    __syncthreads();

    f32x16 dqt[2];
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int e = 0; e < 16; ++e) dqt[fb][e] = 0.f;

    for (int kb = 0; kb < nb; ++kb) {
        f32x16 sacc, dpacc;
#pragma unroll
        for (int e = 0; e < 16; ++e) { sacc[e] = 0.f; dpacc[e] = 0.f; }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bf16x8 ka = *(const bf16x8 *)(Ks + (kb * 32 + l32) * ATT_LDR + c * 16 + hf * 8);
            const bf16x8 va = *(const bf16x8 *)(Vs + (kb * 32 + l32) * ATT_LDR + c * 16 + hf * 8);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[c], sacc, 0, 0, 0);
            dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, dof[c], dpacc, 0, 0, 0);
        }
        // rows of the result = keys 32 kb + 8 (i/4) + 4 hf + i%4, column = this lane's query
        float ds[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = kb * 32 + (i >> 2) * 8 + hf * 4 + (i & 3);
            const float pv = key < S ? __builtin_amdgcn_exp2f(fmaf(sacc[i], a.c2, -L)) : 0.f;
            ds[i] = pv * (dpacc[i] - D);
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bf16x8 sb = att_pack8(ds, c);
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) {
                const bf16x8 kt_ = att_read_t(Kt, fb * 32 + l32, kb * 32 + 16 * c + hf * 4);
                dqt[fb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt_, sb, dqt[fb], 0, 0, 0);
            }
        }
    }
    if (q < S) {
        bf16_t *dst = a.DQKV + (long long)z * a.sDQKV + (tok0 + q) * ld + head * ATT_DK;
#pragma unroll
        for (int fb = 0; fb < 2; ++fb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 r = {(bf16_t)(dqt[fb][4 * g] * a.scale), (bf16_t)(dqt[fb][4 * g + 1] * a.scale),
                            (bf16_t)(dqt[fb][4 * g + 2] * a.scale), (bf16_t)(dqt[fb][4 * g + 3] * a.scale)};
                *(bf16x4 *)(dst + fb * 32 + g * 8 + hf * 4) = r;
            }
    }
}

// Shapes this file's kernels take
inline bool attn_supports(long long d, int heads, long long S, long long M)
{
    return heads > 0 && d == (long long)heads * ATT_DK && S >= 1 && S <= ATT_ROWS && M % S == 0 && M / S <= 0x7fffffffLL;
}

inline hipError_t launch_attn_fwd(const AttnArgs &a, int heads, int K, hipStream_t s)
{
    dim3 grid((unsigned)(a.M / a.S), (unsigned)heads, (unsigned)K);
    attn_fwd_kernel<<<grid, 64 * a.nb, 0, s>>>(a);
    return hipGetLastError();
}

inline hipError_t launch_attn_bwd(const AttnArgs &a, int heads, int K, hipStream_t s)
{
    static bool lds_limit_raised = false;     // contexts are not thread-safe
    if (!lds_limit_raised) {
        hipError_t e = hipFuncSetAttribute((const void *)attn_bwd_kv_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)ATT_BWD_KV_SMEM);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void *)attn_bwd_q_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)ATT_BWD_Q_SMEM);
        if (e != hipSuccess) return e;
        lds_limit_raised = true;
    }
    dim3 grid((unsigned)(a.M / a.S), (unsigned)heads, (unsigned)K);
    attn_bwd_kv_kernel<<<grid, 64 * a.nb, ATT_BWD_KV_SMEM, s>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    attn_bwd_q_kernel<<<grid, 64 * a.nb, ATT_BWD_Q_SMEM, s>>>(a);
    return hipGetLastError();
}

}  // namespace qsr
