// attention.h -- the core of multi-head self-attention, o = softmax(q k^T / sqrt(dk)) v within each
// sequence, forward and backward, on the gfx950 bf16 matrix cores (the attention half of the ViT-B
// encoder block that Sec. 4 / App. C.2 of arXiv 2310.14423 trains: heads of width 64, sequences of
// 196-197 tokens).  The projections around it are ordinary GEMMs (gemm_bf16.h, gemm_pp.h).
//
// One workgroup per (sequence, head, worker); sequences are short, so a whole head's K and V (or
// Q and dO) tiles sit in LDS, as they are in memory ([token][feature]), and each wavefront owns one
// block of 32 tokens.  Everything is computed in the transposed sense, S^T = K Q^T, so that a lane
// owns one query (the column l%32 of v_mfma_f32_32x32x16_bf16's result) and the keys run over its
// 16 accumulator registers:
//   * the softmax statistics of a query are reductions over a lane's own registers plus one
//     exchange with lane l^32 (kept as running maximum and sum over the key blocks, the partial
//     output rescaled when the maximum moves);
//   * the probabilities are, as they lie in the registers, the B operand of the next product
//     (O^T = V^T P^T): accumulator registers 8c..8c+7 of a lane are eight key indices of one
//     16-wide contraction step.  Which eight is a fixed permutation (keys 16c + 8(j/4) + 4(l/32) +
//     j%4 for slot j), and a contraction may run in any order as long as both operands use the
//     same one: the A operand, V^T, comes from the [token][feature] tile through the LDS transpose
//     read (ds_read_b64_tr_b16), whose 4-token groups are pointed at exactly those tokens.
//     No probability ever passes through LDS, and no transposed copy of a tile exists.
// The backward pass recomputes the probabilities from the saved log-sum-exp (base 2) of each query
// and splits in two kernels by what is summed over: dK, dV (a wavefront owns 32 keys and walks the
// query blocks, lanes = keys, S itself rather than S^T; dV and dK in two passes over the query
// blocks, which keeps the registers of a wavefront under 128 so that two workgroups share a
// compute unit and one's loads overlap the other's products; one pass for both, four products of
// twelve fewer per query block but 166 registers, timed 396 against 337 us per launch) and dQ (a wavefront owns 32 queries
// and walks the key blocks, lanes = queries).
//
// Limits: head width 64, sequence length <= 224 (7 blocks of 32; the last block may be ragged:
// rows beyond the sequence are zero in LDS and masked in the probabilities).
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include "gemm_bf16.h"

namespace qsr {

constexpr int ATT_DK = 64;                    // head width
constexpr int ATT_MAXB = 7;                   // 32-token blocks per sequence
constexpr int ATT_ROWS = ATT_MAXB * 32;
constexpr int ATT_LDR = ATT_DK + 8;           // row stride (bf16) of a [token][feature] tile in LDS:
                                              // 16-byte fragment reads and transpose reads both conflict-free
constexpr int ATT_TILE = ATT_ROWS * ATT_LDR;  // elements of one tile

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

// A zero accumulator as a constant: the first MFMA of a chain then takes the inline constant 0
// instead of sixteen register moves.
__device__ __forceinline__ f32x16 att_zero16()
{
    const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
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

// A operand "tile^T" from a [token][feature] tile: row = feature 32 fb + l%32, contraction slots =
// tokens t0 + 8(j/4) + 4(l/32) + j%4.  The LDS transpose read hands lane j of each group of 16
// lanes element j%4 of the 64-bit words addressed by lanes j/4, j/4+4, j/4+8, j/4+12 of the group:
// lane r = q + 4e of a group points at token e, features 4q..4q+3 of a 4-token x 16-feature block.
__device__ __forceinline__ bf16x8 att_read_tr(const bf16_t *tile, int t0, int fb, int lane)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const int grp = lane >> 4, r16 = lane & 15;
    const bf16_t *q0 = tile + (t0 + (grp >> 1) * 4 + (r16 >> 2)) * ATT_LDR + fb * 32 + (grp & 1) * 16 + (r16 & 3) * 4;
    union { struct { s16x4 a, b; } s; bf16x8 v; } u;
    u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)q0);
    u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(q0 + 8 * ATT_LDR));
    return u.v;
}

// rows [0, 32 nb) of one head's [S][64] slice (row stride ld in global memory) -> LDS tile, rows >= S zero
__device__ __forceinline__ void att_load_tile(bf16_t *tile, const bf16_t *src, long long ld, int S, int nb, int tid)
{
    for (int it = tid; it < nb * 256; it += nb * 64) {
        const int t = it >> 3, pc = it & 7;
        bf16x8 v = att_zero8();
        if (t < S) v = *(const bf16x8 *)(src + (long long)t * ld + pc * 8);
        *(bf16x8 *)(tile + t * ATT_LDR + pc * 8) = v;
    }
}

// Forward: O and the log-sum-exp per query.  blockDim.x = 64 * nb, wavefront w owns queries 32w..
__global__ __launch_bounds__(64 * ATT_MAXB, 4) void attn_fwd_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(16))) bf16_t Ks[ATT_TILE];
    __shared__ __attribute__((aligned(16))) bf16_t Vs[ATT_TILE];
    const int seq = blockIdx.x, head = blockIdx.y, z = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, l32 = lane & 31;
    const int S = a.S, nb = a.nb;
    const long long ld = 3LL * a.d;
    const bf16_t *base = a.QKV + (long long)z * a.sQKV + (long long)seq * S * ld + head * ATT_DK;

    att_load_tile(Ks, base + a.d, ld, S, nb, tid);
    att_load_tile(Vs, base + 2 * a.d, ld, S, nb, tid);
    const int q = wave * 32 + l32;
    const int qrow = min(q, S - 1);
    bf16x8 qf[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) qf[c] = *(const bf16x8 *)(base + (long long)qrow * ld + c * 16 + hf * 8);
    __syncthreads();

    // Running softmax over the key blocks.  m is the reference exponent of the probabilities held so
    // far (both halves of a query agree on it), sum this half's share of their sum.  m follows the
    // running maximum lazily: it moves only when a block's maximum exceeds it by more than 8 (in
    // log2 units), so probabilities stay below 2^8 and the rescaling of the partial output, 32
    // multiplications per lane, is skipped for most blocks (the branch is uniform over the
    // wavefront).  Keys beyond the sequence exist only in the last block: only that one is masked.
    float m = -INFINITY, sum = 0.f;
    f32x16 ot[2] = {att_zero16(), att_zero16()};      // O^T = V^T P^T, unnormalized
    auto block = [&](int kb, auto masked) {
        // scores, transposed: acc[i] = q . k_key, key = 32 kb + 8 (i/4) + 4 hf + i%4
        f32x16 acc = att_zero16();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bf16x8 kf = *(const bf16x8 *)(Ks + (kb * 32 + l32) * ATT_LDR + c * 16 + hf * 8);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], acc, 0, 0, 0);
        }
        float st[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            st[i] = acc[i];
            if (decltype(masked)::value && kb * 32 + (i >> 2) * 8 + hf * 4 + (i & 3) >= S) st[i] = -INFINITY;
        }
        float mx = st[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, st[i]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * a.c2;  // finite: every block holds a key of the sequence
        const bool move = mx > m + 8.0f;
        if (__builtin_amdgcn_ballot_w64(move)) {
            const float m_new = move ? mx : m;
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            sum *= alpha;
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                for (int e = 0; e < 16; ++e) ot[fb][e] *= alpha;
            m = m_new;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            st[i] = __builtin_amdgcn_exp2f(fmaf(st[i], a.c2, -m));
            sum += st[i];
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bf16x8 pb = att_pack8(st, c);
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) {
                const bf16x8 vf = att_read_tr(Vs, kb * 32 + 16 * c, fb, lane);
                ot[fb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb, ot[fb], 0, 0, 0);
            }
        }
    };
    for (int kb = 0; kb < nb - 1; ++kb) block(kb, std::false_type{});
    block(nb - 1, std::true_type{});
    sum += __shfl_xor(sum, 32, 64);
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
        if (hf == 0) a.LSE[(long long)z * a.sLSE + (long long)head * a.M + tok] = m + log2f(sum);
    }
}

constexpr size_t ATT_BWD_KV_SMEM = (size_t)2 * ATT_TILE * sizeof(bf16_t) + 2 * ATT_ROWS * sizeof(float);

// Backward, dK and dV: wavefront w owns keys 32w.. (lanes = keys) and walks the query blocks.
//   P = 2^(c2 S - lse),  dV = P^T dO,  dP = dO V^T,  D = rowsum(dO o),  dS = P (dP - D),
//   dK = dS^T Q / sqrt(dk)
__global__ __launch_bounds__(64 * ATT_MAXB, 4) void attn_bwd_kv_kernel(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char att_smem[];
    bf16_t *Qs = (bf16_t *)att_smem;
    bf16_t *dOs = Qs + ATT_TILE;
    float *Ds = (float *)(dOs + ATT_TILE);
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
        for (int e = 0; e < 8; ++e) dot = fmaf((float)dv[e], (float)ov[e], dot);
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
    bf16x8 kf[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) kf[c] = *(const bf16x8 *)(base + (long long)krow * ld + a.d + c * 16 + hf * 8);
    __syncthreads();
    bf16_t *dst = a.DQKV + (long long)z * a.sDQKV + (tok0 + krow) * ld + head * ATT_DK;

    // Scores of query block qb against this lane's key: rows of the MFMA result = queries
    // 32 qb + 8 (i/4) + 4 hf + i%4, column = the key.  Nothing is masked: a query row beyond the
    // sequence has q = dO = 0 in LDS and lse = D = 0, so its probability is 2^0 and it multiplies
    // zeros in both products; a key beyond the sequence is a lane of its own (an MFMA column),
    // whose results are not stored.
    auto scores = [&](int qb) {
        f32x16 sacc = att_zero16();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bf16x8 qa = *(const bf16x8 *)(Qs + (qb * 32 + l32) * ATT_LDR + c * 16 + hf * 8);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[c], sacc, 0, 0, 0);
        }
        return sacc;
    };
    auto store = [&](const f32x16 (&acc)[2], long long col0, float mul) {
        if (key < S) {
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 r = {(bf16_t)(acc[fb][4 * g] * mul), (bf16_t)(acc[fb][4 * g + 1] * mul),
                                (bf16_t)(acc[fb][4 * g + 2] * mul), (bf16_t)(acc[fb][4 * g + 3] * mul)};
                    *(bf16x4 *)(dst + col0 + fb * 32 + g * 8 + hf * 4) = r;
                }
        }
    };

    // pass 1: dV^T = dO^T P
    f32x16 acc2[2] = {att_zero16(), att_zero16()};
    for (int qb = 0; qb < nb; ++qb) {
        const f32x16 sacc = scores(qb);
        float p[16];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int q0 = qb * 32 + g * 8 + hf * 4;
            const float4 l4 = *(const float4 *)(Ls + q0);
            const float lq[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
            for (int r = 0; r < 4; ++r) p[4 * g + r] = __builtin_amdgcn_exp2f(fmaf(sacc[4 * g + r], a.c2, -lq[r]));
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bf16x8 pb = att_pack8(p, c);
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
                acc2[fb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(att_read_tr(dOs, qb * 32 + 16 * c, fb, lane), pb, acc2[fb], 0, 0, 0);
        }
    }
    store(acc2, 2LL * a.d, 1.0f);

    // pass 2: dK^T = Q^T dS
    bf16x8 vf[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) vf[c] = *(const bf16x8 *)(base + (long long)krow * ld + 2 * a.d + c * 16 + hf * 8);
    acc2[0] = att_zero16(); acc2[1] = att_zero16();
    for (int qb = 0; qb < nb; ++qb) {
        const f32x16 sacc = scores(qb);
        f32x16 dpacc = att_zero16();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bf16x8 da = *(const bf16x8 *)(dOs + (qb * 32 + l32) * ATT_LDR + c * 16 + hf * 8);
            dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da, vf[c], dpacc, 0, 0, 0);
        }
        float ds[16];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int q0 = qb * 32 + g * 8 + hf * 4;
            const float4 l4 = *(const float4 *)(Ls + q0), d4 = *(const float4 *)(Ds + q0);
            const float lq[4] = {l4.x, l4.y, l4.z, l4.w}, dq[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = 4 * g + r;
                ds[i] = __builtin_amdgcn_exp2f(fmaf(sacc[i], a.c2, -lq[r])) * (dpacc[i] - dq[r]);
            }
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bf16x8 sb = att_pack8(ds, c);
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
                acc2[fb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(att_read_tr(Qs, qb * 32 + 16 * c, fb, lane), sb, acc2[fb], 0, 0, 0);
        }
    }
    store(acc2, a.d, a.scale);
}

// Backward, dQ: wavefront w owns queries 32w.. (lanes = queries) and walks the key blocks.
//   dQ = dS K / sqrt(dk), computed as dQ^T = K^T dS^T with dS^T in the registers
__global__ __launch_bounds__(64 * ATT_MAXB, 4) void attn_bwd_q_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(16))) bf16_t Ks[ATT_TILE];
    __shared__ __attribute__((aligned(16))) bf16_t Vs[ATT_TILE];
    const int seq = blockIdx.x, head = blockIdx.y, z = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, l32 = lane & 31;
    const int S = a.S, nb = a.nb;
    const long long ld = 3LL * a.d, tok0 = (long long)seq * S;
    const bf16_t *base = a.QKV + (long long)z * a.sQKV + tok0 * ld + head * ATT_DK;
    const bf16_t *dob = a.DO + (long long)z * a.sDO + tok0 * a.d + head * ATT_DK;
    const bf16_t *ob = a.O + (long long)z * a.sO + tok0 * a.d + head * ATT_DK;

    att_load_tile(Ks, base + a.d, ld, S, nb, tid);
    att_load_tile(Vs, base + 2 * a.d, ld, S, nb, tid);
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

    // Keys beyond the sequence exist only in the last block: only there the probabilities are masked
    // (their K and V rows are zero in LDS, but 2^(-lse) need not be finite).
    f32x16 dqt[2] = {att_zero16(), att_zero16()};
    auto block = [&](int kb, auto masked) {
        f32x16 sacc = att_zero16(), dpacc = att_zero16();
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
            float pv = __builtin_amdgcn_exp2f(fmaf(sacc[i], a.c2, -L));
            if (decltype(masked)::value && kb * 32 + (i >> 2) * 8 + hf * 4 + (i & 3) >= S) pv = 0.f;
            ds[i] = pv * (dpacc[i] - D);
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bf16x8 sb = att_pack8(ds, c);
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
                dqt[fb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(att_read_tr(Ks, kb * 32 + 16 * c, fb, lane), sb, dqt[fb], 0, 0, 0);
        }
    };
    for (int kb = 0; kb < nb - 1; ++kb) block(kb, std::false_type{});
    block(nb - 1, std::true_type{});
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
        lds_limit_raised = true;
    }
    dim3 grid((unsigned)(a.M / a.S), (unsigned)heads, (unsigned)K);
    attn_bwd_kv_kernel<<<grid, 64 * a.nb, ATT_BWD_KV_SMEM, s>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    attn_bwd_q_kernel<<<grid, 64 * a.nb, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace qsr
