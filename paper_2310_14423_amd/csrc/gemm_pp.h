// gemm_pp.h -- batched bf16 "TN" GEMM for gfx950 with persistent workgroups and a two-group
// ("ping-pong") schedule: the weight gradients of the residual-MLP workload,
//
//     C[z][m][n] = sum_k A[z][k][m] * B[z][k][n]      (both operands stored [k][feature], k = token)
//
// so the 8 consecutive k a lane of the MFMA needs lie in 8 different rows.  The slabs are staged in
// LDS as they are in memory (tokens x features) and the fragments are fetched with the gfx950 LDS
// transpose read (ds_read_b64_tr_b16): within each group of 16 lanes, lane j receives element
// j%4 of the 64-bit words addressed by lanes j/4, j/4+4, j/4+8, j/4+12 of the group (checked on
// the hardware).  Pointing lane r = q + 4e of a group at token e, features 4q..4q+3 of a
// 4-token x 16-feature block therefore hands lane j feature j and the 4 tokens in order; two
// such reads give the 8 k values of an MFMA operand, and the four groups of a wavefront cover
// 32 features x 16 tokens in exactly the instruction's operand layout.
// Design, and what it was measured against (MI355X: 768 x 3072 outputs, 12608 tokens, 8 workers; a
// first version with 128 x 128 tiles, register-staged copies and a common barrier per slab took
// 743 us per launch, this one 434):
//
//  * Tiles of 192 x 384 (wavefront 96 x 96).  768 x 3072 outputs per worker are 32 such tiles, so
//    8 workers fill the 256 compute units exactly once: no tail, and per multiply-add half the
//    bytes fetched from L2 of the 128 x 128 tiles, which bound the plain kernel.
//  * One workgroup per compute unit walks its list of tiles (usually one).  Tile order: worker,
//    panels of 4 N-tiles, M-tile, N-tile inside the panel; each XCD (workgroup id mod 8) takes a
//    contiguous eighth of that order: one XCD's L2 sees one worker's activations.
//  * Slabs of 32 tokens are copied global -> LDS directly (global_load_lds_dwordx4) into a ring of
//    NS stages, NS-1 slabs ahead.  LDS keeps [32-feature column block][32 tokens][32 features], the
//    form the transpose reads (ds_read_b64_tr_b16) take without bank conflicts.  Token rows beyond
//    K are read from a block of zeros.
//  * The 8 wavefronts form two groups (the upper and the lower half of the tile's rows; the two
//    wavefronts that share a SIMD belong to different groups).  A group alternates between a
//    memory phase (fragments of one slab LDS -> registers, issue of the next copies) and a multiply
//    phase (18 MFMAs on those registers), separated by workgroup barriers, and the second group
//    runs one phase behind the first: while one wavefront of a SIMD multiplies, the other fetches.
//    (The same loop in NT form ran at 2.0 PFLOP/s with its operands in L2, against 1.05 for the
//    common-barrier loop of gemm_bf16.h and 2.18 for bare MFMA issue.  For the NT GEMMs of this
//    workload it still did not pay: they are bound by L2 delivery and by their epilogues, and a
//    persistent workgroup must see its epilogue's stores complete before it can count copies
//    again, where a fresh workgroup starts at once.)
//  * Bias gradients (column sums of B over the tokens) come from the B fragments the first group
//    already holds for its MFMAs: one bf16 dot product with ones per register pair, in the shadow
//    of the multiply phase.  Re-reading the slabs from LDS for them made the workgroups of the
//    first M-tile 35 % slower than the rest.
//
//  * Problems with few tiles (a 768 x 768 gradient for 8 workers is 64) can have the reduction cut
//    into ranges (GemmNT::split): each (tile, range) is a work item of its own, handed to the epilogue
//    as a batch entry of its own; the caller adds the partial results up in a fixed order.
//
// The copies are written as inline asm: seen as a builtin, the compiler treats every later LDS
// access as possibly aliasing the copies in flight and waits for all outstanding vector memory
// operations before it.
//
// lda/ldb must be multiples of 8 elements, M and N multiples of 8 (ragged against the tile: operand
// columns are clamped on load, the epilogue is bounds-checked); K may be ragged if GemmNT::zeros
// is given.
#pragma once
#include <type_traits>

#include "gemm_bf16.h"

namespace qsr {

// BLKA / BLKB: the operand is stored in 32-token x 32-feature blocks (gemm_bf16.h); lda / ldb then
// hold its feature count.  A 1 KiB chunk of a slab (16 tokens x 32 features of one column block) is
// then 1 KiB of consecutive memory, and a whole slab of a tile one piece of 12 or 24 KiB; row-major
// a chunk is 16 pieces of 64 B a whole row apart.  Either way a slab lies 32 * ld elements behind
// the one before.
template <int NS, bool BLKA, bool BLKB, class Epi>
__global__ __launch_bounds__(512) void gemm_pp_tn_kernel(GemmNT p, Epi epi, int Z)
{
    constexpr int BM = 192, BN = 384, BK = 32, WN = 4;
    constexpr int TM = BM / 2 / 32, TN = BN / WN / 32;            // 3 x 3 blocks of 32 x 32 per wavefront
    constexpr int PANEL = 4;                                      // N-tiles per panel of the tile order
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;               // 36 KB
    constexpr int A_CHUNKS = BM * BK * 2 / 1024, CHUNKS = (BM + BN) * BK * 2 / 1024;
    constexpr int CPW = (CHUNKS + 7) / 8;                         // 1 KiB chunks per wavefront and slab
    extern __shared__ __attribute__((aligned(1024))) unsigned char gemm_smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;                     // wm is also the ping-pong group
    const int nx = (p.N + BN - 1) / BN, ny = (p.M + BM - 1) / BM;
    const int split = p.split > 1 ? p.split : 1;                  // ranges of the reduction, each a work item
    const int per_z = nx * ny, T = Z * split * per_z, Tc = (T + 7) / 8;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    const int c0 = xcd * Tc, c1 = min(T, c0 + Tc);
    const int n_my = c1 - c0 > slot ? (c1 - c0 - slot + slots - 1) / slots : 0;
    if (n_my == 0) return;
    // work item i of this workgroup: zz = batch * split + range, and the tile's origin
    auto decode = [&](int i, int &zz, int &m0, int &n0) {
        const int f = c0 + slot + i * slots;
        zz = f / per_z;
        int r = f - zz * per_z;
        const int pn = r / (ny * PANEL);
        r -= pn * ny * PANEL;
        const int bw = min(PANEL, nx - pn * PANEL);
        const int my = r / bw;
        m0 = my * BM;
        n0 = (pn * PANEL + r - my * bw) * BN;
    };

    // ---- copies: chunk c of a slab is 1 KiB of LDS at c * 1024 inside the stage (16 tokens x 32
    // features of one column block); wavefront w copies the chunks w, w + 8, ... ----------------
    const unsigned lds_ring = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)gemm_smem;
    const bf16_t *src[CPW];
    const long long stepA = (long long)BK * p.lda, stepB = (long long)BK * p.ldb;   // elements per slab
    int k_end = p.K;                                // end of the current item's range of the reduction
    int d_stage = 0;                                // stage the next copy goes to
    int d_row = 0;                                  // first token of the next slab to copy
    auto set_src = [&](int i) {
        int zz, m0, n0;
        decode(i, zz, m0, n0);
        const int z = zz / split, k0 = (zz - z * split) * (split > 1 ? p.k_chunk : 0);
        k_end = split > 1 ? min(p.K, k0 + p.k_chunk) : p.K;
        d_row = k0;
        d_stage = 0;
        const bf16_t *A = p.A + (long long)z * p.sA + (long long)k0 * p.lda;     // k0 is a multiple of 32:
        const bf16_t *B = p.B + (long long)z * p.sB + (long long)k0 * p.ldb;     // the first block row of the range
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int chunk = c * 8 + wave;
            const bool isA = chunk < A_CHUNKS;
            const int cc = isA ? chunk : chunk - A_CHUNKS;
            const int fblk = cc >> 1, t = (cc & 1) * 16 + (lane >> 2);   // column block, token inside the slab
            const int f = fblk * 32 + (lane & 3) * 8;
            if (isA) {
                const int fc = min(m0 + f, p.M - 8);
                src[c] = BLKA ? A + (long long)(fc >> 5) * 1024 + t * 32 + (fc & 31) : A + (long long)t * p.lda + fc;
            } else {
                const int fc = min(n0 + f, p.N - 8);
                src[c] = BLKB ? B + (long long)(fc >> 5) * 1024 + t * 32 + (fc & 31) : B + (long long)t * p.ldb + fc;
            }
        }
    };
    auto issue_slab = [&]() {                       // copies this wavefront's chunks of the next slab
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int chunk = c * 8 + wave;
            if (CHUNKS % 8 == 0 || chunk < CHUNKS) {
                const unsigned dst = __builtin_amdgcn_readfirstlane(lds_ring + d_stage * STAGE_BYTES + chunk * 1024);
                const int cc = chunk < A_CHUNKS ? chunk : chunk - A_CHUNKS;
                const bf16_t *g = d_row + (cc & 1) * 16 + (lane >> 2) < k_end ? src[c] : p.zeros + (lane & 3) * 8;
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(dst), "v"(g) : "memory", "m0");
                src[c] += __builtin_amdgcn_readfirstlane(chunk) < A_CHUNKS ? stepA : stepB;
            }
        }
        d_stage = d_stage + 1 == NS ? 0 : d_stage + 1;
        d_row += BK;
    };
    // wavefronts whose last chunk index lies beyond the slab issue one copy less per slab
    const bool short_wave = CHUNKS % 8 != 0 && (CPW - 1) * 8 + wave >= CHUNKS;

    f32x16 acc[TM][TN];
    bf16x8 fa[2][TM], fb[2][TN];
    // lane's place in the transpose reads: token and feature offset
    // inside a 16-token x 32-feature operand block
    const int grp = lane >> 4, r16 = lane & 15;
    const int tok_off = (grp >> 1) * 8 + (r16 >> 2), feat_off = (grp & 1) * 16 + (r16 & 3) * 4;
    auto load_frags = [&](int stage) {
        const bf16_t *sa = (const bf16_t *)(gemm_smem + stage * STAGE_BYTES), *sb = sa + BM * BK;
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            auto frag = [&](const bf16_t *blk) {    // blk: [32 tokens][32 features] of one column block
                const bf16_t *q0 = blk + (ks * 16 + tok_off) * 32 + feat_off;
                union { struct { s16x4 a, b; } s; bf16x8 v; } u;
                u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)q0);
                u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(q0 + 4 * 32));
                return u.v;
            };
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[ks][i] = frag(sa + (wm * TM + i) * (32 * 32));
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[ks][j] = frag(sb + (wn * TN + j) * (32 * 32));
        }
    };
    auto barrier = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    // waits until at most `slabs` of this wavefront's slab copies are outstanding, and for its LDS reads
    auto wait_copies = [&](auto slabs) {
        constexpr int FULL = CPW * decltype(slabs)::value, SHORT = (CPW - 1) * decltype(slabs)::value;
        if (short_wave) __builtin_amdgcn_s_waitcnt(0x0070 | (SHORT & 15) | ((SHORT >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0070 | (FULL & 15) | ((FULL >> 4) << 14));
    };

    // column sums of B: lane l of a B fragment has 8 consecutive tokens of column l % 32
    float csum[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) csum[j] = 0.f;

    for (int ti = 0; ti < n_my; ++ti) {
        int cz, cm0, cn0;
        decode(ti, cz, cm0, cn0);
        // prime the ring with the first NS-1 slabs of the item
        set_src(ti);
        const int nk = (k_end - d_row + BK - 1) / BK;             // a ragged last slab is filled up with zero rows
#pragma unroll
        for (int s = 0; s < NS - 1; ++s)
            if (s < nk) issue_slab();
        __builtin_amdgcn_s_waitcnt(0x0f70);        // vmcnt(0)
        barrier();
        if (wm == 1) barrier();                    // the second group runs one phase behind
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
        const bool colsum_wg = p.colsum_B != nullptr && cm0 == 0;
        const bool do_colsum = colsum_wg && wm == 0;
        int c_stage = 0;
        for (int k = 0; k < nk; ++k) {
            // memory phase
            load_frags(c_stage);
            c_stage = c_stage + 1 == NS ? 0 : c_stage + 1;
            if (k + NS - 1 < nk) {
                issue_slab();
                wait_copies(std::integral_constant<int, NS - 2>{});   // this wavefront's share of slab k+1 has landed
            } else {
                wait_copies(std::integral_constant<int, 0>{});
            }
            barrier();
            // multiply phase
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks][j], fa[ks][i], acc[i][j], 0, 0, 0);
            if (do_colsum) {
                // the first group of the workgroups of the first M-tile adds up the tokens of its B
                // fragments (fixed order): the bias gradient that goes with the weight gradient
                typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const bf16x2 two = {fb[ks][j][2 * e], fb[ks][j][2 * e + 1]};
                            csum[j] = __builtin_amdgcn_fdot2_f32_bf16(two, ones, csum[j], false);
                        }
            }
            __builtin_amdgcn_s_setprio(0);
            barrier();
        }
        if (wm == 0) barrier();                    // both groups are through with the ring
        // epilogue staged inside the ring; behind it the two halves of the column sums
        constexpr int EPI_FLOATS = 8 * 32 * (TN * 32 + 4);
        static_assert((EPI_FLOATS + 2 * BN) * 4 <= NS * STAGE_BYTES, "staging inside the ring");
        float *cs_part = (float *)gemm_smem + EPI_FLOATS;          // [token half of the fragment][column]
        if (do_colsum) {
#pragma unroll
            for (int j = 0; j < TN; ++j) cs_part[(lane >> 5) * BN + wn * (BN / WN) + j * 32 + (lane & 31)] = csum[j];
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) csum[j] = 0.f;
        epilogue_via_lds<TM, TN>(acc, (float *)gemm_smem + wave * (32 * (TN * 32 + 4)), lane,
                                 cm0 + wm * (BM / 2), cn0 + wn * (BN / WN), p.M, p.N, cz, epi);
        __builtin_amdgcn_s_waitcnt(0x0070);        // vmcnt(0), lgkmcnt(0)
        barrier();                                 // epilogues and partial column sums are written
        if (colsum_wg && tid < BN && cn0 + tid < p.N)
            p.colsum_B[(long long)cz * p.s_colsum + cn0 + tid] = cs_part[tid] + cs_part[BN + tid];
        barrier();                                 // the ring is free to be primed again
    }
}

// Whether launch_gemm_pp_tn can take the problem.
inline bool gemm_pp_tn_supports(const GemmNT &p)
{
    if (p.K < 1 || p.lda % 8 != 0 || p.ldb % 8 != 0) return false;
    if (p.M % 8 != 0 || p.N % 8 != 0 || p.M < 8 || p.N < 8) return false;
    if (p.split > 1 && (p.k_chunk < 32 || p.k_chunk % 32 != 0 || (long long)(p.split - 1) * p.k_chunk >= p.K)) return false;
    return p.K % 32 == 0 || p.zeros != nullptr;
}

// compute units of the current device (one persistent workgroup each)
inline int gemm_pp_cu_count()
{
    static int n_cu = 0;                      // contexts are not thread-safe; one GPU per process
    if (n_cu == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 8)
            n_cu = 256;
    }
    return n_cu;
}

template <bool BLKA, bool BLKB, class Epi>
inline hipError_t launch_gemm_pp_tn(const GemmNT &p, const Epi &epi, int batch, hipStream_t s)
{
    // blocked operands: 32-column blocks (the ranges of a split reduction start at multiples of 32 tokens)
    if ((BLKA && p.lda % 32 != 0) || (BLKB && p.ldb % 32 != 0)) return hipErrorInvalidValue;
    constexpr int NS = 3;                     // 3 stages timed 4-6 % faster than 4
    constexpr size_t smem = (size_t)NS * (192 + 384) * 32 * 2;
    static_assert(smem <= 160 * 1024, "ring does not fit the 160 KB LDS");
    auto kern = gemm_pp_tn_kernel<NS, BLKA, BLKB, Epi>;
    static bool lds_limit_raised = false;     // per instantiation; contexts are not thread-safe
    if (!lds_limit_raised) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        lds_limit_raised = true;
    }
    const int grid = gemm_pp_cu_count() / 8 * 8;
    kern<<<grid, 512, smem, s>>>(p, epi, batch);
    return hipGetLastError();
}

}  // namespace qsr
