// gemm_pp.h -- batched bf16 GEMM for gfx950 with persistent workgroups and a two-group
// ("ping-pong") schedule.  Same contraction and operand conventions as gemm_bf16.h:
//
//     NT:  C[z][m][n] = sum_k A[z][m][k] * B[z][n][k]      (both operands K-contiguous)
//     TN:  C[z][m][n] = sum_k A[z][k][m] * B[z][k][n]      (both operands stored [k][feature])
//
// What differs from the kernels in gemm_bf16.h, and why (all measured on MI355X, tokens x width
// x hidden = 12608 x 768 x 3072, 8 workers):
//
//  * One workgroup per compute unit walks a list of tiles.  The slabs of all its tiles form one
//    continuous stream through a ring of NS LDS stages (32 reduction steps each), so the copies
//    for the next tile are in flight while the epilogue of the current one runs, and a tile
//    never starts with an empty ring.
//  * The 8 wavefronts form two groups (the upper and the lower half of the tile's rows; the two
//    wavefronts that share a SIMD belong to different groups).  A group alternates between a
//    memory phase (fragments of one slab LDS -> registers, issue of the copies NS-1 slabs ahead)
//    and a multiply phase (16 or 18 MFMAs on those registers), separated by workgroup barriers,
//    and the second group runs one phase behind the first: while one wavefront of a SIMD
//    multiplies, the other fetches.  With the operands already in L2 this loop runs at
//    2.0 PFLOP/s (the plain MFMA issue rate of the chip is 2.18); the common-barrier loop of
//    gemm_bf16.h reaches 1.05.
//  * Tile order: worker, then panels of 4 N-tiles, then M-tile, then N-tile inside the panel;
//    each XCD (workgroup id mod 8) takes a contiguous eighth of that order and its workgroups
//    walk it side by side.  One XCD's L2 then sees one worker's weights only, and the tiles that
//    run together share their A rows and B rows: 30-45 % fewer bytes fetched into L2 than with
//    one launch dimension per worker.
//  * The epilogue passes each wavefront's block through a private 16-row LDS area (outside the
//    ring, which is busy) and ends by draining its stores, so that the counted waits of the ring
//    only ever see copies.
//
// The copies are global_load_lds_dwordx4 written as inline asm: seen as a builtin, the compiler
// treats every LDS access of the epilogue as possibly aliasing the copies in flight and waits
// for all outstanding vector memory operations (its own stores included) before each of them.
//
// lda/ldb must be multiples of 8 elements and N a multiple of 4.  M and N may be ragged (operand
// rows or columns clamped on load, the epilogue is bounds-checked).  NT: K a multiple of 32.
// TN: M and N multiples of 8; K may be ragged if GemmNT::zeros is given (k-rows beyond K are read
// from there).
#pragma once
#include <type_traits>

#include "gemm_bf16.h"

namespace qsr {

// A wavefront's TM x 2 blocks of 32 x 32 accumulators go out through `stage` (16 rows x 64
// floats, private to the wavefront), 16 rows at a time; the float4 slots of a row are
// XOR-swizzled with the row, which makes both the column-owner writes and the row-owner reads
// conflict-free without padding (ring + staging fill the 160 KB exactly).  Functor protocol as in
// epilogue_via_lds.
template <int TM, class Epi>
__device__ __forceinline__ void epilogue_via_lds16(f32x16 (&acc)[TM][2], float *stage, int lane,
                                                   int row0, int col0, int M, int N, int z, const Epi &epi)
{
    const int r_w = lane & 15, c4 = lane & 15, col = col0 + c4 * 4;
    // What the functor reads from global memory is requested one pass ahead, before the stores of
    // the pass in between: vector memory operations complete in order, so a wait for loads issued
    // after a pass's stores would also wait for those stores.  Unconditional, with coordinates
    // clamped into the matrix: no branch, so the loads of a pass are issued together.
    typename Epi::Aux aux[2][4];
    auto request = [&](int pass, int buf) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int row = row0 + pass * 16 + it * 4 + (lane >> 4);
            aux[buf][it] = epi.pre(z, min(row, M - 1), min(col, N - 4));
        }
    };
    request(0, 0);
#pragma unroll
    for (int pass = 0; pass < 2 * TM; ++pass) {
        const int i = pass >> 1, h = pass & 1;
        if (pass + 1 < 2 * TM) request(pass + 1, (pass + 1) & 1);
        if (((lane >> 4) & 1) == h) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int eg = 0; eg < 4; ++eg) {
                    const int slot = j * 8 + eg * 2 + (lane >> 5);
                    *(float4 *)(stage + r_w * 64 + ((slot ^ r_w) * 4)) =
                        make_float4(acc[i][j][eg * 4 + 0], acc[i][j][eg * 4 + 1], acc[i][j][eg * 4 + 2],
                                    acc[i][j][eg * 4 + 3]);
                }
        }
        __builtin_amdgcn_wave_barrier();               // LDS executes a wavefront's accesses in order
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int r = it * 4 + (lane >> 4);
            const float4 t = *(const float4 *)(stage + r * 64 + ((c4 ^ r) * 4));
            const int row = row0 + pass * 16 + r;
            if (row < M && col < N) {
                const float v[4] = {t.x, t.y, t.z, t.w};
                epi(z, row, col, v, aux[pass & 1][it]);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// TNMODE = false: NT form, tile 256 x 256 (wavefront 128 x 64), NS = 4 stages, slabs of all tiles
//                 in one continuous stream, epilogue staged outside the ring.
// TNMODE = true : TN form, tile 192 x 384 (wavefront 96 x 96): 768 x 3072 outputs per worker are
//                 32 such tiles, so 8 workers fill 256 compute units exactly once.  The reduction
//                 runs over the tokens (hundreds of slabs per tile), so the ring is simply drained
//                 and primed again between tiles and the epilogue is staged inside it.
template <bool TNMODE, int NS, class Epi>
__global__ __launch_bounds__(512) void gemm_pp_kernel(GemmNT p, Epi epi, int Z)
{
    constexpr int BM = TNMODE ? 192 : 256, BN = TNMODE ? 384 : 256, BK = 32, WN = 4;
    constexpr int TM = BM / 2 / 32, TN = BN / WN / 32;
    constexpr int PANEL = 4;                       // N-tiles per panel of the tile order
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    constexpr int A_CHUNKS = BM * BK * 2 / 1024, CHUNKS = (BM + BN) * BK * 2 / 1024;
    constexpr int CPW = (CHUNKS + 7) / 8;          // 1 KiB chunks per wavefront and slab
    constexpr bool CONT = !TNMODE;                 // continuous ring across tiles
    extern __shared__ __attribute__((aligned(1024))) unsigned char gemm_smem[];
    // epilogue staging of the continuous form: its own object, apart from the (busy) ring
    __shared__ __attribute__((aligned(16))) float stage_lds[CONT ? 8 * 16 * 64 : 4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;       // wm is also the ping-pong group
    const int nx = (p.N + BN - 1) / BN, ny = (p.M + BM - 1) / BM;
    const int nk = (p.K + BK - 1) / BK;            // TN: a ragged last slab is filled up with zero rows
    const int per_z = nx * ny, T = Z * per_z, Tc = (T + 7) / 8;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    const int c0 = xcd * Tc, c1 = min(T, c0 + Tc);
    const int n_my = c1 - c0 > slot ? (c1 - c0 - slot + slots - 1) / slots : 0;
    if (n_my == 0) return;
    auto decode = [&](int i, int &z, int &m0, int &n0) {
        const int f = c0 + slot + i * slots;
        z = f / per_z;
        int r = f - z * per_z;
        const int pn = r / (ny * PANEL);
        r -= pn * ny * PANEL;
        const int bw = min(PANEL, nx - pn * PANEL);
        const int my = r / bw;
        m0 = my * BM;
        n0 = (pn * PANEL + r - my * bw) * BN;
    };

    // ---- copies: chunk c of a slab is 1 KiB of LDS at c * 1024 inside the stage; wavefront w
    // copies the chunks w, w + 8, ... -----------------------------------------------------------
    // NT: chunk = 16 operand rows x 32 k (64 B each); LDS slot s of row r holds the 16-byte piece
    //     s ^ ((r >> 2) & 3) of that row (conflict-free 128-bit fragment reads).
    // TN: chunk = 16 k-rows (tokens) x 32 features of one 32-feature column block; LDS keeps
    //     [column block][32 k][32 features], which the transpose reads take without conflicts.
    const unsigned lds_ring = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)gemm_smem;
    const bf16_t *src[CPW];
    // elements per slab (uniform over the wavefront: a chunk index decides A or B)
    const long long stepA = TNMODE ? (long long)BK * p.lda : BK, stepB = TNMODE ? (long long)BK * p.ldb : BK;
    auto set_src = [&](int i) {
        int z, m0, n0;
        decode(i, z, m0, n0);
        const bf16_t *A = p.A + (long long)z * p.sA;
        const bf16_t *B = p.B + (long long)z * p.sB;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int chunk = c * 8 + wave;
            const bool isA = chunk < A_CHUNKS;
            const int cc = isA ? chunk : chunk - A_CHUNKS;
            if (!TNMODE) {
                const int row = cc * 16 + (lane >> 2);
                const int piece = (lane & 3) ^ ((row >> 2) & 3);
                src[c] = isA ? A + (long long)min(m0 + row, p.M - 1) * p.lda + piece * 8
                             : B + (long long)min(n0 + row, p.N - 1) * p.ldb + piece * 8;
            } else {
                const int fblk = cc >> 1, t = (cc & 1) * 16 + (lane >> 2);   // column block, k-row inside the slab
                const int f = fblk * 32 + (lane & 3) * 8;
                src[c] = isA ? A + (long long)t * p.lda + min(m0 + f, p.M - 8)
                             : B + (long long)t * p.ldb + min(n0 + f, p.N - 8);
            }
        }
    };
    int d_stage = 0;                                // stage the next copy goes to
    int d_row = 0;                                  // TN: first k-row of the next slab to copy
    auto issue_slab = [&]() {                       // copies this wavefront's chunks of the next slab
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int chunk = c * 8 + wave;
            if (CHUNKS % 8 == 0 || chunk < CHUNKS) {
                const unsigned dst = __builtin_amdgcn_readfirstlane(lds_ring + d_stage * STAGE_BYTES + chunk * 1024);
                const bf16_t *g = src[c];
                if (TNMODE) {
                    const int cc = chunk < A_CHUNKS ? chunk : chunk - A_CHUNKS;
                    if (d_row + (cc & 1) * 16 + (lane >> 2) >= p.K) g = p.zeros + (lane & 3) * 8;
                }
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
    auto zero_acc = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    };
    bf16x8 fa[2][TM], fb[2][TN];
    // TN: lane's place in the transpose reads (see gemm_tn_bf16_kernel): k offset and feature
    // offset inside a 16-k x 32-feature operand block
    const int grp = lane >> 4, r16 = lane & 15;
    const int tok_off = (grp >> 1) * 8 + (r16 >> 2), feat_off = (grp & 1) * 16 + (r16 & 3) * 4;
    auto load_frags = [&](int stage) {
        const bf16_t *sa = (const bf16_t *)(gemm_smem + stage * STAGE_BYTES), *sb = sa + BM * BK;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if (!TNMODE) {
                const int piece = ks * 2 + (lane >> 5);
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int row = wm * (BM / 2) + i * 32 + (lane & 31);
                    fa[ks][i] = *(const bf16x8 *)(sa + row * BK + ((piece ^ ((row >> 2) & 3)) * 8));
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int row = wn * (BN / WN) + j * 32 + (lane & 31);
                    fb[ks][j] = *(const bf16x8 *)(sb + row * BK + ((piece ^ ((row >> 2) & 3)) * 8));
                }
            } else {
                typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
                auto frag = [&](const bf16_t *blk) {   // blk: [32 k][32 features] of one column block
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
        }
    };
    auto mfmas = [&]() {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks][j], fa[ks][i], acc[i][j], 0, 0, 0);
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
    typedef std::integral_constant<int, 0> none_out;
    typedef std::integral_constant<int, NS - 2> younger_out;

    // S: slabs in the stream that is primed once (all tiles, or one tile at a time)
    const int S = CONT ? n_my * nk : nk;
    int d_tile = 0, d_k = 0;                        // tile and slab the next copy belongs to (continuous form)
    auto issue_next = [&]() {
        issue_slab();
        if (CONT && ++d_k == nk) {
            d_k = 0;
            if (++d_tile < n_my) set_src(d_tile);
        }
    };
    auto prime = [&](int tile) {
        set_src(tile);
        d_stage = 0;
        d_row = 0;
#pragma unroll
        for (int s = 0; s < NS - 1; ++s)
            if (s < S) issue_next();
        __builtin_amdgcn_s_waitcnt(0x0f70);        // vmcnt(0)
        barrier();
        if (wm == 1) barrier();                    // the second group runs one phase behind
    };

    float *stage16 = stage_lds + wave * (16 * 64);
    // TN: column sums of B, taken from the B fragments the first group already holds for its MFMAs:
    // lane l of a fragment has 8 consecutive k of column l % 32, which one dot product with ones
    // per register pair adds up (v_dot2c_f32_bf16), in the shadow of the multiply phase.
    float csum[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) csum[j] = 0.f;
    int c_stage = 0;
    if (CONT) prime(0);
    for (int ti = 0, q = 0; ti < n_my; ++ti) {
        int cz, cm0, cn0;
        decode(ti, cz, cm0, cn0);
        if (!CONT) { prime(ti); c_stage = 0; q = 0; }
        zero_acc();
        const bool colsum_wg = TNMODE && p.colsum_B != nullptr && cm0 == 0;
        const bool do_colsum = colsum_wg && wm == 0;
        for (int k = 0; k < nk; ++k, ++q) {
            load_frags(c_stage);
            c_stage = c_stage + 1 == NS ? 0 : c_stage + 1;
            if (q + NS - 1 < S) {
                issue_next();
                wait_copies(younger_out{});        // this wavefront's share of slab q+1 has landed
            } else {
                wait_copies(none_out{});
            }
            barrier();
            __builtin_amdgcn_s_setprio(1);
            mfmas();
            if (do_colsum) {
                // the workgroups of the first M-tile add up the k-rows of their B slabs (fixed
                // order): the bias gradient that goes with the weight gradient
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
        if constexpr (CONT) {
            epilogue_via_lds16<TM>(acc, stage16, lane, cm0 + wm * (BM / 2), cn0 + wn * (BN / WN), p.M, p.N, cz, epi);
            __builtin_amdgcn_s_waitcnt(0x0f70);    // vmcnt(0): stores drained, only copies are counted from here on
        } else {
            if (wm == 0) barrier();                // both groups are through with the ring
            constexpr int EPI_FLOATS = 8 * 32 * (TN * 32 + 4);
            static_assert((EPI_FLOATS + 2 * BN) * 4 <= NS * STAGE_BYTES, "staging inside the ring");
            float *cs_part = (float *)gemm_smem + EPI_FLOATS;       // [k half of the fragment][column]
            if (do_colsum) {
#pragma unroll
                for (int j = 0; j < TN; ++j) cs_part[(lane >> 5) * BN + wn * (BN / WN) + j * 32 + (lane & 31)] = csum[j];
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) csum[j] = 0.f;
            epilogue_via_lds<TM, TN>(acc, (float *)gemm_smem + wave * (32 * (TN * 32 + 4)), lane,
                                     cm0 + wm * (BM / 2), cn0 + wn * (BN / WN), p.M, p.N, cz, epi);
            __builtin_amdgcn_s_waitcnt(0x0070);    // vmcnt(0), lgkmcnt(0)
            barrier();                             // epilogues and partial column sums are written
            if (colsum_wg && tid < BN && cn0 + tid < p.N)
                p.colsum_B[(long long)cz * p.s_colsum + cn0 + tid] = cs_part[tid] + cs_part[BN + tid];
            barrier();                             // the ring is free to be primed again
        }
    }
    if (CONT && wm == 0) barrier();
}

// Whether launch_gemm_pp can take the problem (otherwise the kernels of gemm_bf16.h do).
inline bool gemm_pp_supports(const GemmNT &p, bool tn)
{
    if (p.K < 1 || p.lda % 8 != 0 || p.ldb % 8 != 0 || p.N % 4 != 0) return false;
    if (!tn) return p.K % 32 == 0;
    if (p.M % 8 != 0 || p.N % 8 != 0 || p.M < 8 || p.N < 8) return false;
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

template <bool TNMODE, class Epi>
inline hipError_t launch_gemm_pp(const GemmNT &p, const Epi &epi, int batch, hipStream_t s)
{
    constexpr int NS = TNMODE ? 3 : 4;        // TN: 3 stages timed 4-6 % faster than 4
    constexpr int BM = TNMODE ? 192 : 256, BN = TNMODE ? 384 : 256;
    constexpr size_t smem = (size_t)NS * (BM + BN) * 32 * 2;
    constexpr size_t stage = TNMODE ? 16 : (size_t)8 * 16 * 64 * 4;
    static_assert(smem + stage <= 160 * 1024, "ring + epilogue staging do not fit the 160 KB LDS");
    static_assert(!TNMODE || (size_t)8 * 32 * (BN / 4 + 4) * 4 <= smem, "TN epilogue staging inside the ring");
    auto kern = gemm_pp_kernel<TNMODE, NS, Epi>;
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
