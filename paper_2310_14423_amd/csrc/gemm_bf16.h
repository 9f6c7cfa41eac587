// gemm_bf16.h -- batched bf16 x bf16 -> fp32 GEMM on the gfx950 matrix cores, "NT" form:
//
//     C[z][m][n] = sum_k A[z][m][k] * B[z][n][k]        (both operands K-contiguous)
//
// which is the operand order the MFMA instruction wants: v_mfma_f32_32x32x16_bf16 takes, per
// lane, 8 consecutive k of one row of A and 8 consecutive k of one column of B.  Lane layout
// (checked on the hardware): lane l holds A[row l%32][k (l/32)*8 .. +7], B[k (l/32)*8 .. +7]
// [col l%32], and accumulator element i is D[(i/4)*8 + (l/32)*4 + i%4][l%32].
//
// Tiling: a workgroup of WM x WN wavefronts computes a BM x BN tile; K is walked in slabs of
// BK = 64 (or 32) staged through two LDS buffers.  The slabs are copied global -> LDS directly
// (global_load_lds_dwordx4: no register staging, no LDS store instructions), slab j+1 in
// flight while slab j is multiplied.  That instruction writes 64 lanes x 16 B to 1 KiB of
// consecutive LDS, so rows are stored unpadded (8 pieces of 16 B) and bank conflicts are
// avoided by an XOR swizzle instead: slot s of row r holds piece s ^ ((r >> 1) & 7) (BK = 32:
// s ^ ((r >> 2) & 3)), which spreads the 128-bit fragment reads of 16 consecutive rows over all
// 64 banks (measured: no conflicts).  Timed on MI355X at 12608 x 768 x 3072, batch 8: register-staged copy 0.58 ms,
// direct copy 0.49 ms, plus the XCD-aware tile order 0.47 ms (1.01 PFLOP/s).
// M and N may be ragged: out-of-range rows are clamped to the last valid row on load (they
// only feed accumulator rows that are never stored) and the epilogue is bounds-checked.
// K must be a multiple of BK and lda/ldb multiples of 8 elements (16-byte rows).
//
// The two operands are handed to the instruction in swapped roles (the B rows as its "A", the A
// rows as its "B"), so that it produces the transposed tile: lane l then owns, for token row
// m = l%32, four consecutive output columns n, which is what the epilogue's LDS staging writes
// with 128-bit stores (see epilogue_via_lds).
//
// Operand layout.  Besides plain row-major, a bf16 matrix [R][C] (C a multiple of 32) can be stored
// in blocks of 32 rows x 32 columns, each block 2 KiB contiguous, blocks ordered [row block]
// [column block] (blk_off below).  Both kinds of GEMM then copy consecutive memory: a 256-row x
// 64-deep slab of this kernel's operands is 8 pieces of 4 KiB (two neighbouring blocks) instead of
// 256 pieces of 128 B a whole row (1.5 - 6 KiB) apart, and a 32-token x 192- or 384-feature slab of
// the weight-gradient kernel (gemm_pp.h), which walks the same arrays along their rows, is 12 or
// 24 KiB in one piece instead of 32 pieces; every global -> LDS copy instruction moves 1 KiB of
// consecutive memory.  (Blocks of 256 rows x 32 columns, 32 KiB per slab here, were timed first:
// this kernel gained 3-4 %, the weight-gradient kernel, whose slab was then 2 KiB pieces exactly
// 16 KiB apart, lost 8 %.)  All weights (B operands) are blocked; activations are blocked where
// their producers write them that way (BLKA), row-major otherwise.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qsr {

// element offset of (r, c) in the blocked layout of an [R][C] matrix; R is padded to 256 rows (the
// tiles of this kernel read whole 256-row panels)
__host__ __device__ __forceinline__ long long blk_off(long long r, long long c, long long C)
{
    return ((r >> 5) * (C >> 5) + (c >> 5)) * 1024 + (r & 31) * 32 + (c & 31);
}
// elements a blocked [R][C] matrix occupies
__host__ __device__ __forceinline__ long long blk_elems(long long R, long long C) { return ((R + 255) >> 8) * 256 * C; }

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GemmNT {
    const bf16_t *A, *B;
    int M, N, K;
    long long lda, ldb;
    long long sA, sB;      // per-batch strides (elements)
    // TN form (gemm_pp.h) only:
    float *colsum_B;       // optional: colsum_B[z*s_colsum + n] = sum_k B[z][k][n]
    long long s_colsum;
    const bf16_t *zeros;   // 64 bytes of zeros, read in place of k-rows beyond K (needed if K % 32 != 0)
    int split;             // > 1: the reduction is cut into `split` ranges of k_chunk rows (a multiple of 32);
    int k_chunk;           //      range s of batch z is handed to the epilogue (and column sums) as batch z*split + s
};

// Epilogue.  The MFMA leaves lane l with 4 consecutive columns of row l%32, i.e. one store
// instruction would touch 32 different rows.  Each wavefront therefore passes its tile, 32 rows
// at a time, through a private LDS area (the slab buffers are free by then) and re-reads it
// so that 16 consecutive lanes hold one row's consecutive columns: whole 128- or 256-byte row
// segments per global instruction (N must be a multiple of 4).  Rows are padded by 16 B:
// conflict-free both ways.  The functor has two parts, so that what it reads from global memory
// can be requested one 32-row block ahead of its use:
//     Aux  epi.pre(z, m, n)            -- loads for C[z][m][n..n+3] (may be empty; also called
//                                         with coordinates clamped into the matrix, N >= 4)
//     void epi(z, m, n, v[4], aux)     -- consumes the accumulators and stores
struct NoAux {};

template <int TM, int TN, class Epi>
__device__ __forceinline__ void epilogue_via_lds(f32x16 (&acc)[TM][TN], float *stage, int lane,
                                                 int row0, int col0, int M, int N, int z, const Epi &epi)
{
    constexpr int W = TN * 32, LD = W + 4;             // floats per staged row
    constexpr int LPR = W / 4;                         // lanes per row on the way out
    constexpr int RPI = 64 / LPR;                      // rows per read instruction
    constexpr int ITERS = 32 / RPI;
    static_assert(32 % RPI == 0, "rows per instruction must divide the block");
    const bool active = lane / LPR < RPI;              // TN = 3: 24 lanes per row, the last 16 lanes idle
    const int c = (lane % LPR) * 4, col = col0 + c;
    // What the functor reads from global memory is requested one block ahead, before the stores of
    // the block in between: vector memory operations complete in order, so a wait for loads issued
    // after a block's stores would also wait for those stores.  Unconditional, with coordinates
    // clamped into the matrix: no branch, so the loads of a block are issued together.
    typename Epi::Aux aux[2][ITERS];
    auto request = [&](int i, int buf) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int row = row0 + i * 32 + min(it * RPI + lane / LPR, 31);
            aux[buf][it] = epi.pre(z, min(row, M - 1), min(col, N - 4));
        }
    };
    request(0, 0);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (i + 1 < TM) request(i + 1, (i + 1) & 1);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int eg = 0; eg < 4; ++eg)
                *(float4 *)(stage + (lane & 31) * LD + j * 32 + eg * 8 + (lane >> 5) * 4) =
                    make_float4(acc[i][j][eg * 4 + 0], acc[i][j][eg * 4 + 1], acc[i][j][eg * 4 + 2],
                                acc[i][j][eg * 4 + 3]);
        __builtin_amdgcn_wave_barrier();               // LDS executes a wavefront's accesses in order
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int r = min(it * RPI + lane / LPR, 31);
            const float4 t = *(const float4 *)(stage + r * LD + c);
            const int row = row0 + i * 32 + r;
            if (active && row < M && col < N) {
                const float v[4] = {t.x, t.y, t.z, t.w};
                epi(z, row, col, v, aux[i & 1][it]);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// BLKA: A is stored in 32 x 32 blocks (see above); B always is.  In LDS a slab of a blocked operand
// is [2 column blocks][rows][32 k], rows of 64 B, slot s of row r holding piece s ^ ((r >> 2) & 3);
// a row-major A slab is [rows][64 k] with slot = piece ^ ((r >> 1) & 7).
template <int BM, int BN, int BK, int WM, int WN, bool BLKA, class Epi>
__global__ __launch_bounds__(WM * WN * 64) void gemm_nt_bf16_kernel(GemmNT p, Epi epi, int batch)
{
    static_assert(BK == 64, "a slab is two 32-column blocks, or rows of 8 pieces of 16 B");
    static_assert(BM == 256 && BN == 256, "tiles are one row block of the blocked layout");
    constexpr int PPR = BK / 8;             // 16-byte pieces per row (row-major slab)
    constexpr int RPC = 64 / PPR;           // rows per 1 KiB chunk (row-major slab)
    constexpr int SWZ = 1;                  // row-major slab: slot = piece ^ ((row >> SWZ) & (PPR - 1))
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_CHUNKS = BM / RPC, B_CHUNKS = BN / RPC;   // 1 KiB chunks per slab
    constexpr int A_PER_WAVE = A_CHUNKS / NW, B_PER_WAVE = B_CHUNKS / NW;
    static_assert(A_CHUNKS % NW == 0 && B_CHUNKS % NW == 0, "chunks / waves");
    constexpr int STAGE_ELEMS = (BM + BN) * BK;

    extern __shared__ __attribute__((aligned(1024))) unsigned char gemm_smem[];
    bf16_t *smem = (bf16_t *)gemm_smem;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    // Workgroups go to the 8 XCDs round-robin by linear id (the grid's x extent is a multiple of
    // 8).  Tile order: batch entry (worker), then panels of 4 N-tiles, then M-tile, then N-tile
    // inside the panel; each XCD takes a contiguous eighth of that order.  One XCD's L2 then sees
    // one worker's B operand (for 8 workers), and the tiles that run together share their A rows
    // and B rows: 30-45 % fewer bytes fetched into L2 than with the batch as a grid dimension.
    const int nx = (p.N + BN - 1) / BN, ny = (p.M + BM - 1) / BM;
    int tile = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
    if (tile >= batch * nx * ny) return;
    const int z = tile / (nx * ny);
    tile -= z * nx * ny;
    constexpr int PANEL = 4;
    const int pn = tile / (ny * PANEL);
    tile -= pn * ny * PANEL;
    const int bw = min(PANEL, nx - pn * PANEL);
    const int by = tile / bw, bx = pn * PANEL + tile - by * bw;
    const int m0 = by * BM, n0 = bx * BN;
    const bf16_t *A = p.A + (long long)z * p.sA;
    const bf16_t *B = p.B + (long long)z * p.sB;

    // Per-lane global source of each 1 KiB chunk this wave copies.  Row-major operand: chunk c is 8
    // rows x 128 B, LDS slot (row, s) holds the global piece s ^ ((row >> 1) & 7) of that row.
    // Blocked operand: chunk c is 16 rows x 64 B, half of a 32 x 32 block (c / 16 the column block of
    // the slab, c % 16 the run of rows), consecutive in memory up to the permutation of the four
    // 16-byte pieces inside each row: slot s of row r holds piece s ^ ((r >> 2) & 3).  Rows beyond the
    // matrix inside the last 256-row panel are allocated (their values only reach accumulator rows
    // never stored).
    const bf16_t *srcA[A_PER_WAVE], *srcB[B_PER_WAVE];
    const int blk_lane = (lane >> 2) * 32 + (((lane & 3) ^ ((lane >> 4) & 3)) * 8);   // inside a blocked chunk
    constexpr long long A_SLAB = BLKA ? 2 * 1024 : BK, B_SLAB = 2 * 1024;              // elements per slab step
#pragma unroll
    for (int i = 0; i < A_PER_WAVE; ++i) {
        const int c = wave * A_PER_WAVE + i;
        if (BLKA) {
            srcA[i] = A + ((long long)(by * 8 + ((c & 15) >> 1)) * (p.K >> 5) + (c >> 4)) * 1024 + (c & 1) * 512 + blk_lane;
        } else {
            const int row = c * RPC + lane / PPR;
            const int piece = (lane % PPR) ^ ((row >> SWZ) & (PPR - 1));
            srcA[i] = A + (long long)min(m0 + row, p.M - 1) * p.lda + piece * 8;
        }
    }
#pragma unroll
    for (int i = 0; i < B_PER_WAVE; ++i) {
        const int c = wave * B_PER_WAVE + i;
        srcB[i] = B + ((long long)(bx * 8 + ((c & 15) >> 1)) * (p.K >> 5) + (c >> 4)) * 1024 + (c & 1) * 512 + blk_lane;
    }
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(1))) const void glb_void;
    auto issue = [&](int stage, int k0) {
        bf16_t *sa = smem + stage * STAGE_ELEMS, *sb = sa + BM * BK;
#pragma unroll
        for (int i = 0; i < A_PER_WAVE; ++i)
            __builtin_amdgcn_global_load_lds((glb_void *)(srcA[i] + (long long)(k0 / BK) * A_SLAB),
                                             (lds_void *)(sa + (wave * A_PER_WAVE + i) * 512), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < B_PER_WAVE; ++i)
            __builtin_amdgcn_global_load_lds((glb_void *)(srcB[i] + (long long)(k0 / BK) * B_SLAB),
                                             (lds_void *)(sb + (wave * B_PER_WAVE + i) * 512), 16, 0, 0);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // Main loop, software-pipelined over the 16-wide k-steps of a slab: the fragments of step
    // ks+1 are read from LDS while the MFMAs of step ks issue, and the last step of a slab is
    // held in registers across the barrier, so that its MFMAs cover the burst of first fragment
    // reads of the next slab that all wavefronts start at once after the barrier (worth 10 % at
    // K = 3072 over stopping with empty MFMA queues at every barrier).  The compiler waits for ALL
    // outstanding LDS reads in two of the four steps of a slab (lgkmcnt(0) right after the next
    // step's six reads went out); with the reads written as asm and waited for by hand (at most
    // six outstanding) every step's reads fly behind the previous step's multiplications, and the
    // kernels take the same time to 2 %: the SIMD's other wavefront already filled those gaps.
    const int nk = p.K / BK;
    constexpr int KS = BK / 16;
    static_assert(KS % 2 == 0, "fragment double buffer parity");
    bf16x8 fa[2][TM], fb[2][TN];
    auto load_frags = [&](int stage, int ks, int fbuf) {
        const bf16_t *sa = smem + stage * STAGE_ELEMS, *sb = sa + BM * BK;
        const int piece = ks * 2 + (lane >> 5);               // of the 8 pieces of a 64-deep row
        // blocked slab: column block piece / 4, rows of four pieces
        const int blk_base = (piece >> 2) * (256 * 32), bp = piece & 3;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = wm * TM * 32 + i * 32 + (lane & 31);
            if (BLKA) fa[fbuf][i] = *(const bf16x8 *)(sa + blk_base + row * 32 + ((bp ^ ((row >> 2) & 3)) * 8));
            else fa[fbuf][i] = *(const bf16x8 *)(sa + row * BK + ((piece ^ ((row >> SWZ) & (PPR - 1))) * 8));
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int row = wn * TN * 32 + j * 32 + (lane & 31);
            fb[fbuf][j] = *(const bf16x8 *)(sb + blk_base + row * 32 + ((bp ^ ((row >> 2) & 3)) * 8));
        }
    };
    auto mfmas = [&](int fbuf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[fbuf][j], fa[fbuf][i], acc[i][j], 0, 0, 0);
    };
    issue(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0f70);                // vmcnt(0): this wavefront's part of slab 0 landed
    __syncthreads();
    if (nk > 1) issue(1, BK);
    load_frags(0, 0, 0);
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
#pragma unroll
        for (int ks = 0; ks < KS - 1; ++ks) {
            load_frags(cur, ks + 1, (ks + 1) & 1);
            mfmas(ks & 1);
        }
        if (kt + 1 < nk) {
            // vmcnt(0): my part of slab kt+1 landed; lgkmcnt(0): my reads of slab kt are done
            __builtin_amdgcn_s_waitcnt(0x0070);
            __syncthreads();                           // slab kt+1 complete, slab kt's buffer free
            if (kt + 2 < nk) issue(cur, (kt + 2) * BK);
            load_frags(cur ^ 1, 0, 0);
            __builtin_amdgcn_sched_barrier(0);         // keep the pending MFMAs behind those reads
        }
        mfmas((KS - 1) & 1);
    }

    __syncthreads();                                   // every wavefront is done with the slabs
    epilogue_via_lds<TM, TN>(acc, (float *)gemm_smem + wave * (32 * (TN * 32 + 4)), lane,
                             m0 + wm * TM * 32, n0 + wn * TN * 32, p.M, p.N, z, epi);
}

typedef short s16x4 __attribute__((ext_vector_type(4)));   // operand of the LDS transpose read

template <int BM, int BN, int BK, int WM, int WN, bool BLKA, class Epi>
inline hipError_t launch_gemm_nt(const GemmNT &p, const Epi &epi, int batch, hipStream_t s)
{
    if (p.K % BK != 0 || p.K < BK) return hipErrorInvalidValue;
    const unsigned tiles = (unsigned)((p.N + BN - 1) / BN) * (unsigned)((p.M + BM - 1) / BM) * (unsigned)batch;
    dim3 grid((tiles + 7) / 8 * 8, 1, 1);
    constexpr size_t smem = 2 * (size_t)(BM + BN) * BK * sizeof(bf16_t);
    static_assert(smem <= 160 * 1024, "tile does not fit the 160 KB LDS");
    static_assert((size_t)WM * WN * 32 * (BN / WN + 4) * sizeof(float) <= smem, "epilogue staging does not fit the slab buffers");
    auto kern = gemm_nt_bf16_kernel<BM, BN, BK, WM, WN, BLKA, Epi>;
    static bool lds_limit_raised = false;     // per instantiation; contexts are not thread-safe
    if (smem > 64 * 1024 && !lds_limit_raised) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        lds_limit_raised = true;
    }
    kern<<<grid, WM * WN * 64, smem, s>>>(p, epi, batch);
    return hipGetLastError();
}

}  // namespace qsr
