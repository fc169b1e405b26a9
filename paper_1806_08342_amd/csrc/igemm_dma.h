// Pipelined variant of the implicit-GEMM kernel for the aligned, MFMA-bound cases.
//
// Same arithmetic and LDS tile layout as igemm.h, but the operand tiles go from global
// memory straight into LDS (global_load_lds_dwordx4, no register staging) through a ring
// of NSTAGE stages, so that loads run NSTAGE-1 K-steps ahead of the MFMAs that consume
// them.  One barrier per K-step, placed between the two 32-deep MFMA batches of the step;
// the fragments of the next batch are read from LDS while the current batch executes.
//
// A wave-level global_load_lds_dwordx4 writes the 64 lanes' 16-byte chunks to 1024
// consecutive LDS bytes in lane order, i.e. 16 tile rows of 64 bytes.  Lane p therefore
// fetches, for row p/4 of its segment, the logical chunk (p%4) ^ swizzle(row): the XOR
// swizzle of the tile is applied on the global-address side.
//
// Requirements (checked by the dispatcher): every 16-byte chunk is 16-byte aligned (pitches
// and base pointers multiples of 16; for convolutions Cin % 16 == 0), K % 64 == 0, and the
// byte offsets inside one tile fit 32 bits.  Rows beyond M / columns beyond N are clamped to
// the last valid one (their results are never stored); out-of-image taps of a convolution
// read a constant chunk holding the code z_x.
#pragma once

#include "fill_table.h"
#include "igemm.h"

namespace qnn {

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    // gfx9 encoding: vmcnt = {imm[15:14], imm[3:0]}, expcnt = imm[6:4], lgkmcnt = imm[11:8]
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// workgroup barrier that the compiler may not move memory operations across; unlike
// __syncthreads() it does not wait for outstanding global loads (the LDS DMA pipeline
// must stay in flight across it)
__device__ __forceinline__ void block_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

__device__ __forceinline__ void dma16(const uint8_t *src, uint8_t *lds_wave_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

// Split-K: when a product has too few output tiles to fill the chip, the K-steps of every tile
// are divided over `splits` workgroups.  Each writes its int32 partial sums (with its share of
// the zero-point correction) to plane `split` of `partial` ([splits][M][N]); a second kernel
// adds the planes and applies bias, rescale and clamp.  Integer sums: any order, same bits.
struct SplitK {
    int splits;       // workgroups per output tile (1: no split)
    int ksteps;       // K-steps of 64 per workgroup (the last one may get fewer, never zero)
    int32_t *partial; // device memory, splits * M * N int32
};

// Tile assignment: consecutive workgroup ids go round-robin over the 8 XCDs, each with
// its own L2.  xcd_rows > 0: the tile grid is cut into xcd_rows x (8 / xcd_rows) rectangles,
// one per XCD, so that an XCD fetches only 1/xcd_rows of A and xcd_rows/8 of B from beyond
// its L2.  xcd_rows == 0: every XCD gets one contiguous band of the row-major tile sequence
// (exact balance; used when the grid does not cut evenly, and with split-K).  Inside its
// share an XCD walks groups of 4 tile rows column by column, so that tiles running at the
// same time share A rows and B columns.  `slot` is the position in the XCD's sequence: workgroup
// blockIdx.x takes the slots blockIdx.x / 8 + i * gridDim.x / 8 (i = 0, 1, ...; with a grid that
// covers the whole sequence every workgroup has one tile, with a smaller one the workgroups are
// persistent and walk the sequence).  Returns false past the end of the sequence.
template <bool SPLIT>
__device__ __forceinline__ bool assign_tile(int slot, int tiles_m, int tiles_n, int per_xcd, int xcd_rows, int splits,
                                            int &tile_row, int &tile_col, int &split)
{
    const int xcd = blockIdx.x & 7;
    constexpr int GROUP = 4;
    split = 0;
    if (!SPLIT && xcd_rows > 0) {
        const int xcd_cols = 8 / xcd_rows;
        const int xr = xcd % xcd_rows, xc = xcd / xcd_rows;
        const int row_lo = tiles_m * xr / xcd_rows, row_hi = tiles_m * (xr + 1) / xcd_rows;
        const int col_lo = tiles_n * xc / xcd_cols, col_hi = tiles_n * (xc + 1) / xcd_cols;
        const int rm = row_hi - row_lo, cn = col_hi - col_lo;
        if (slot >= rm * cn) return false;
        const int g_idx = slot / (GROUP * cn), in_group = slot - g_idx * GROUP * cn;
        const int first_row = g_idx * GROUP;
        const int rows_here = (rm - first_row) < GROUP ? (rm - first_row) : GROUP;
        tile_row = row_lo + first_row + in_group % rows_here;
        tile_col = col_lo + in_group / rows_here;
    } else {
        const int64_t tiles_total = (int64_t)tiles_m * tiles_n;
        int64_t lin = (int64_t)xcd * per_xcd + slot;
        if (slot >= per_xcd || lin >= tiles_total * (SPLIT ? splits : 1)) return false;
        // split-K: the workgroups of one K range are neighbours (they share the A rows / B columns
        // of that range in their XCD's L2)
        split = SPLIT ? (int)(lin / tiles_total) : 0;
        lin -= split * tiles_total;
        const int64_t group_span = (int64_t)GROUP * tiles_n;
        const int first_row = (int)(lin / group_span) * GROUP;
        const int rows_here = (tiles_m - first_row) < GROUP ? (tiles_m - first_row) : GROUP;
        const int in_group = (int)(lin % group_span);
        tile_row = first_row + in_group % rows_here;
        tile_col = in_group / rows_here;
    }
    return true;
}

// 4-bit weights (B4): the packed nibbles travel to LDS as they are -- a K-step of a B row is 32
// bytes, two 16-byte chunks (one per 32-deep sub-step), a wave-level load covers 32 rows -- and
// are expanded to int8 (times 16, see expand_int4) in registers after the fragment read.  Chunk c
// of row r sits at position c ^ ((r / 8) % 2), which makes the 8-byte fragment reads of 32
// consecutive rows conflict-free.  Waves without a B segment of their own (narrow tiles) fetch
// the constant chunk into the unused half of the B area, so that every wave issues the same
// number of loads per K-step.
__device__ __forceinline__ i32x4 expand_int4(u32x2 raw)
{
    // byte j of raw holds element 2j in its low and element 2j+1 in its high nibble; each element
    // becomes one byte holding 16 times its value (the nibble in the high half of the byte)
    i32x4 w;
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        const uint32_t even = (raw[d] << 4) & 0xF0F0F0F0u, odd = raw[d] & 0xF0F0F0F0u;
        w[2 * d] = (int32_t)__builtin_amdgcn_perm(odd, even, 0x05010400u);
        w[2 * d + 1] = (int32_t)__builtin_amdgcn_perm(odd, even, 0x07030602u);
    }
    return w;
}

template <int BM, int BN, int WM, int WN, int A_MODE, int NSTAGE, bool SPLIT = false, bool ZW = false, bool B4 = false,
          int MINW = 1>
__global__ void __launch_bounds__(WM *WN * 64, MINW)
    igemm_dma_kernel(const IgemmArgs g, const int tiles_m, const int tiles_n, const int per_xcd, const int xcd_rows,
                     const SplitK sk, const int tune)
{
    constexpr int NW = WM * WN, BK = 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int B_SEG_ROWS = B4 ? 32 : 16;                // B rows per wave-level load (1 KB)
    constexpr int B_SEGS = BN / B_SEG_ROWS;                 // wave-level loads per stage that carry B rows
    constexpr int A_LOADS = BM / 16 / NW, B_LOADS = (B_SEGS + NW - 1) / NW; // wave-level loads per stage and wave
    static_assert(BM % (16 * NW) == 0 && (B4 || BN % (16 * NW) == 0), "whole 16-row segments per wave");
    static_assert(!B4 || !SPLIT, "4-bit weights run unsplit");
    constexpr int STAGE_BYTES = (BM + BN) * BK;
    constexpr int LOADS = A_LOADS + B_LOADS;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // wave-uniform: keeps LDS bases in SGPRs
    const int wave_m = wave / WN, wave_n = wave % WN;
    // Workgroups walk their XCD's tile sequence with stride gridDim.x / 8: one tile each when the grid
    // covers the sequence, several when the launch is persistent (fewer workgroups than tiles).
    const int slot_stride = gridDim.x >> 3;
    for (int slot = blockIdx.x >> 3, tile_iter = 0;; slot += slot_stride, ++tile_iter) {
        int tile_row, tile_col, split;
        if (!assign_tile<SPLIT>(slot, tiles_m, tiles_n, per_xcd, xcd_rows, sk.splits, tile_row, tile_col, split)) break;
        const int64_t m0 = (int64_t)tile_row * BM;
        const int n0 = tile_col * BN;


        // ---- per-lane source description of the chunks this lane fetches at every K-step
        // A_MATRIX and B: a wave-uniform base pointer plus a 32-bit per-lane offset that does not
        // change from K-step to K-step (the K advance goes into the uniform part).
        const uint8_t *a_src[A_LOADS], *a_pix[A_LOADS];
        int a_koff[A_LOADS], a_hi0[A_LOADS], a_wi0[A_LOADS];
        uint32_t a_lane_off[A_LOADS], b_lane_off[B_LOADS];
        const uint8_t *const a_tile = g.A + m0 * g.lda;                 // A_MATRIX only
        const uint8_t *const b_tile = g.B + (B4 ? ((int64_t)n0 * g.ldb) >> 1 : (int64_t)n0 * g.ldb);
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) {
            const int row = (wave * A_LOADS + j) * 16 + (lane >> 2);
            a_koff[j] = (((lane & 3) ^ lds_swizzle(row)) & 3) * 16;
            int64_t m = m0 + row;
            m = m < g.M ? m : g.M - 1;
            a_hi0[j] = a_wi0[j] = 0;
            a_lane_off[j] = 0;
            a_src[j] = a_pix[j] = nullptr;
            if constexpr (A_MODE == A_MATRIX) {
                a_lane_off[j] = (uint32_t)((m - m0) * g.lda) + (uint32_t)a_koff[j];
            } else {
                const int64_t img = m / ((int64_t)g.Ho * g.Wo);
                const int rem = (int)(m - img * ((int64_t)g.Ho * g.Wo));
                const int ho = rem / g.Wo, wo = rem - ho * g.Wo;
                a_src[j] = g.A + img * ((int64_t)g.H * g.W * g.Cin);
                a_hi0[j] = ho * g.sh - g.ph;
                a_wi0[j] = wo * g.sw - g.pw;
                // address of tap (0,0), channel koff of this row's window (may lie outside the image:
                // only dereferenced after the bounds check)
                a_pix[j] = a_src[j] + ((int64_t)a_hi0[j] * g.W + a_wi0[j]) * g.Cin + a_koff[j];
            }
        }
#pragma unroll
        for (int j = 0; j < B_LOADS; ++j) {
            if constexpr (B4) {
                const int row = (wave * B_LOADS + j) * 32 + (lane >> 1);
                const int b_koff = ((lane & 1) ^ ((row >> 3) & 1)) * 16; // bytes: 32 packed elements per chunk
                int n = n0 + row;
                n = n < g.N ? n : g.N - 1;
                b_lane_off[j] = (uint32_t)(((int64_t)(n - n0) * g.ldb) >> 1) + (uint32_t)b_koff;
            } else {
                const int row = (wave * B_LOADS + j) * 16 + (lane >> 2);
                const int b_koff = (((lane & 3) ^ lds_swizzle(row)) & 3) * 16;
                int n = n0 + row;
                n = n < g.N ? n : g.N - 1;
                b_lane_off[j] = (uint32_t)((int64_t)(n - n0) * g.ldb) + (uint32_t)b_koff;
            }
        }
        const uint8_t *fill_a = &g_fill_table.v[g.z_a][0];
        ChannelParams<TN> cparams = {};
        if constexpr (!SPLIT) cparams = load_channel_params<BN, WN, TN>(g, n0);
        // K-steps [kt_first, kt_first + ktiles) of the product; the dispatcher guarantees K % 64 == 0
        const int kt_first = SPLIT ? split * sk.ksteps : 0;
        const int ktiles = SPLIT ? ((g.K / BK - kt_first) < sk.ksteps ? (g.K / BK - kt_first) : sk.ksteps) : g.K / BK;
        const bool tap_uniform = A_MODE == A_CONV && (g.Cin % BK) == 0;

        // load number `idx` (0 .. LOADS-1) of K-step kt: A segments first, then B segments.
        // K-steps past the end fetch one constant 16-byte chunk instead (into a buffer nobody reads
        // any more): no extra memory traffic, and the number of loads per K-step stays uniform,
        // which the vmcnt-based waits rely on.
        auto issue_load = [&](int kt, int idx) {
            uint8_t *stage = smem + (kt % NSTAGE) * STAGE_BYTES;
            const bool live = kt < ktiles; // wave-uniform
            const int k0 = (kt_first + kt) * BK;
            if (idx < A_LOADS) {
                const int j = idx;
                const uint8_t *src = fill_a;
                if constexpr (A_MODE == A_MATRIX) {
                    if (live) src = (a_tile + k0) + a_lane_off[j]; // K % 64 == 0: no tail
                } else {
                    const int k = k0 + a_koff[j];
                    if (live && tap_uniform) {
                        // Cin % 64 == 0: the whole K-step lies inside one tap, so the tap decomposition
                        // is wave-uniform (scalar unit) and only the bounds check is per lane
                        const uint32_t tap = fast_div((uint32_t)k0, (uint32_t)g.Cin, g.magic_cin);
                        const int ci0 = k0 - (int)tap * g.Cin;
                        const uint32_t ta = fast_div(tap, (uint32_t)g.kw, g.magic_kw);
                        const int tb = (int)tap - (int)ta * g.kw;
                        const int64_t delta = ((int64_t)ta * g.W + tb) * g.Cin + ci0;
                        const int hi = a_hi0[j] + (int)ta, wi = a_wi0[j] + tb;
                        if ((unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W) src = a_pix[j] + delta;
                    } else if (live) {
                        const uint32_t tap = fast_div((uint32_t)k, (uint32_t)g.Cin, g.magic_cin);
                        const int ci = k - (int)tap * g.Cin;
                        const uint32_t ta = fast_div(tap, (uint32_t)g.kw, g.magic_kw);
                        const int tb = (int)tap - (int)ta * g.kw;
                        const int hi = a_hi0[j] + (int)ta, wi = a_wi0[j] + tb;
                        if (hi >= 0 && hi < g.H && wi >= 0 && wi < g.W) src = a_src[j] + ((int64_t)hi * g.W + wi) * g.Cin + ci;
                    }
                }
                dma16(src, stage + (wave * A_LOADS + j) * 1024);
            } else {
                const int j = idx - A_LOADS;
                if constexpr (B4) {
                    const int seg = wave * B_LOADS + j; // wave-uniform
                    const bool mine = seg < B_SEGS;
                    const uint8_t *src = (live && mine) ? (b_tile + (k0 >> 1)) + b_lane_off[j] : fill_a;
                    // segments beyond the tile: into the unused second half of the B area
                    dma16(src, stage + BM * BK + (mine ? seg * 1024 : BN * 32));
                } else {
                    const uint8_t *src = live ? (b_tile + k0) + b_lane_off[j] : fill_a;
                    dma16(src, stage + BM * BK + (wave * B_LOADS + j) * 1024);
                }
            }
        };
        auto issue_stage = [&](int kt) {
#pragma unroll
            for (int idx = 0; idx < LOADS; ++idx) issue_load(kt, idx);
        };

        i32x16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
        int32_t colsum[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) colsum[j] = 0;

        const int frag_row = lane & 31, frag_half = lane >> 5;
        int a_off[TM][2], b_off[TN][2]; // LDS byte offsets of this lane's fragments within a stage
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int i = 0; i < TM; ++i) a_off[i][ks] = lds_chunk_offset(wave_m * WTM + i * 32 + frag_row, ks * 2 + frag_half);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = wave_n * WTN + j * 32 + frag_row;
                b_off[j][ks] = BM * BK + (B4 ? row * 32 + ((ks ^ ((row >> 3) & 1)) << 4) + frag_half * 8
                                             : lds_chunk_offset(row, ks * 2 + frag_half));
            }
        }
        // One "piece" p of a fragment set: pieces 0..TM-1 are the A fragments, TM..TM+TN-1 the B fragments
        auto read_piece = [&](const uint8_t *stage, int ks, int p, i32x4 (&fa)[TM], i32x4 (&fb)[TN]) {
            if (p < TM) fa[p] = *reinterpret_cast<const i32x4 *>(stage + a_off[p][ks]);
            else if constexpr (B4) fb[p - TM] = expand_int4(*reinterpret_cast<const u32x2 *>(stage + b_off[p - TM][ks]));
            else fb[p - TM] = *reinterpret_cast<const i32x4 *>(stage + b_off[p - TM][ks]);
        };
        // weight column sums (only needed when z_a != 128): wave row wave_m covers the K sub-steps
        // ks with ks % WM == wave_m; the partial sums are combined in the epilogue
        const bool need_colsum = g.z_a != 128;
        auto add_colsum = [&](i32x4 (&fb)[TN]) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int d = 0; d < 4; ++d) colsum[j] = __builtin_amdgcn_sdot4(fb[j][d], 0x01010101, colsum[j], false);
        };
        constexpr int PIECES = TM + TN, MMAS = TM * TN;
        // MFMAs of one K sub-step with the LDS reads of the next fragment set (and optionally the
        // DMA loads of a later stage) spread evenly between them, so that neither the LDS nor
        // the texture-address queue sees a burst that would stall MFMA issue
        auto mma_interleaved = [&](i32x4 (&fa)[TM], i32x4 (&fb)[TN], const uint8_t *next_stage, int next_ks,
                                   i32x4 (&na)[TM], i32x4 (&nb)[TN], bool do_read, int dma_kt) {
            i32x4 xs[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i) xs[i] = fa[i] ^ (int32_t)0x80808080; // uint8 code -> signed (code - 128)
            int piece = 0, load = 0;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xs[i], fb[j], acc[i][j], 0, 0, 0);
                    const int done = i * TN + j + 1;
                    // after every MMAS/PIECES MFMAs issue one fragment read (and one DMA load)
                    while (do_read && piece < PIECES && done * PIECES >= (piece + 1) * MMAS) {
                        read_piece(next_stage, next_ks, piece, na, nb);
                        ++piece;
                    }
                    while (dma_kt >= 0 && load < LOADS && done * LOADS >= (load + 1) * MMAS) {
                        issue_load(dma_kt, load);
                        ++load;
                    }
                }
        };

        // ---- prologue: NSTAGE-1 stages in flight
#pragma unroll
        for (int s = 0; s < NSTAGE - 1; ++s) issue_stage(s);
        // stage 0 has landed when at most the later stages' loads are outstanding
        wait_vmcnt<(NSTAGE - 2) * LOADS>();
        block_barrier();

        i32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
#pragma unroll
        for (int p = 0; p < PIECES; ++p) read_piece(smem, 0, p, fa0, fb0);
        // Issue priority of the main loop (the epilogue always runs at the default, lowest one).
        // tune bit 0: the second half of the workgroup's waves -- the ones that share a SIMD with a
        //   wave of the first half -- stay low, so that inside a K-step one wave of a SIMD runs its
        //   MFMAs while the other one reads its fragments, instead of both doing the same thing;
        // tune bit 1: persistent launches with two workgroups per CU: the workgroups that were
        //   dispatched second stay low during their first tile only, which puts the two workgroups of
        //   a CU half a tile apart, so that one's epilogue runs under the other's MFMAs.
        const bool low_prio = ((tune & 1) && wave >= NW / 2) || ((tune & 2) && tile_iter == 0 && ((blockIdx.x >> 8) & 1));
        if (!low_prio) __builtin_amdgcn_s_setprio(1);
        for (int kt = 0; kt < ktiles; ++kt) {
            const uint8_t *stage = smem + (kt % NSTAGE) * STAGE_BYTES;
            // sub-step 0: MFMAs on (fa0, fb0) while (fa1, fb1) are read from the same stage
            if (need_colsum && (0 % WM) == wave_m) add_colsum(fb0);
            mma_interleaved(fa0, fb0, stage, 1, fa1, fb1, true, -1);
#pragma unroll
            for (int q = 0; q < PIECES; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, MMAS / PIECES, 0); // MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);             // DS read
            }
            // stage kt+1 must have landed: only the NSTAGE-3 stages issued after it may be in flight
            // (every K-step issues exactly LOADS loads, real or fill, so the count is uniform)
            static_assert(NSTAGE >= 3, "the refilled buffer must not be the one still being read");
            wait_vmcnt<(NSTAGE - 3) * LOADS>();
            block_barrier(); // also: every wave is done reading stage kt-1, whose buffer is refilled next
            // sub-step 1: MFMAs on (fa1, fb1) while the first fragments of stage kt+1 are read and the
            // loads of stage kt+NSTAGE-1 are issued (past the last stage: stale data, never used)
            if (need_colsum && (1 % WM) == wave_m) add_colsum(fb1);
            mma_interleaved(fa1, fb1, smem + ((kt + 1) % NSTAGE) * STAGE_BYTES, 0, fa0, fb0, true, kt + NSTAGE - 1);
            if constexpr (LOADS == PIECES) {
#pragma unroll
                for (int q = 0; q < PIECES; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, MMAS / PIECES, 0); // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);             // DS read
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);             // VMEM read (LDS DMA)
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
        wait_vmcnt<0>(); // drain the fill loads of the last K-steps before the tile memory is reused
        block_barrier(); // all fragment reads done before the tile memory is reused for the output
        if constexpr (WM > 1) {
            if (need_colsum) { // every wave row holds the sums of its own K sub-steps only
                int32_t *part = reinterpret_cast<int32_t *>(smem) + BM * (BN + 16) / 4; // past the output tile
#pragma unroll
                for (int j = 0; j < TN; ++j) part[(wave * TN + j) * 64 + lane] = colsum[j];
                __syncthreads();
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    int32_t t = 0;
#pragma unroll
                    for (int wm = 0; wm < WM; ++wm) t += part[((wm * WN + wave_n) * TN + j) * 64 + lane];
                    colsum[j] = t;
                }
            }
        }
        if constexpr (SPLIT) {
            // partial sums straight from the accumulator layout: per register, 32 lanes write 32
            // consecutive int32 of one row (128-byte runs)
            int32_t *plane = sk.partial + (int64_t)split * g.M * g.N;
#pragma clang loop unroll(full)
            for (int j = 0; j < TN; ++j) {
                const int32_t corr = (128 - g.z_a) * (colsum[j] + __shfl_xor(colsum[j], 32));
                const int col = n0 + wave_n * WTN + j * 32 + frag_row;
#pragma clang loop unroll(full)
                for (int i = 0; i < TM; ++i)
#pragma clang loop unroll(full)
                    for (int r = 0; r < 16; ++r) {
                        const int64_t row = m0 + wave_m * WTM + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
                        if (row < g.M && col < g.N) plane[row * g.N + col] = acc[i][j][r] + corr;
                    }
            }
        } else {
            igemm_epilogue<BM, BN, WM, WN, B4, ZW>(g, acc, colsum, cparams, smem, m0, n0);
        }
        // every wave has left the output tile before the next tile's loads overwrite it
        block_barrier();
    }
}

// Second pass of split-K: out[m][n] = clamp(z_out + RESCALE(sum_s partial[s][m][n] + bias[n])).
// One thread per 4 consecutive columns of one row.
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const IgemmArgs g, const SplitK sk)
{
    const int64_t groups = ((int64_t)g.N + 3) / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= g.M * groups) return;
    const int64_t m = idx / groups;
    const int n = (int)(idx - m * groups) * 4;
    const int64_t plane = g.M * g.N;
    const int32_t *p = sk.partial + m * g.N + n;
    int32_t a[4] = {0, 0, 0, 0};
    if ((g.N & 3) == 0) { // whole, 16-byte aligned groups
        for (int s = 0; s < sk.splits; ++s) {
            const i32x4 v = __builtin_nontemporal_load(reinterpret_cast<const i32x4 *>(p + s * plane));
            a[0] += v.x, a[1] += v.y, a[2] += v.z, a[3] += v.w;
        }
    } else {
        for (int s = 0; s < sk.splits; ++s)
            for (int e = 0; e < 4 && n + e < g.N; ++e) a[e] += p[s * plane + e];
    }
    const int32_t act_lo = g.lo_rel + g.z_out, act_hi = g.hi_rel + g.z_out;
    uint32_t packed = 0;
    int valid = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (n + e >= g.N) break;
        const int32_t b = g.bias ? g.bias[n + e] : 0, mu = g.mult[n + e], sf = g.shift[n + e];
        int32_t y;
        if (g.small_acc >= 2 && sf >= 1 && sf <= 20 && b > -(1 << 27) && b < (1 << 27)) {
            y = rescale_fused(a[e], make_fused(mu, sf, b, g.z_out, act_lo, act_hi));
        } else {
            y = clamp_i32(g.lo_rel, g.hi_rel, rescale_general(a[e] + b, make_rescale(mu, sf))) + g.z_out;
        }
        packed |= (uint32_t)y << (8 * e);
        ++valid;
    }
    uint8_t *dst = g.C + m * g.ldc + n;
    if (valid == 4 && (reinterpret_cast<uintptr_t>(dst) & 3) == 0) {
        *reinterpret_cast<uint32_t *>(dst) = packed;
    } else {
        for (int e = 0; e < valid; ++e) dst[e] = (uint8_t)(packed >> (8 * e));
    }
}

} // namespace qnn
