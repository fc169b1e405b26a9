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
// Requirements (checked by the dispatcher): every 16-byte chunk is 16-byte aligned
// (K, pitches and base pointers multiples of 16; for convolutions Cin % 16 == 0).
// Rows beyond M / columns beyond N are clamped to the last valid one (their results are
// never stored); chunks beyond K read a constant chunk: zero for the weights, the code z_x
// for out-of-image taps of the activations.
#pragma once

#include "igemm.h"

namespace qnn {

// 256 constant 16-byte chunks: entry v is the byte v repeated (fill codes for padding taps)
struct FillTable {
    uint8_t v[256][16];
    constexpr FillTable() : v{}
    {
        for (int i = 0; i < 256; ++i)
            for (int j = 0; j < 16; ++j) v[i][j] = (uint8_t)i;
    }
};
__device__ const FillTable g_fill_table{};

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

template <int BM, int BN, int WM, int WN, int A_MODE, int NSTAGE>
__global__ void __launch_bounds__(WM *WN * 64) igemm_dma_kernel(const IgemmArgs g, const int tiles_m, const int tiles_n,
                                                                const int per_xcd)
{
    constexpr int NW = WM * WN, NT = NW * 64, BK = 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int A_LOADS = BM / 16 / NW, B_LOADS = BN / 16 / NW; // wave-level loads per stage
    static_assert(BM % (16 * NW) == 0 && BN % (16 * NW) == 0, "whole 16-row segments per wave");
    constexpr int STAGE_BYTES = (BM + BN) * BK;
    constexpr int LOADS = A_LOADS + B_LOADS;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- tile assignment: consecutive workgroup ids go round-robin over the 8 XCDs, each
    // with its own L2; give every XCD one contiguous band of the tile sequence, and walk the
    // band in groups of 4 tile rows so that concurrently running tiles share A rows / B columns.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int64_t lin = (int64_t)xcd * per_xcd + slot;
    if (slot >= per_xcd || lin >= (int64_t)tiles_m * tiles_n) return;
    constexpr int GROUP = 4;
    const int64_t group_span = (int64_t)GROUP * tiles_n;
    const int first_row = (int)(lin / group_span) * GROUP;
    const int rows_here = (tiles_m - first_row) < GROUP ? (tiles_m - first_row) : GROUP;
    const int in_group = (int)(lin % group_span);
    const int64_t m0 = (int64_t)(first_row + in_group % rows_here) * BM;
    const int n0 = (in_group / rows_here) * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / WN, wave_n = wave % WN;

    // ---- per-lane source description of the chunks this lane fetches at every K-step
    const uint8_t *a_src[A_LOADS];
    int a_koff[A_LOADS], a_hi0[A_LOADS], a_wi0[A_LOADS];
    const uint8_t *b_src[B_LOADS];
    int b_koff[B_LOADS];
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
        const int row = (wave * A_LOADS + j) * 16 + (lane >> 2);
        a_koff[j] = (((lane & 3) ^ (row >> 1) ^ (row >> 3)) & 3) * 16;
        int64_t m = m0 + row;
        m = m < g.M ? m : g.M - 1;
        a_hi0[j] = a_wi0[j] = 0;
        if constexpr (A_MODE == A_MATRIX) {
            a_src[j] = g.A + m * g.lda;
        } else {
            const int64_t img = m / ((int64_t)g.Ho * g.Wo);
            const int rem = (int)(m - img * ((int64_t)g.Ho * g.Wo));
            const int ho = rem / g.Wo, wo = rem - ho * g.Wo;
            a_src[j] = g.A + img * ((int64_t)g.H * g.W * g.Cin);
            a_hi0[j] = ho * g.sh - g.ph;
            a_wi0[j] = wo * g.sw - g.pw;
        }
    }
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) {
        const int row = (wave * B_LOADS + j) * 16 + (lane >> 2);
        b_koff[j] = (((lane & 3) ^ (row >> 1) ^ (row >> 3)) & 3) * 16;
        int n = n0 + row;
        n = n < g.N ? n : g.N - 1;
        b_src[j] = g.B + (int64_t)n * g.ldb;
    }
    const uint8_t *fill_a = &g_fill_table.v[g.z_a][0];
    const uint8_t *fill_b = &g_fill_table.v[0][0];

    auto issue_stage = [&](int kt) {
        uint8_t *stage = smem + (kt % NSTAGE) * STAGE_BYTES;
        const int k0 = kt * BK;
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) {
            const int k = k0 + a_koff[j];
            const uint8_t *src = fill_a;
            if (k < g.K) {
                if constexpr (A_MODE == A_MATRIX) {
                    src = a_src[j] + k;
                } else {
                    const uint32_t tap = fast_div((uint32_t)k, (uint32_t)g.Cin, g.magic_cin);
                    const int ci = k - (int)tap * g.Cin;
                    const uint32_t ta = fast_div(tap, (uint32_t)g.kw, g.magic_kw);
                    const int tb = (int)tap - (int)ta * g.kw;
                    const int hi = a_hi0[j] + (int)ta, wi = a_wi0[j] + tb;
                    if (hi >= 0 && hi < g.H && wi >= 0 && wi < g.W) src = a_src[j] + ((int64_t)hi * g.W + wi) * g.Cin + ci;
                }
            }
            dma16(src, stage + (wave * A_LOADS + j) * 1024);
        }
#pragma unroll
        for (int j = 0; j < B_LOADS; ++j) {
            const int k = k0 + b_koff[j];
            const uint8_t *src = k < g.K ? b_src[j] + k : fill_b;
            dma16(src, stage + BM * BK + (wave * B_LOADS + j) * 1024);
        }
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

    const int ktiles = (g.K + BK - 1) / BK;
    const int frag_row = lane & 31, frag_half = lane >> 5;
    int a_off[TM][2], b_off[TN][2]; // LDS byte offsets of this lane's fragments within a stage
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i) a_off[i][ks] = lds_chunk_offset(wave_m * WTM + i * 32 + frag_row, ks * 2 + frag_half);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            b_off[j][ks] = BM * BK + lds_chunk_offset(wave_n * WTN + j * 32 + frag_row, ks * 2 + frag_half);
    }
    auto read_frags = [&](const uint8_t *stage, int ks, i32x4 (&fa)[TM], i32x4 (&fb)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const i32x4 *>(stage + a_off[i][ks]);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const i32x4 *>(stage + b_off[j][ks]);
    };
    auto mma = [&](i32x4 (&fa)[TM], i32x4 (&fb)[TN]) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int d = 0; d < 4; ++d) colsum[j] = __builtin_amdgcn_sdot4(fb[j][d], 0x01010101, colsum[j], false);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const i32x4 xs = fa[i] ^ (int32_t)0x80808080; // uint8 code -> signed (code - 128)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xs, fb[j], acc[i][j], 0, 0, 0);
        }
    };

    // ---- prologue: NSTAGE-1 stages in flight
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
        if (s < ktiles) issue_stage(s);
    // stage 0 has landed when at most the later stages' loads are outstanding
    if (ktiles >= NSTAGE - 1) wait_vmcnt<(NSTAGE - 2) * LOADS>();
    else wait_vmcnt<0>();
    block_barrier();

    i32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    read_frags(smem, 0, fa0, fb0);
    for (int kt = 0; kt < ktiles; ++kt) {
        const uint8_t *stage = smem + (kt % NSTAGE) * STAGE_BYTES;
        read_frags(stage, 1, fa1, fb1);
        mma(fa0, fb0);
        if (kt + 1 < ktiles) {
            // stage kt+1 must have landed: only stage kt+2 .. may still be in flight
            if (kt + NSTAGE - 1 <= ktiles) wait_vmcnt<(NSTAGE - 3) * LOADS>();
            else wait_vmcnt<0>();
            block_barrier(); // also: every wave is done reading stage kt-1, whose buffer is refilled next
            if (kt + NSTAGE - 1 < ktiles) issue_stage(kt + NSTAGE - 1);
            read_frags(smem + ((kt + 1) % NSTAGE) * STAGE_BYTES, 0, fa0, fb0);
        }
        mma(fa1, fb1);
    }
    block_barrier(); // all fragment reads done before the tile memory is reused for the output
    igemm_epilogue<BM, BN, WM, WN, false>(g, acc, colsum, smem, m0, n0);
}

} // namespace qnn
