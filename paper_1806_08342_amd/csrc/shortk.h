// Dense quantized layer with a short reduction (K <= 256): 1x1 convolutions and GEMMs whose
// cost is the epilogue and the memory streams, not the MFMAs.
//
// Weight-stationary and barrier-free: a wave owns up to 32*NB output columns, loads their weights
// ONCE into registers as MFMA B fragments (4-bit weights are unpacked there, kept times 16),
// derives the per-column epilogue constants once (column sums for the zero-point correction,
// bias, fixed-point multiplier and shift), and then walks over blocks of 32 rows: the A fragments
// of a block come straight from global memory (each lane fetches the 16 bytes its MFMA operand
// needs; the next block's are requested as soon as the current block's MFMAs are issued), NB*KS MFMAs,
// epilogue, and the 32 x 32*NB byte tile goes through a wave-private LDS area to become 16-byte
// row stores.  Waves never synchronise with each other; a workgroup is just four such waves on
// neighbouring column groups of the same rows (they share the A rows through the vector cache).
// Arithmetic as in igemm.h (eq. 4-6 with z_w = 0, bias, RESCALE, clamp).
#pragma once

#include <type_traits>

#include "igemm.h"

namespace qnn {

struct ShortKArgs {
    IgemmArgs g;       // A_MATRIX fields, or the geometry of a strided 1x1 convolution
    int col_groups;    // ceil(N / (32 * NB))
    int walkers;       // waves that share one column group (they interleave over the row blocks)
    int strided;       // rows of A are pixels (n, ho*sh, wo*sw) of an NHWC image (1x1 convolution, stride > 1)
};

// 16 consecutive k of one row / column as 4 dwords, zero beyond K.  VEC = bytes per load.
template <int VEC> __device__ __forceinline__ i32x4 shortk_load16(const uint8_t *p, int k, int K)
{
    i32x4 v = {0, 0, 0, 0};
    if constexpr (VEC == 16) {
        if (k + 16 <= K) v = *reinterpret_cast<const i32x4 *>(p + k);
    } else if constexpr (VEC == 8) {
        if (k + 8 <= K) {
            const u32x2 a = *reinterpret_cast<const u32x2 *>(p + k);
            v[0] = (int32_t)a.x, v[1] = (int32_t)a.y;
        }
        if (k + 16 <= K) {
            const u32x2 b = *reinterpret_cast<const u32x2 *>(p + k + 8);
            v[2] = (int32_t)b.x, v[3] = (int32_t)b.y;
        }
    } else {
#pragma unroll
        for (int d = 0; d < 4; ++d)
            if (k + 4 * d + 4 <= K) v[d] = *reinterpret_cast<const int32_t *>(p + k + 4 * d);
    }
    return v;
}

// Epilogue constants of one column in the cheapest exact form (valid for 1 <= shift <= 20 and
// |acc + corr| < 2^29).  With a = acc + corr, n = shift:
//   T = hi32(4a * mult),  s = T >> 31,  w = T + 2s + c,  c = 2*(2^(n-1) + (z_out << n)) + 1
//   out = clamp(w, act_min << (n+1), ((act_max + 1) << (n+1)) - 1) >> (n + 1)
// which equals clamp(z_out + RESCALE(a)) bit for bit: the rounding-doubling high multiply
// (ties up) and the rounding shift (ties away from zero) collapse into one floor division, and
// clamping before the final shift lets that shift write its byte straight into the packed dword.
struct ShortKColumn {
    int32_t mult, corr, c, n1, lo, hi, shift;
};

// ADD: the rescaling add with a residual tensor (g.R) is applied to the output tile on its way
// from LDS to global memory; the residual chunks of a row block are requested one round ahead.
// The add is a function of two 8-bit codes, so the workgroup (8 waves here, to share it) first
// tabulates all 65536 results in LDS; combining a pair of codes is then one byte gather.
// ALDS (K = 128 or 256, plain matrices, 16-byte aligned rows): the A rows of a row block are shared by the waves
// of a workgroup, which then own neighbouring column groups of the SAME rows.  The block's 32 x K bytes are
// copied once per workgroup straight into LDS (global_load_lds_dwordx4, whole 128-byte lines per 8 lanes, next
// block's copy in flight during the current block) and every wave reads its fragments from there.  Fetching the
// fragments from global memory costs one vector-cache access per lane and instruction (every lane is on a row
// of its own): counters showed the address unit busy for 58 % and the vector cache for 70-80 % of that kernel's
// time, on a par with the vector ALU.  LDS positions are XOR-swizzled on the global-address side, so that the
// 16 lanes that share a cycle of a 16-byte LDS read hit 16 different bank groups.
template <int NB, int KS, bool INT4, int VEC, int BVEC, int ADD = 0, bool ALDS = false> // ADD: 0 none, 1 two 256-entry tables, 2 pair table
__global__ void __launch_bounds__(ADD == 2 ? 512 : 256, ADD == 2 ? 1 : (KS <= 1 ? 3 : 2)) shortk_kernel(const ShortKArgs s)
{
    constexpr int PITCH = 32 * NB + 32; // bytes per staged output row: the 8 rows a store instruction touches fall in distinct banks
    constexpr int WAVES = ADD == 2 ? 8 : 4; // the pair table is shared by 8 waves (one workgroup per CU)
    constexpr int KBYTES = KS * 32, CPR = KBYTES / 16; // ALDS: bytes and 16-byte chunks of an A row (K == KS * 32)
    constexpr int ATILE = 32 * KBYTES;
    static_assert(!ALDS || (KS == 4 || KS == 8), "the staged form exists for K = 128 and K = 256");
    __shared__ __attribute__((aligned(16))) uint8_t a_tiles[ALDS ? 2 * ATILE : 16];
    __shared__ __attribute__((aligned(16))) uint8_t stage_static[ADD ? 16 : 4 * 32 * PITCH];
    extern __shared__ __attribute__((aligned(16))) uint8_t dyn_lds[]; // ADD: [table(s)][output tiles of the waves]
    uint8_t *const pair_tab = dyn_lds;
    constexpr int TAB_BYTES = ADD == 2 ? 65536 : 2048; // pair table, or the two 256-entry tables
    uint8_t *const stage_all = ADD ? dyn_lds + TAB_BYTES : stage_static;
    const IgemmArgs &g = s.g;
    // small layers skip the pair table (building it would cost more than it saves) and combine through
    // the two 256-entry tables of rescaled codes instead
    constexpr bool use_pairs = ADD == 2;
    int32_t *const tab = reinterpret_cast<int32_t *>(use_pairs ? stage_all : pair_tab); // pairs: in the tile area for now
    if constexpr (ADD) { // the only workgroup barriers, before any wave may leave
        add_fill_tables(tab, g.add, threadIdx.x, WAVES * 64);
        __syncthreads();
        if constexpr (use_pairs) {
            const AddOut ao = make_add_out(g.add);
            // entry [m][r] = code of the sum; a lane fills 4 consecutive r of one m per step
            for (int q = threadIdx.x; q < 65536 / 4; q += 512) {
                const uint32_t m = (uint32_t)q >> 6, r0 = ((uint32_t)q & 63u) * 4u;
                const uint32_t mm = m * 0x01010101u, rr = (r0 * 0x01010101u) + 0x03020100u;
                reinterpret_cast<uint32_t *>(pair_tab)[q] =
                    ao.fused ? add_codes4<true>(mm, rr, tab, ao) : add_codes4<false>(mm, rr, tab, ao);
            }
            __syncthreads();
        }
    }
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform: row-block arithmetic stays scalar
    uint8_t *stage = stage_all + wave * (32 * PITCH);
    const int frow = lane & 31, fhalf = lane >> 5;

    // wave -> (column group, walker): neighbouring waves take neighbouring column groups of the same rows
    int cg, walker;
    bool active = true; // ALDS: a wave beyond the last column group only helps with the copies and the barriers
    if constexpr (ALDS) {
        const int groups = (s.col_groups + WAVES - 1) / WAVES; // workgroups side by side; the grid is groups x walkers
        cg = (int)(blockIdx.x % groups) * WAVES + wave;
        walker = (int)(blockIdx.x / groups);
        active = cg < s.col_groups;
        cg = active ? cg : s.col_groups - 1;
    } else {
        const int64_t gw = (int64_t)blockIdx.x * WAVES + wave;
        cg = (int)(gw % s.col_groups), walker = (int)(gw / s.col_groups);
        if (walker >= s.walkers) return; // no barriers below: a wave may leave alone
    }
    const int n0 = cg * 32 * NB;
    const int blocks_here = (g.N - n0 + 31) / 32 < NB ? (g.N - n0 + 31) / 32 : NB; // column blocks that exist

    // ---- weights: B fragments of all K sub-steps, for good
    i32x4 fb[KS][NB];
    ShortKColumn col[NB];
    bool fused_ok = g.small_acc >= 2;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        int n = n0 + j * 32 + frow;
        const bool real = n < g.N;
        n = real ? n : g.N - 1;
        int32_t colsum = 0;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int k = ks * 32 + fhalf * 16;
            if constexpr (INT4) {
                const uint8_t *p = g.B + (((int64_t)n * g.ldb) >> 1);
                uint32_t r2[2] = {0u, 0u};
                if (k + 8 <= g.K) r2[0] = *reinterpret_cast<const uint32_t *>(p + (k >> 1));
                if (k + 16 <= g.K) r2[1] = *reinterpret_cast<const uint32_t *>(p + (k >> 1) + 4);
#pragma unroll
                for (int d = 0; d < 2; ++d) { // r2[d] holds elements 8d .. 8d+7, two per byte, low nibble first
                    const uint32_t even = (r2[d] << 4) & 0xF0F0F0F0u, odd = r2[d] & 0xF0F0F0F0u;
                    fb[ks][j][2 * d] = (int32_t)((even & 0xFFu) | ((odd & 0xFFu) << 8) | ((even & 0xFF00u) << 8) |
                                                 ((odd & 0xFF00u) << 16));
                    fb[ks][j][2 * d + 1] = (int32_t)(((even >> 16) & 0xFFu) | (((odd >> 16) & 0xFFu) << 8) |
                                                     (((even >> 24) & 0xFFu) << 16) | ((odd >> 24) << 24));
                }
            } else {
                fb[ks][j] = shortk_load16<BVEC>(g.B + (int64_t)n * g.ldb, k, g.K);
            }
#pragma unroll
            for (int d = 0; d < 4; ++d) colsum = __builtin_amdgcn_sdot4(fb[ks][j][d], 0x01010101, colsum, false);
        }
        colsum += __shfl_xor(colsum, 32);
        if (INT4) colsum >>= 4; // weights are kept times 16; exact
        const int32_t b = g.bias ? g.bias[n] : 0, mu = g.mult[n], sf = g.shift[n];
        fused_ok = fused_ok && sf >= 1 && sf <= 20 && b > -(1 << 27) && b < (1 << 27);
        const int nn = (sf >= 1 && sf <= 20) ? sf : 1;
        col[j].mult = mu;
        col[j].corr = b + (128 - g.z_a) * colsum;
        col[j].n1 = nn + 1;
        col[j].c = 2 * ((1 << (nn - 1)) + (g.z_out << nn)) + 1;
        col[j].lo = (g.lo_rel + g.z_out) << (nn + 1);
        col[j].hi = ((g.hi_rel + g.z_out + 1) << (nn + 1)) - 1;
        col[j].shift = sf; // the general path
    }
    const bool fused = __all(fused_ok);

    // ---- rows (the dispatcher guarantees M < 2^31)
    const int M = (int)g.M;
    const int row_blocks = (M + 31) / 32;
    const int64_t lane_row_off = (int64_t)frow * g.lda + fhalf * 16; // A_MATRIX: offset of this lane's fragment inside a row block
    auto load_rows = [&](int rb, i32x4 (&fa)[KS]) {
        const uint8_t *p;
        if (s.strided) {
            int m = rb * 32 + frow;
            m = m < M ? m : M - 1;
            const uint32_t per_image = (uint32_t)g.Ho * (uint32_t)g.Wo;
            const uint32_t img = (uint32_t)m / per_image, rem = (uint32_t)m - img * per_image;
            const uint32_t ho = rem / (uint32_t)g.Wo, wo = rem - ho * (uint32_t)g.Wo;
            p = g.A + (((int64_t)img * g.H + ho * g.sh) * g.W + wo * g.sw) * g.Cin + fhalf * 16;
        } else if (rb * 32 + 32 <= M) {
            p = g.A + (int64_t)rb * 32 * g.lda + lane_row_off; // uniform base + invariant lane offset
        } else {
            int m = rb * 32 + frow;
            m = m < M ? m : M - 1;
            p = g.A + (int64_t)m * g.lda + fhalf * 16;
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) fa[ks] = shortk_load16<VEC>(p, ks * 32, g.K - fhalf * 16);
    };

    // ALDS: copy of row block rbx into a_tiles[buf]; wave w, pass i moves LDS chunks (i * WAVES + w) * 64 + lane:
    // LDS chunk q = (row, position p) holds global chunk p ^ swz(row) of that row
    auto swz = [](int row) { return CPR == 16 ? (row & 15) : ((row >> 1) & 7); };
    auto issue_tile = [&](int rbx, int buf) __attribute__((always_inline)) {
        constexpr int PASSES = (32 * CPR + WAVES * 64 - 1) / (WAVES * 64);
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
            const int q0 = (i * WAVES + wave) * 64; // wave-uniform
            if (q0 >= 32 * CPR) break;
            const int q = q0 + lane;
            const int row = q / CPR, pos = q % CPR;
            int m = rbx * 32 + row;
            m = m < M ? m : M - 1;
            const uint8_t *src = g.A + (int64_t)m * g.lda + ((pos ^ swz(row)) * 16);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)(a_tiles + buf * ATILE + q0 * 16), 16, 0, 0);
        }
    };
    auto read_tile = [&](int buf, i32x4 (&fa)[KS]) __attribute__((always_inline)) {
        const uint8_t *base = a_tiles + buf * ATILE + frow * KBYTES;
        const int sw = swz(frow);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) fa[ks] = *reinterpret_cast<const i32x4 *>(base + (((2 * ks + fhalf) ^ sw) * 16));
    };

    // lane-invariant parts of the LDS and global addresses of the output tile
    int st_lds[NB], st_row[NB];
    bool st_col_ok[NB];
    int64_t st_off[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int idx = i * 64 + lane;
        st_row[i] = idx / (2 * NB);
        const int col0 = n0 + (idx % (2 * NB)) * 16;
        st_col_ok[i] = col0 < g.N && active;
        st_lds[i] = st_row[i] * PITCH + (idx % (2 * NB)) * 16;
        st_off[i] = (int64_t)st_row[i] * g.ldc + col0;
    }
    const int put_base = (4 * fhalf + (lane & 3)) * PITCH + (frow & ~3);
    // whole 16-byte chunks only, all aligned: one store per lane and chunk, no tail handling
    const bool chunks_whole = g.c_vec16 && ((g.N & 15) == 0 || n0 + 32 * NB <= g.N);

    const int quad_lane = lane & 3;
    const uint32_t sel1 = (quad_lane & 1) ? 0x03070105u : 0x06020400u;
    const uint32_t sel2 = (quad_lane & 2) ? 0x03020706u : 0x05040100u;
    const int32_t lo_rel = g.lo_rel, hi_rel = g.hi_rel, z_out = g.z_out;

    // residual chunks of a row block (ADD): same lanes and addresses as the stores of that block
    int64_t st_roff[NB];
    u32x4 rres[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        st_roff[i] = (int64_t)st_row[i] * g.ldr + (n0 + (i * 64 + lane) % (2 * NB) * 16);
        rres[i] = u32x4{0u, 0u, 0u, 0u};
    }
    auto load_res = [&](int rbx) __attribute__((always_inline)) {
        const uint8_t *const r_block = g.R + (int64_t)rbx * 32 * g.ldr; // wave-uniform
#pragma unroll
        for (int i = 0; i < NB; ++i)
            if (st_col_ok[i] && rbx * 32 + st_row[i] < M) rres[i] = *reinterpret_cast<const u32x4 *>(r_block + st_roff[i]);
    };
    // 16 codes of the layer (v) and of the residual (r) -> 16 output codes: the byte pairs are
    // interleaved into 16-bit table indices [m << 8 | r], one byte gather each
    const AddOut ao = make_add_out(g.add);
    auto add16 = [&](u32x4 v, u32x4 r) __attribute__((always_inline)) {
        u32x4 y;
        if constexpr (use_pairs) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t i01 = __builtin_amdgcn_perm(v[d], r[d], 0x05010400u), i23 = __builtin_amdgcn_perm(v[d], r[d], 0x07030602u);
                const uint32_t t0 = pair_tab[i01 & 0xffffu], t1 = pair_tab[i01 >> 16], t2 = pair_tab[i23 & 0xffffu], t3 = pair_tab[i23 >> 16];
                y[d] = t0 | (t1 << 8) | (t2 << 16) | (t3 << 24);
            }
        } else if (ao.fused) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                y[d] = add_codes4<true>(v[d], r[d], tab, ao);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma nounroll
            for (int d = 0; d < 4; ++d) y[d] = add_codes4<false>(v[d], r[d], tab, ao);
        }
        return y;
    };

    // the output tile of row block rbx, from the wave's LDS area to global memory.  Called one
    // round late, right after the next block's MFMAs are issued and before the loads of the block
    // after it: the stores then never sit between a load and the wait for that load.
    auto store_block = [&](int rbx) __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint8_t *const c_block = g.C + (int64_t)rbx * 32 * g.ldc; // wave-uniform
        if constexpr (ADD) { // the launcher uses ADD only when every output chunk is a whole, aligned 16-byte chunk
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                if (st_col_ok[i] && rbx * 32 + st_row[i] < M)
                    *reinterpret_cast<u32x4 *>(c_block + st_off[i]) =
                        add16(*reinterpret_cast<const u32x4 *>(stage + st_lds[i]), rres[i]);
                __builtin_amdgcn_sched_barrier(0); // one chunk at a time: the table reads of all chunks at once would spill
            }
        } else if (chunks_whole && rbx * 32 + 32 <= M) { // the common case: only the lane-invariant column test
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (st_col_ok[i])
                    *reinterpret_cast<u32x4 *>(c_block + st_off[i]) = *reinterpret_cast<const u32x4 *>(stage + st_lds[i]);
        } else if (chunks_whole) {
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (st_col_ok[i] && rbx * 32 + st_row[i] < M)
                    *reinterpret_cast<u32x4 *>(c_block + st_off[i]) = *reinterpret_cast<const u32x4 *>(stage + st_lds[i]);
        } else {
#pragma nounroll
            for (int i = 0; i < NB; ++i) {
                const int idx = i * 64 + lane;
                const int row = idx / (2 * NB), ch = idx % (2 * NB);
                const int n = n0 + ch * 16;
                if (rbx * 32 + row >= M || n >= g.N) continue;
                uint8_t *dst = c_block + (int64_t)row * g.ldc + n;
                const uint8_t *src = stage + row * PITCH + ch * 16;
#pragma nounroll
                for (int e = 0; e < 16 && n + e < g.N; ++e) dst[e] = src[e];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    // the row loop exists twice (fast and general epilogue) and the choice is made once, outside:
    // inside the loop the compiler would evaluate both forms for every output and select
    auto walk = [&](auto mode_tag) { // 0: general rescale, 1: fused form, 2: fused form without the tie term
    constexpr bool FUSED = decltype(mode_tag)::value > 0, TIES = decltype(mode_tag)::value == 1;
    i32x4 fa[KS];
    int rb = walker, rb_stored = -1, turn = 0;
    if constexpr (ALDS) { // two copies in flight; the first block's fragments are in registers before the loop
        if (rb < row_blocks) {
            issue_tile(rb, 0);
            if (rb + s.walkers < row_blocks) issue_tile(rb + s.walkers, 1);
            __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8)); // vmcnt(0)
            asm volatile("" ::: "memory");
            __syncthreads();
            read_tile(0, fa);
        }
    } else {
        if (rb < row_blocks) load_rows(rb, fa);
    }
    for (; rb < row_blocks; rb += s.walkers, turn ^= 1) {
        i32x16 acc[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = 0;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const i32x4 xs = fa[ks] ^ (int32_t)0x80808080; // uint8 code -> signed (code - 128)
#pragma unroll
            for (int j = 0; j < NB; ++j)
                acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xs, fb[ks][j], acc[j], 0, 0, 0); // columns past N: clamped loads, never stored
        }
        if constexpr (ALDS) {
            // The fragments are consumed.  The next block's copy (issued one round ago, like every store still
            // outstanding) has landed in this wave's part; after the barrier in all parts, and every wave has read
            // the current block (one round ago), whose buffer the copy of the block after next may overwrite.
            // The read-back of the next block's fragments then passes under the epilogue below.
            if (rb + s.walkers < row_blocks) { // uniform over the workgroup
                __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8)); // vmcnt(0)
                asm volatile("" ::: "memory");
                __syncthreads();
                read_tile(turn ^ 1, fa);
                asm volatile("" ::: "memory");
                if (rb + 2 * s.walkers < row_blocks) issue_tile(rb + 2 * s.walkers, turn);
            }
        }
        if (rb_stored >= 0) store_block(rb_stored);
        if constexpr (ADD) load_res(rb); // used one round from now, when this block is stored
        // the fragments are consumed: fetch the next block's into the same registers now, so that
        // the loads are in flight during the epilogue
        if constexpr (!ALDS) {
            if (rb + s.walkers < row_blocks) load_rows(rb + s.walkers, fa);
        }

        // ---- epilogue into the wave's LDS tile: after the 4x4 byte transposition inside each
        // quad of lanes a lane holds 4 consecutive columns of one row
        auto put = [&](int j, int q, uint32_t x) {
            uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true);
            x = __builtin_amdgcn_perm(o, x, sel1);
            o = (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, true);
            x = __builtin_amdgcn_perm(o, x, sel2);
            *reinterpret_cast<uint32_t *>(stage + put_base + q * 8 * PITCH + j * 32) = x;
        };
        if constexpr (FUSED) {
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                if (j >= blocks_here) break;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint32_t x = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int32_t a = acc[j][4 * q + e];
                        if (INT4) a >>= 4;
                        const int32_t t = __mulhi((int32_t)((uint32_t)(a + col[j].corr) << 2), col[j].mult);
                        x = shift_into_byte(x, med3_i32(fused_w_from_t<TIES>(t, col[j].c), col[j].lo, col[j].hi), col[j].n1, e);
                    }
                    put(j, q, x);
                }
            }
        } else { // any multiplier / shift / bias: the general form
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                if (j >= blocks_here) break;
                const RescaleParams rp = make_rescale(col[j].mult, col[j].shift);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint32_t x = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int32_t a = acc[j][4 * q + e];
                        if (INT4) a >>= 4;
                        const int32_t y = clamp_i32(lo_rel, hi_rel, rescale_general(a + col[j].corr, rp)) + z_out;
                        x |= (uint32_t)y << (8 * e);
                    }
                    put(j, q, x);
                }
            }
        }
        // the tile is private to the wave and LDS operations of one wave complete in order:
        // no barrier, only the data dependence through memory
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        rb_stored = rb; // its stores are issued in the next round, after that round's MFMAs
    }
    if (rb_stored >= 0) store_block(rb_stored);
    };
    if (!fused) walk(std::integral_constant<int, 0>{});
    else if (g.lo_rel < 0) walk(std::integral_constant<int, 1>{});
    else walk(std::integral_constant<int, 2>{}); // act_min >= z_out: the clamp absorbs the tie term
}

} // namespace qnn
