// Entry points of the dense quantized layers, qnn_qgemm and qnn_qconv2d: this file validates
// arguments, picks the kernel family (launch routines in igemm_*.hip), the tile configuration and
// the staging vector width, and launches the pipelined tile kernels of igemm_dma.h itself.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "igemm_dma.h"
#include "igemm_launch.h"
#include "tuning.h"

namespace qnn {

enum TileConfig {
    TILE_64x64 = 0,
    TILE_128x128,
    TILE_DMA_128x128,
    TILE_DMA_256x256,
    TILE_DMA_256x64,
    TILE_DMA_128x128_S3,
    TILE_DMA_256x64_S3,
    TILE_DMA_256x128,
    TILE_DMA_64x64,
    TILE_DMA_128x256_P, // 4 waves of 64x128, 3 stages, two persistent workgroups per CU
    TILE_DMA_256x128_P, // 4 waves of 128x64, 3 stages, two persistent workgroups per CU
    TILE_DMA_256x256_W4, // 4 waves of 128x128 (one per SIMD, accumulators in the second half of the register file)
    TILE_COUNT
};

static const char *const kTileNames[TILE_COUNT] = {"64x64",     "128x128",      "dma128x128",  "dma256x256", "dma256x64",
                                                   "dma128x128s3", "dma256x64s3", "dma256x128", "dma64x64",  "p128x256",
                                                   "p256x128",  "dma256x256w4"};
static const int kTileM[TILE_COUNT] = {64, 128, 128, 256, 256, 128, 256, 256, 64, 128, 256, 256};
static const int kTileN[TILE_COUNT] = {64, 128, 128, 256, 64, 128, 64, 128, 64, 256, 128, 256};

struct Plan {
    TileConfig tile;
    int splits; // > 1: split-K (128x128 and 64x64 pipelined tiles only)
};

// Tile choice.  `dma_ok`: weights with contiguous columns, 16-byte aligned chunks, K % 64 == 0.
//  - large products: 256x256 tiles (8 waves, 4 LDS stages, one workgroup per CU), or the
//    256x128 / 128x128 / 256x64 tile that wastes the least work in partly filled rounds;
//  - short K (<= 256): 3 LDS stages instead of 4, so that more workgroups fit a CU and one
//    workgroup's epilogue overlaps another one's loads and MFMAs;
//  - products with too few output tiles for 256 CUs: split-K over 128x128 or 64x64 tiles
//    (`split_bytes`: scratch memory the caller offers for the partial sums; 4-bit weights run unsplit).
static Plan choose_plan(int64_t M, int64_t N, int64_t K, bool dma_ok, bool int4, size_t split_bytes)
{
    const Tuning &tu = tuning();
    auto fits = [&](int splits) { return (uint64_t)splits * (uint64_t)M * (uint64_t)N * 4u <= (uint64_t)split_bytes; };
    if (tu.forced()) { // tuning aid: force one configuration
        for (int t = 0; t < TILE_COUNT; ++t)
            if (std::strcmp(tu.force_tile, kTileNames[t]) == 0 && (t < TILE_DMA_128x128 || dma_ok)) {
                if (int4 && t >= TILE_DMA_128x128 && t != TILE_DMA_128x128 && t != TILE_DMA_256x256 && t != TILE_DMA_64x64) break;
                int splits = 1;
                if (!int4 && (t == TILE_DMA_128x128 || t == TILE_DMA_64x64)) splits = tu.force_split > 0 ? tu.force_split : 1;
                const int ksteps = (int)(K / 64);
                splits = splits < 1 ? 1 : (splits > ksteps ? ksteps : splits);
                if (!fits(splits)) splits = 1;
                return Plan{(TileConfig)t, splits};
            }
    }
    if (dma_ok && M >= 128 && int4) { // the pipelined kernel expands nibbles for three tile shapes
        const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256), t128 = ((M + 127) / 128) * ((N + 127) / 128);
        if (K > 256 && N >= 128 && t256 >= 160) return Plan{TILE_DMA_256x256, 1};
        if (N >= 128 && t128 >= 192) return Plan{TILE_DMA_128x128, 1};
        return Plan{TILE_DMA_64x64, 1};
    }
    if (dma_ok && M >= 128) {
        if (K <= 256) { // epilogue-bound: small tiles, several workgroups per CU
            if (N <= 64) return Plan{TILE_DMA_256x64_S3, 1};
            if (N >= 128) return Plan{TILE_DMA_128x128_S3, 1};
        } else {
            // short reductions over several rounds of tiles: the 4-wave 128x256 tile with two workgroups per CU, whose
            // epilogues run under the other workgroup's loop (measured 11-25 % ahead of the 8-wave tiles for
            // K = 320 ... 512 from two rounds on, 5 % at K = 768, level at K = 1024 and on single rounds)
            if (K <= 768 && N >= 256 && ((M + 127) / 128) * ((N + 255) / 256) >= 1024) return Plan{TILE_DMA_128x256_P, 1};
            // pick the configuration with the least padded work: whole waves of workgroups over the
            // chip, weighted by the measured relative MFMA rate of each configuration
            struct Cand { TileConfig t; int per_cu; double rate; };
            // (the 4-wave 256x128 tile, two workgroups per CU: only for a single column of tiles and many rounds --
            // the 3x3 convolutions over 128 channels -- where one workgroup's epilogue runs under the other's loop)
            static const Cand cands[] = {{TILE_DMA_256x256, 1, 1.00}, {TILE_DMA_256x128, 1, 0.88},
                                         {TILE_DMA_128x128, 2, 0.72}, {TILE_DMA_256x64, 2, 0.60},
                                         {TILE_DMA_256x128_P, 2, 1.00}};
            double best = 0.0;
            TileConfig pick = TILE_COUNT;
            for (const Cand &c : cands) {
                const int bm = kTileM[c.t], bn = kTileN[c.t];
                if (N < bn / 2 || M < bm / 2) continue; // mostly empty tiles
                if (c.t == TILE_DMA_256x128_P && (N > 128 || M < 512 * 256)) continue;
                const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
                if (tiles < 160) continue; // would leave too many CUs idle: smaller tiles are better then
                const int64_t slots = 256 * c.per_cu;
                const int64_t waves = (tiles + slots - 1) / slots;
                // time of `waves` rounds; up to 256 tiles every tile has a CU of its own and runs at
                // the full rate of its configuration
                const double cost = tiles <= 256 ? (double)bm * bn / c.rate : (double)waves * c.per_cu * bm * bn / c.rate;
                if (pick == TILE_COUNT || cost < best) best = cost, pick = c.t;
            }
            if (pick != TILE_COUNT) return Plan{pick, 1};
            // Under-filled chip: a lone workgroup's K loop runs at the pace of its own latencies, not
            // of the MFMA pipe, so many small tiles win.  With very few tiles and a long K, the K-steps
            // of each tile are divided over several workgroups as well (measured break-even points:
            // the second pass and the partial sums cost about as much as 16 K-steps).
            const int ksteps = (int)(K / 64);
            const int64_t tiles128 = ((M + 127) / 128) * ((N + 127) / 128), tiles64 = ((M + 63) / 64) * ((N + 63) / 64);
            Plan plan{TILE_DMA_64x64, 1};
            if (tiles128 <= 128 && tiles128 > 16 && ksteps >= 128) plan = Plan{TILE_DMA_128x128, tiles128 <= 64 ? 4 : 2};
            else if (tiles64 <= 64 && ksteps >= 32) {
                const int64_t want = (256 + tiles64 - 1) / tiles64, most = ksteps / 16;
                plan.splits = (int)(want < most ? want : most);
            }
            while (plan.splits > 1 && !fits(plan.splits)) --plan.splits;
            return plan;
        }
    }
    return Plan{(N <= 64 || M <= 64) ? TILE_64x64 : TILE_128x128, 1};
}

// Scratch memory comes from the caller (`workspace` of the entry points): the int32 activation row
// sums of the asymmetric-weight entry points (M values, first) and the partial sums of split-K
// (splits x M x N values, behind them at the next multiple of 256 bytes).
constexpr uint64_t kMaxSplitBytes = (uint64_t)1 << 40;
static size_t rowsum_bytes(int64_t M) { return (size_t)((M * 4 + 255) / 256 * 256); }

static size_t workspace_bytes_for(int64_t M, int64_t N, int64_t K, int weight_bits, bool asym)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    if (asym) return rowsum_bytes(M);
    if ((K % 64) != 0) return 0;                                  // unaligned: the staged kernel, never split
    if (!tuning().forced() && (M <= 64 || K <= 256)) return 0; // few-row and short-K kernels
    const Plan plan = choose_plan(M, N, K, true, weight_bits == 4, (size_t)kMaxSplitBytes);
    if (plan.splits <= 1) return 0;
    const int ksteps = (int)((K / 64 + plan.splits - 1) / plan.splits);
    const int splits = (int)((K / 64 + ksteps - 1) / ksteps);
    return splits > 1 ? (size_t)splits * (size_t)M * (size_t)N * 4 : 0;
}

// One rectangle of the tile grid per XCD: pick the cut (8x1, 4x2, 2x4, 1x8) with the least operand
// traffic from beyond the L2s (8/r copies of A's share + r copies of B's), among those that leave
// the XCDs within 10 % of an even load; else (xcd_rows stays 0) bands of the linear tile sequence.
static void choose_xcd_cut(const IgemmArgs &g, int tiles_m, int tiles_n, int64_t work, int &per_xcd, int &xcd_rows)
{
    const int forced = tuning().xcd_rows;
    double best = 0.0;
    for (int r : {8, 4, 2, 1}) {
        const int c = 8 / r;
        if (forced >= 0 ? r != forced : false) continue;
        if (tiles_m < r || tiles_n < c) continue;
        const int64_t biggest = (int64_t)((tiles_m + r - 1) / r) * ((tiles_n + c - 1) / c);
        if (forced < 0 && biggest * 8 * 10 > work * 11) continue;
        const double traffic = (double)c * (double)g.M + (double)r * (double)g.N; // per unit of K
        if (xcd_rows == 0 || traffic < best) best = traffic, xcd_rows = r, per_xcd = (int)biggest;
    }
}

// `per_cu` > 0: persistent launch with that many workgroups per CU (each walks its XCD's tile
// sequence); 0: one workgroup per tile.  `prio`: issue-priority scheme of the main loop (see the kernel).
template <int BM, int BN, int WM, int WN, int A_MODE, int NSTAGE, bool SPLIT = false, bool ZW = false, bool B4 = false,
          int MINW = 1>
static hipError_t launch_dma(const IgemmArgs &g, hipStream_t s, SplitK sk = SplitK{1, 0, nullptr}, int per_cu = 0, int prio = 0)
{
    constexpr int kStages = NSTAGE * (BM + BN) * 64;
    constexpr int kOut = BM * (BN + 16) + 4 * WM * WN * (BN / WN / 32) * 64 + 2048 + 4 * BM; // + add tables + row sums
    constexpr int kLds = kStages > kOut ? kStages : kOut; // operand ring, reused for the output tile + column sums + add tables
    auto kernel = igemm_dma_kernel<BM, BN, WM, WN, A_MODE, NSTAGE, SPLIT, ZW, B4, MINW>;
    static LdsOptIn opt_in; // per instantiation
    if (hipError_t e = opt_in.ensure(reinterpret_cast<const void *>(kernel), kLds); e != hipSuccess) return e;
    const int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (g.N + BN - 1) / BN;
    const int64_t work = (int64_t)tiles_m * tiles_n * sk.splits;
    int per_xcd = (int)((work + 7) / 8), xcd_rows = 0;
    if (!SPLIT) choose_xcd_cut(g, tiles_m, tiles_n, work, per_xcd, xcd_rows);
    const Tuning &tu = tuning();
    if (tu.persist == 0) per_cu = 0;
    else if (tu.persist > 0) per_cu = tu.persist;
    if (tu.gemm_prio >= 0) prio = tu.gemm_prio;
    int slots = per_xcd; // workgroups per XCD
    if (per_cu > 0 && slots > 32 * per_cu) slots = 32 * per_cu;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(slots * 8)), dim3(WM * WN * 64), kLds, s, g, tiles_m, tiles_n, per_xcd, xcd_rows,
                       sk, prio);
    hipError_t e = hipGetLastError();
    if (SPLIT && e == hipSuccess) {
        const int64_t threads = g.M * (((int64_t)g.N + 3) / 4);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, g, sk);
        e = hipGetLastError();
    }
    return e;
}

// Per-column weight zero-points (eq. 5-6 with z_w != 0): the activation row sums go to the caller's
// scratch memory first (one pass over A), then one tile configuration whose epilogue subtracts
// z_w[n] * rowsum[m]: a pipelined tile when the operands are aligned, else the staged 64x64 tile.
static qnn_status run_igemm_zw(IgemmArgs &g, int a_mode, int b_mode, int vec, int kh, void *workspace, size_t workspace_bytes,
                               hipStream_t s)
{
    if (!workspace || workspace_bytes < rowsum_bytes(g.M) || !aligned_to(workspace, 16)) return QNN_EINVAL;
    int32_t *rowsum = static_cast<int32_t *>(workspace);
    if (qnn_status st = launch_rowsum(g, a_mode, kh, rowsum, s); st != QNN_OK) return st;
    g.rowsum = rowsum;
    const bool i4 = b_mode == B_INT4;
    const bool aligned_for_dma = vec == 16 && (g.K % 64) == 0 && g.lda < (1 << 23) && g.ldb < (1 << 23) &&
                                 (!i4 || (aligned_to(g.B, 16) && (g.ldb % 32) == 0));
    if ((b_mode == B_INT8 || i4) && aligned_for_dma && ((g.M + 127) / 128) * ((g.N + 127) / 128) <= 0x7ffffff) {
        // large products: the 256x256 tile once it fills most of the chip, else 128x128
        const bool big = ((g.M + 255) / 256) * ((g.N + 255) / 256) >= 160 && g.K > 256;
        const bool mat = a_mode == A_MATRIX;
        hipError_t e;
        if (big && i4)
            e = mat ? launch_dma<256, 256, 4, 2, A_MATRIX, 4, false, true, true>(g, s) : launch_dma<256, 256, 4, 2, A_CONV, 4, false, true, true>(g, s);
        else if (big)
            e = mat ? launch_dma<256, 256, 4, 2, A_MATRIX, 4, false, true>(g, s) : launch_dma<256, 256, 4, 2, A_CONV, 4, false, true>(g, s);
        else if (i4)
            e = mat ? launch_dma<128, 128, 2, 2, A_MATRIX, 4, false, true, true>(g, s) : launch_dma<128, 128, 2, 2, A_CONV, 4, false, true, true>(g, s);
        else
            e = mat ? launch_dma<128, 128, 2, 2, A_MATRIX, 4, false, true>(g, s) : launch_dma<128, 128, 2, 2, A_CONV, 4, false, true>(g, s);
        return launch_status(e);
    }
    if (((g.M + 63) / 64) * ((g.N + 63) / 64) > 0x7ffffff) return QNN_EINVAL;
    launch_plain_tile_zw(g, a_mode, b_mode, vec, s);
    return launch_status(hipGetLastError());
}

// Shared back end.  `vec` is the widest staging vector (in k elements) that the alignment
// of A, B and K allows.
static qnn_status run_igemm(IgemmArgs &g, int a_mode, int b_mode, int vec, void *workspace, size_t workspace_bytes,
                            hipStream_t s, int kh = 1)
{
    const int64_t max_tiles = 0x7ffffff;
    g.small_acc = g.K <= 8192 ? 2 : (g.K <= 16384 ? 1 : 0); // |acc| <= K * 2^14
    g.c_vec16 = aligned_to(g.C, 16) && (g.ldc % 16 == 0);
    g.r_vec16 = g.R != nullptr && aligned_to(g.R, 16) && (g.ldr % 16 == 0);
    if (g.zw) return run_igemm_zw(g, a_mode, b_mode, vec, kh, workspace, workspace_bytes, s);
    if (a_mode == A_MATRIX && shortk_eligible(g, b_mode, false)) return launch_shortk(g, b_mode, false, s);
    // kernels that do not apply a residual add themselves run without it; the add follows as a second pass
    auto add_pass = [&](qnn_status st) {
        if (st != QNN_OK || !g.R) return st;
        return launch_add_inplace(g.C, g.ldc, g.R, g.ldr, g.M, g.N, g.add, s);
    };
    {
        qnn_status st;
        IgemmArgs plain = g;
        plain.R = nullptr;
        if (try_skinny(plain, a_mode, b_mode, vec, s, &st)) return add_pass(st);
        if (try_bres(plain, a_mode, b_mode, s, &st)) return add_pass(st);
    }
    const bool mat = a_mode == A_MATRIX;
    const bool i4 = b_mode == B_INT4;
    // the pipelined kernel: 16-byte aligned chunks of A and B (4-bit: 32 elements per chunk), whole K-steps
    const bool dma_ok = (b_mode == B_INT8 || i4) && vec == 16 && (g.K % 64) == 0 && g.lda < (1 << 23) && g.ldb < (1 << 23) &&
                        (!i4 || (aligned_to(g.B, 16) && (g.ldb % 32) == 0));
    if (!aligned_to(workspace, 16)) workspace = nullptr;
    const Plan plan = choose_plan(g.M, g.N, g.K, dma_ok, i4, workspace ? workspace_bytes : 0);
    const TileConfig cfg = plan.tile;
    const int64_t bm = kTileM[cfg], bn = kTileN[cfg];
    // Large outputs on the pipelined tiles: the add as a pass of its own is faster than the add inside the tile
    // epilogue (measured 36 + 16 us against 57 us on 12544 x 2048 x 512: the epilogue looks both codes up in LDS
    // tables, and a streaming pass hides that behind its loads); small layers keep the single launch.
    if (g.R && cfg >= TILE_DMA_128x128 && g.M * (int64_t)g.N >= ((int64_t)1 << 24)) {
        IgemmArgs plain = g;
        plain.R = nullptr;
        return add_pass(run_igemm(plain, a_mode, b_mode, vec, workspace, workspace_bytes, s, kh));
    }
    if (plan.splits > 1) {
        SplitK sk;
        sk.ksteps = (g.K / 64 + plan.splits - 1) / plan.splits;
        sk.splits = (g.K / 64 + sk.ksteps - 1) / sk.ksteps; // no empty K range
        sk.partial = static_cast<int32_t *>(workspace);
        if (sk.partial && sk.splits > 1) {
            hipError_t e;
            IgemmArgs plain = g; // the reduction kernel writes the product's code; the add follows
            plain.R = nullptr;
            if (cfg == TILE_DMA_128x128)
                e = mat ? launch_dma<128, 128, 2, 2, A_MATRIX, 4, true>(plain, s, sk) : launch_dma<128, 128, 2, 2, A_CONV, 4, true>(plain, s, sk);
            else
                e = mat ? launch_dma<64, 64, 2, 2, A_MATRIX, 4, true>(plain, s, sk) : launch_dma<64, 64, 2, 2, A_CONV, 4, true>(plain, s, sk);
            return add_pass(launch_status(e));
        }
    }
    if (((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn) > max_tiles) return QNN_EINVAL;
    const SplitK one{1, 0, nullptr};
    switch (cfg) {
    case TILE_64x64:
        launch_plain_tile(false, g, a_mode, b_mode, vec, s);
        break;
    case TILE_128x128:
        launch_plain_tile(true, g, a_mode, b_mode, vec, s);
        break;
    case TILE_DMA_128x128:
        if (i4) return launch_status(mat ? launch_dma<128, 128, 2, 2, A_MATRIX, 4, false, false, true>(g, s) : launch_dma<128, 128, 2, 2, A_CONV, 4, false, false, true>(g, s));
        return launch_status(mat ? launch_dma<128, 128, 2, 2, A_MATRIX, 4>(g, s) : launch_dma<128, 128, 2, 2, A_CONV, 4>(g, s));
    case TILE_DMA_128x128_S3:
        return launch_status(mat ? launch_dma<128, 128, 2, 2, A_MATRIX, 3>(g, s) : launch_dma<128, 128, 2, 2, A_CONV, 3>(g, s));
    case TILE_DMA_256x256:
        if (i4) return launch_status(mat ? launch_dma<256, 256, 4, 2, A_MATRIX, 4, false, false, true>(g, s) : launch_dma<256, 256, 4, 2, A_CONV, 4, false, false, true>(g, s));
        // persistent workgroups (one per CU) whose second wave of every SIMD trails the first: measured
        // 5-10 % faster than one workgroup per tile on products of several rounds, equal on one round
        return launch_status(mat ? launch_dma<256, 256, 4, 2, A_MATRIX, 4>(g, s, one, 1, 1) : launch_dma<256, 256, 4, 2, A_CONV, 4>(g, s, one, 1, 1));
    case TILE_DMA_256x64:
        return launch_status(mat ? launch_dma<256, 64, 4, 1, A_MATRIX, 4>(g, s) : launch_dma<256, 64, 4, 1, A_CONV, 4>(g, s));
    case TILE_DMA_64x64:
        if (i4) return launch_status(mat ? launch_dma<64, 64, 2, 2, A_MATRIX, 4, false, false, true>(g, s) : launch_dma<64, 64, 2, 2, A_CONV, 4, false, false, true>(g, s));
        return launch_status(mat ? launch_dma<64, 64, 2, 2, A_MATRIX, 4>(g, s) : launch_dma<64, 64, 2, 2, A_CONV, 4>(g, s));
    case TILE_DMA_256x128:
        return launch_status(mat ? launch_dma<256, 128, 4, 2, A_MATRIX, 4>(g, s, one, 1, 0) : launch_dma<256, 128, 4, 2, A_CONV, 4>(g, s, one, 1, 0));
    case TILE_DMA_256x64_S3:
        return launch_status(mat ? launch_dma<256, 64, 4, 1, A_MATRIX, 3>(g, s) : launch_dma<256, 64, 4, 1, A_CONV, 3>(g, s));
    case TILE_DMA_128x256_P:
        return launch_status(mat ? launch_dma<128, 256, 2, 2, A_MATRIX, 3, false, false, false, 2>(g, s, one, 2, 2)
                                 : launch_dma<128, 256, 2, 2, A_CONV, 3, false, false, false, 2>(g, s, one, 2, 2));
    case TILE_DMA_256x128_P:
        return launch_status(mat ? launch_dma<256, 128, 2, 2, A_MATRIX, 3, false, false, false, 2>(g, s, one, 0, 0)
                                 : launch_dma<256, 128, 2, 2, A_CONV, 3, false, false, false, 2>(g, s, one, 0, 0));
    case TILE_DMA_256x256_W4:
        return launch_status(mat ? launch_dma<256, 256, 2, 2, A_MATRIX, 4>(g, s) : launch_dma<256, 256, 2, 2, A_CONV, 4>(g, s));
    default:
        return QNN_EINVAL;
    }
    return launch_status(hipGetLastError());
}

static int pick_vec(int64_t k_like, std::initializer_list<const void *> ptrs, std::initializer_list<int64_t> pitches,
                    int weight_bits)
{
    // candidate widths in elements; a 4-bit element is half a byte
    for (int vec : {16, 8}) {
        const int64_t a_bytes = vec;                                  // activations: 1 byte per element
        const int64_t b_bytes = weight_bits == 4 ? vec / 2 : vec;     // weights
        bool ok = (k_like % vec) == 0;
        int idx = 0;
        for (const void *p : ptrs) ok = ok && aligned_to(p, idx++ == 0 ? a_bytes : b_bytes);
        for (int64_t pitch : pitches) ok = ok && (pitch % vec) == 0;
        if (ok) return vec;
    }
    return 1;
}

// Scratch memory of qnn_qgemm_noalloc: a fixed device array that is part of the library's code object,
// so that the entry point never allocates.  Every GPU the library runs on holds its own copy at its
// own address; the array's name is only a host-side handle, the device address comes from
// hipGetSymbolAddress (once per device, with that device current) and is what the kernels get.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static qnn_status static_scratch(void **out)
{
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return launch_status(e);
    if (dev < 0 || dev >= kMaxDevices) return QNN_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)); e != hipSuccess) return launch_status(e);
        if (!ptr) return QNN_ELAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return QNN_OK;
}

} // namespace qnn

using namespace qnn;

// residual == nullptr: the plain layer; else the add of `add` is applied behind it
static qnn_status fill_add(IgemmArgs &g, const uint8_t *residual, int64_t ldr, const qnn_add_params *add, int32_t z_mid)
{
    if (!residual) return QNN_OK;
    if (!add || ldr < g.N) return QNN_EINVAL;
    auto bad_shift = [](int32_t v) { return v < -31 || v > 31; };
    if (add->left_shift < 0 || add->left_shift > 22 || add->z_r < 0 || add->z_r > 255) return QNN_EINVAL;
    if (bad_shift(add->shift_m) || bad_shift(add->shift_r) || bad_shift(add->shift_o)) return QNN_EINVAL;
    if (bad_out_range(add->z_out, add->act_min, add->act_max)) return QNN_EINVAL;
    g.R = residual, g.ldr = ldr;
    g.add = AddParams{z_mid,          add->mult_m,  add->shift_m, add->z_r,   add->mult_r,  add->shift_r,
                      add->left_shift, add->mult_o, add->shift_o, add->z_out, add->act_min, add->act_max};
    return QNN_OK;
}

static qnn_status qgemm_impl(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                             int weight_bits, int64_t M, int64_t N, int64_t K, const int32_t *bias, const int32_t *mult,
                             const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *C,
                             int64_t ldc, void *workspace, size_t workspace_bytes, void *stream, const uint8_t *residual,
                             int64_t ldr, const qnn_add_params *add, const int32_t *z_w = nullptr)
{
    if (M < 0 || N <= 0 || K <= 0 || K > 65536 || N > 0x7fffffff || lda < K || ldc < N) return QNN_EINVAL;
    if (z_a < 0 || z_a > 255 || bad_out_range(z_out, act_min, act_max)) return QNN_EINVAL;
    if (weight_bits != 8 && weight_bits != 4) return QNN_EINVAL;
    if (b_layout != QNN_B_COLUMNS_CONTIGUOUS && b_layout != QNN_B_ROWS_CONTIGUOUS) return QNN_EINVAL;
    if (b_layout == QNN_B_COLUMNS_CONTIGUOUS ? ldb < K : ldb < N) return QNN_EINVAL;
    if (weight_bits == 4 && (b_layout != QNN_B_COLUMNS_CONTIGUOUS || (K % 2) || (ldb % 2))) return QNN_EINVAL;
    if (M == 0) return QNN_OK; // an empty batch: nothing to compute, no pointer is looked at
    if (!A || !B || !mult || !shift || !C) return QNN_EINVAL;

    IgemmArgs g = {};
    g.A = A, g.lda = lda;
    g.B = static_cast<const uint8_t *>(B), g.ldb = ldb;
    g.M = M, g.N = (int32_t)N, g.K = (int32_t)K, g.z_a = z_a;
    g.bias = bias, g.mult = mult, g.shift = shift;
    g.z_out = z_out, g.lo_rel = act_min - z_out, g.hi_rel = act_max - z_out;
    g.C = C, g.ldc = ldc;
    if (qnn_status st = fill_add(g, residual, ldr, add, z_out); st != QNN_OK) return st;
    g.zw = z_w;
    if (z_w && K > 32768) return QNN_EINVAL; // |sum| < 2^31 needs K * 255 * 255 < 2^31 once z_w != 0
    int b_mode = weight_bits == 4 ? B_INT4 : (b_layout == QNN_B_ROWS_CONTIGUOUS ? B_INT8_ROWS : B_INT8);
    int vec = 1;
    if (b_mode != B_INT8_ROWS) vec = pick_vec(K, {A, B}, {lda, ldb}, weight_bits);
    return run_igemm(g, A_MATRIX, b_mode, vec, workspace, workspace_bytes, as_stream(stream));
}


static qnn_status qconv2d_impl(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                               int kw, int weight_bits, int stride_h, int stride_w, int pad_h, int pad_w,
                               const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t z_out,
                               int32_t act_min, int32_t act_max, uint8_t *y, void *workspace, size_t workspace_bytes,
                               void *stream, const uint8_t *residual, const qnn_add_params *add,
                               const int32_t *z_w = nullptr)
{
    if (N < 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || kh <= 0 || kw <= 0) return QNN_EINVAL;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return QNN_EINVAL;
    if (H + 2 * (int64_t)pad_h < kh || W + 2 * (int64_t)pad_w < kw) return QNN_EINVAL;
    const int64_t K = (int64_t)kh * kw * Cin;
    if (K > 65536 || z_x < 0 || z_x > 255 || bad_out_range(z_out, act_min, act_max)) return QNN_EINVAL;
    if (weight_bits != 8 && weight_bits != 4) return QNN_EINVAL;
    if (weight_bits == 4 && (Cin % 2)) return QNN_EINVAL;
    if (N == 0) return QNN_OK; // an empty batch: nothing to compute, no pointer is looked at
    if (!x || !w || !mult || !shift || !y) return QNN_EINVAL;
    const int Ho = (H + 2 * pad_h - kh) / stride_h + 1, Wo = (W + 2 * pad_w - kw) / stride_w + 1;

    IgemmArgs g = {};
    g.A = x;
    g.H = H, g.W = W, g.Cin = Cin, g.Ho = Ho, g.Wo = Wo, g.kw = kw;
    g.sh = stride_h, g.sw = stride_w, g.ph = pad_h, g.pw = pad_w;
    g.magic_cin = magic_for((uint32_t)Cin), g.magic_kw = magic_for((uint32_t)kw);
    g.B = static_cast<const uint8_t *>(w), g.ldb = K;
    g.M = (int64_t)N * Ho * Wo, g.N = Cout, g.K = (int32_t)K, g.z_a = z_x;
    g.bias = bias, g.mult = mult, g.shift = shift;
    g.z_out = z_out, g.lo_rel = act_min - z_out, g.hi_rel = act_max - z_out;
    g.C = y, g.ldc = Cout;
    if (qnn_status st = fill_add(g, residual, Cout, add, z_out); st != QNN_OK) return st;
    g.r_vec16 = g.R != nullptr && aligned_to(g.R, 16) && (g.ldr % 16 == 0);
    g.zw = z_w;
    if (z_w && K > 32768) return QNN_EINVAL;
    const int b_mode = weight_bits == 4 ? B_INT4 : B_INT8;
    if (!z_w) {
        qnn_status st;
        IgemmArgs plain = g; // the stem kernels do not apply a residual add
        plain.R = nullptr;
        if (try_stem(plain, N, kh, stride_h, stride_w, weight_bits, as_stream(stream), &st)) {
            if (st != QNN_OK || !g.R) return st;
            return launch_add_inplace(g.C, g.ldc, g.R, g.ldr, g.M, g.N, g.add, as_stream(stream));
        }
    }

    const bool pointwise = kh == 1 && kw == 1 && stride_h == 1 && stride_w == 1 && pad_h == 0 && pad_w == 0;
    if (pointwise) { // a 1x1 convolution over NHWC is a plain matrix product
        g.lda = Cin;
        return run_igemm(g, A_MATRIX, b_mode, pick_vec(Cin, {x, w}, {(int64_t)Cin}, weight_bits), workspace, workspace_bytes,
                         as_stream(stream));
    }
    if (!z_w && kh == 1 && kw == 1 && pad_h == 0 && pad_w == 0 && shortk_eligible(g, b_mode, true)) // strided 1x1: rows are pixels
        return launch_shortk(g, b_mode, true, as_stream(stream));
    // pieces must not straddle a tap: the vector width divides Cin
    return run_igemm(g, A_CONV, b_mode, pick_vec(Cin, {x, w}, {(int64_t)Cin}, weight_bits), workspace, workspace_bytes,
                     as_stream(stream), kh);
}



extern "C" {

const char *qnn_qgemm_plan(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return "";
    const Tuning &tu = tuning();
    if (M > 64 && K <= 256 && (K % 8) == 0 && !tu.forced() && !tu.no_shortk) return "shortk";
    if (M <= 64 && (K % 64) == 0) return "skinny16";
    if (M >= 32768 && K > 256 && K <= 1024 && (K % 32) == 0 && N <= 256 && !tu.forced() && tu.bres != 0) return "bres";
    // reported for the aligned int8 case (what the benchmark shapes are), with all the scratch memory it asks for
    const Plan plan = choose_plan(M, N, K, (K % 64) == 0, false, (size_t)kMaxSplitBytes);
    if (plan.splits <= 1) return kTileNames[plan.tile];
    static thread_local char name[48];
    std::snprintf(name, sizeof name, "%s/k%d", kTileNames[plan.tile], plan.splits);
    return name;
}

size_t qnn_qgemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int weight_bits, int asym)
{
    return workspace_bytes_for(M, N, K, weight_bits, asym != 0);
}

size_t qnn_qconv2d_workspace_bytes(int N, int H, int W, int Cin, int Cout, int kh, int kw, int weight_bits, int stride_h,
                                   int stride_w, int pad_h, int pad_w, int asym)
{
    if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 || stride_h <= 0 || stride_w <= 0 ||
        pad_h < 0 || pad_w < 0 || H + 2 * (int64_t)pad_h < kh || W + 2 * (int64_t)pad_w < kw)
        return 0;
    const int64_t Ho = (H + 2 * (int64_t)pad_h - kh) / stride_h + 1, Wo = (W + 2 * (int64_t)pad_w - kw) / stride_w + 1;
    return workspace_bytes_for((int64_t)N * Ho * Wo, Cout, (int64_t)kh * kw * Cin, weight_bits, asym != 0);
}

qnn_status qnn_qgemm(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                     int weight_bits, int64_t M, int64_t N, int64_t K, const int32_t *bias, const int32_t *mult,
                     const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *C, int64_t ldc,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    return qgemm_impl(A, lda, z_a, B, ldb, b_layout, weight_bits, M, N, K, bias, mult, shift, z_out, act_min, act_max, C,
                      ldc, workspace, workspace_bytes, stream, nullptr, 0, nullptr);
}

qnn_status qnn_qgemm_noalloc(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                             int weight_bits, int64_t M, int64_t N, int64_t K, const int32_t *bias, const int32_t *mult,
                             const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *C, int64_t ldc,
                             void *stream)
{
    const size_t need = workspace_bytes_for(M, N, K, weight_bits, false);
    if (need > kStaticScratchBytes) {
        char text[160];
        std::snprintf(text, sizeof text, "qnn_qgemm_noalloc: this product asks for %zu bytes of scratch, the static array holds %zu",
                      need, kStaticScratchBytes);
        set_last_error(text);
        return QNN_EUNSUPPORTED;
    }
    void *ptr = nullptr;
    if (need > 0)
        if (qnn_status st = static_scratch(&ptr); st != QNN_OK) return st;
    return qgemm_impl(A, lda, z_a, B, ldb, b_layout, weight_bits, M, N, K, bias, mult, shift, z_out, act_min, act_max, C,
                      ldc, ptr, need, stream, nullptr, 0, nullptr);
}

qnn_status qnn_qgemm_add(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                         int weight_bits, int64_t M, int64_t N, int64_t K, const int32_t *bias, const int32_t *mult,
                         const int32_t *shift, int32_t z_mid, int32_t mid_min, int32_t mid_max, const uint8_t *residual,
                         int64_t ldr, const qnn_add_params *add, uint8_t *C, int64_t ldc, void *workspace,
                         size_t workspace_bytes, void *stream)
{
    if (!residual || !add) return QNN_EINVAL;
    return qgemm_impl(A, lda, z_a, B, ldb, b_layout, weight_bits, M, N, K, bias, mult, shift, z_mid, mid_min, mid_max, C,
                      ldc, workspace, workspace_bytes, stream, residual, ldr, add);
}

qnn_status qnn_qgemm_asym(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                          int weight_bits, const int32_t *z_w, int64_t M, int64_t N, int64_t K, const int32_t *bias,
                          const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max,
                          uint8_t *C, int64_t ldc, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!z_w) return QNN_EINVAL;
    return qgemm_impl(A, lda, z_a, B, ldb, b_layout, weight_bits, M, N, K, bias, mult, shift, z_out, act_min, act_max, C,
                      ldc, workspace, workspace_bytes, stream, nullptr, 0, nullptr, z_w);
}

qnn_status qnn_qconv2d_asym(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                            int kw, int weight_bits, const int32_t *z_w, int stride_h, int stride_w, int pad_h, int pad_w,
                            const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t z_out,
                            int32_t act_min, int32_t act_max, uint8_t *y, void *workspace, size_t workspace_bytes,
                            void *stream)
{
    if (!z_w) return QNN_EINVAL;
    return qconv2d_impl(x, N, H, W, Cin, z_x, w, Cout, kh, kw, weight_bits, stride_h, stride_w, pad_h, pad_w, bias, mult,
                        shift, z_out, act_min, act_max, y, workspace, workspace_bytes, stream, nullptr, nullptr, z_w);
}

qnn_status qnn_qconv2d(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                       int kw, int weight_bits, int stride_h, int stride_w, int pad_h, int pad_w, const int32_t *bias,
                       const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max,
                       uint8_t *y, void *workspace, size_t workspace_bytes, void *stream)
{
    return qconv2d_impl(x, N, H, W, Cin, z_x, w, Cout, kh, kw, weight_bits, stride_h, stride_w, pad_h, pad_w, bias, mult,
                        shift, z_out, act_min, act_max, y, workspace, workspace_bytes, stream, nullptr, nullptr);
}

qnn_status qnn_qconv2d_add(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                           int kw, int weight_bits, int stride_h, int stride_w, int pad_h, int pad_w,
                           const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t z_mid,
                           int32_t mid_min, int32_t mid_max, const uint8_t *residual, const qnn_add_params *add,
                           uint8_t *y, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!residual || !add) return QNN_EINVAL;
    return qconv2d_impl(x, N, H, W, Cin, z_x, w, Cout, kh, kw, weight_bits, stride_h, stride_w, pad_h, pad_w, bias, mult,
                        shift, z_mid, mid_min, mid_max, y, workspace, workspace_bytes, stream, residual, add);
}

} // extern "C"
