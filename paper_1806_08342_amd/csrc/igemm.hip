// Entry points of the dense quantized layers, qnn_qgemm and qnn_qconv2d: this file validates
// arguments, picks the kernel family (launch routines in igemm_*.hip), the tile configuration and
// the staging vector width, and launches the pipelined tile kernels of igemm_dma.h itself.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "igemm_dma.h"
#include "igemm_launch.h"

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
    TILE_COUNT
};

static const char *const kTileNames[TILE_COUNT] = {"64x64",     "128x128",      "dma128x128",  "dma256x256",
                                                   "dma256x64", "dma128x128s3", "dma256x64s3", "dma256x128", "dma64x64"};
static const int kTileM[TILE_COUNT] = {64, 128, 128, 256, 256, 128, 256, 256, 64};
static const int kTileN[TILE_COUNT] = {64, 128, 128, 256, 64, 128, 64, 128, 64};

// scratch block per device: split-K partial sums in the first half, unpacked 4-bit weights in the second
constexpr size_t kSplitBytes = (size_t)32 << 20, kUnpackBytes = (size_t)32 << 20;
constexpr size_t kWorkspaceBytes = kSplitBytes + kUnpackBytes;

struct Plan {
    TileConfig tile;
    int splits; // > 1: split-K (128x128 and 64x64 pipelined tiles only)
};

static int env_int(const char *name, int fallback)
{
    const char *e = std::getenv(name);
    return e ? std::atoi(e) : fallback;
}

// Tile choice.  `dma_ok`: int8 weights with contiguous columns, 16-byte aligned chunks, K % 64 == 0.
//  - large products: 256x256 tiles (8 waves, 4 LDS stages, one workgroup per CU), or the
//    256x128 / 128x128 / 256x64 tile that wastes the least work in partly filled rounds;
//  - short K (<= 256): 3 LDS stages instead of 4, so that more workgroups fit a CU and one
//    workgroup's epilogue overlaps another one's loads and MFMAs;
//  - products with too few output tiles for 256 CUs: split-K over 128x128 or 64x64 tiles.
static Plan choose_plan(int64_t M, int64_t N, int64_t K, bool dma_ok)
{
    if (const char *force = std::getenv("QNN_FORCE_TILE")) { // tuning aid: force one configuration
        for (int t = 0; t < TILE_COUNT; ++t)
            if (std::strcmp(force, kTileNames[t]) == 0 && (t < TILE_DMA_128x128 || dma_ok)) {
                int splits = 1;
                if (t == TILE_DMA_128x128 || t == TILE_DMA_64x64) splits = env_int("QNN_FORCE_SPLIT", 1);
                const int ksteps = (int)(K / 64);
                splits = splits < 1 ? 1 : (splits > ksteps ? ksteps : splits);
                if ((int64_t)splits * M * N * 4 > (int64_t)kSplitBytes) splits = 1;
                return Plan{(TileConfig)t, splits};
            }
    }
    if (dma_ok && M >= 128) {
        if (K <= 256) { // epilogue-bound: small tiles, several workgroups per CU
            if (N <= 64) return Plan{TILE_DMA_256x64_S3, 1};
            if (N >= 128) return Plan{TILE_DMA_128x128_S3, 1};
        } else {
            // pick the configuration with the least padded work: whole waves of workgroups over the
            // chip, weighted by the measured relative MFMA rate of each configuration
            struct Cand { TileConfig t; int per_cu; double rate; };
            static const Cand cands[] = {{TILE_DMA_256x256, 1, 1.00}, {TILE_DMA_256x128, 1, 0.88},
                                         {TILE_DMA_128x128, 2, 0.72}, {TILE_DMA_256x64, 2, 0.60}};
            double best = 0.0;
            TileConfig pick = TILE_COUNT;
            for (const Cand &c : cands) {
                const int bm = kTileM[c.t], bn = kTileN[c.t];
                if (N < bn / 2 || M < bm / 2) continue; // mostly empty tiles
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
            while (plan.splits > 1 && (int64_t)plan.splits * M * N * 4 > (int64_t)kSplitBytes) --plan.splits;
            return plan;
        }
    }
    return Plan{(N <= 64 || M <= 64) ? TILE_64x64 : TILE_128x128, 1};
}

// Scratch memory of the split-K path and of the 4-bit weight unpacking pass: one fixed block per device, allocated at the first call
// that needs it and kept until the process ends.  Calls on different streams are ordered with
// an event (the block is shared); while a stream is being captured into a graph no event is
// recorded, and no block is allocated if none exists yet (the caller then runs unsplit).
constexpr int kMaxDevices = 64;
struct Workspace {
    int32_t *ptr = nullptr;
    hipEvent_t done = nullptr;
    hipStream_t last = nullptr;
    bool used = false;
};
static Workspace g_workspace[kMaxDevices];
static std::mutex g_workspace_mutex;

static bool stream_is_capturing(hipStream_t s)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st != hipStreamCaptureStatusNone;
}

// the device's scratch block, made safe to overwrite from stream `s`; nullptr if unavailable
static int32_t *acquire_workspace(hipStream_t s, bool capturing)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_workspace_mutex);
    Workspace &w = g_workspace[dev];
    if (!w.ptr) {
        if (capturing) return nullptr; // allocation is not allowed during capture
        if (hipMalloc(reinterpret_cast<void **>(&w.ptr), kWorkspaceBytes) != hipSuccess ||
            hipEventCreateWithFlags(&w.done, hipEventDisableTiming) != hipSuccess) {
            (void)hipGetLastError();
            if (w.ptr) (void)hipFree(w.ptr);
            w.ptr = nullptr;
            return nullptr;
        }
    }
    if (!capturing && w.used && w.last != s) (void)hipStreamWaitEvent(s, w.done, 0);
    return w.ptr;
}

static void release_workspace(hipStream_t s, bool capturing)
{
    if (capturing) return;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return;
    std::lock_guard<std::mutex> lock(g_workspace_mutex);
    Workspace &w = g_workspace[dev];
    if (hipEventRecord(w.done, s) == hipSuccess) w.used = true, w.last = s;
}

// One rectangle of the tile grid per XCD: pick the cut (8x1, 4x2, 2x4, 1x8) with the least operand
// traffic from beyond the L2s (8/r copies of A's share + r copies of B's), among those that leave
// the XCDs within 10 % of an even load; else (xcd_rows stays 0) bands of the linear tile sequence.
static void choose_xcd_cut(const IgemmArgs &g, int tiles_m, int tiles_n, int64_t work, int &per_xcd, int &xcd_rows)
{
    static const int forced = std::getenv("QNN_XCD_ROWS") ? std::atoi(std::getenv("QNN_XCD_ROWS")) : -1;
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

template <int BM, int BN, int WM, int WN, int A_MODE, int NSTAGE, bool SPLIT = false, bool ZW = false>
static hipError_t launch_dma(const IgemmArgs &g, hipStream_t s, SplitK sk = SplitK{1, 0, nullptr})
{
    constexpr int kStages = NSTAGE * (BM + BN) * 64;
    constexpr int kOut = BM * (BN + 16) + 4 * WM * WN * (BN / WN / 32) * 64 + 2048 + 4 * BM; // + add tables + row sums
    constexpr int kLds = kStages > kOut ? kStages : kOut; // operand ring, reused for the output tile + column sums + add tables
    auto kernel = igemm_dma_kernel<BM, BN, WM, WN, A_MODE, NSTAGE, SPLIT, ZW>;
    static LdsOptIn opt_in; // per instantiation
    if (hipError_t e = opt_in.ensure(reinterpret_cast<const void *>(kernel), kLds); e != hipSuccess) return e;
    const int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (g.N + BN - 1) / BN;
    const int64_t work = (int64_t)tiles_m * tiles_n * sk.splits;
    int per_xcd = (int)((work + 7) / 8), xcd_rows = 0;
    if (!SPLIT) choose_xcd_cut(g, tiles_m, tiles_n, work, per_xcd, xcd_rows);
    hipLaunchKernelGGL(kernel, dim3((unsigned)(per_xcd * 8)), dim3(WM * WN * 64), kLds, s, g, tiles_m, tiles_n, per_xcd,
                       xcd_rows, sk);
    hipError_t e = hipGetLastError();
    if (SPLIT && e == hipSuccess) {
        const int64_t threads = g.M * (((int64_t)g.N + 3) / 4);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, g, sk);
        e = hipGetLastError();
    }
    return e;
}



// 4-bit weights for the pipelined kernel: one pass turns the nibble pairs of B ([N][K/2] bytes,
// element 2j in the low nibble of byte j) into int8 [N][K] in scratch memory; the product then runs
// on the int8 path.  Weights are small next to the activations of the layers this is used for
// (M > 64), and the short-K and few-row kernels unpack in registers instead.
__global__ void __launch_bounds__(256) unpack_int4_kernel(const uint8_t *__restrict__ src, int64_t ld_src_bytes, int N, int K,
                                                         int8_t *__restrict__ dst)
{
    const int pieces = K / 16; // 16 elements = 8 packed bytes -> 16 bytes
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)N * pieces) return;
    const int n = (int)(idx / pieces), p = (int)(idx - (int64_t)n * pieces);
    const u32x2 raw = *reinterpret_cast<const u32x2 *>(src + n * ld_src_bytes + p * 8);
    const uint32_t r2[2] = {raw.x, raw.y};
    u32x4 out;
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        uint32_t lo = r2[d] & 0x0F0F0F0Fu, hi = (r2[d] >> 4) & 0x0F0F0F0Fu; // elements 0,2,4,6 / 1,3,5,7 of this dword
        lo |= ((lo >> 3) & 0x01010101u) * 0xF0u;                           // sign-extend each nibble to a byte
        hi |= ((hi >> 3) & 0x01010101u) * 0xF0u;
        out[2 * d] = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
        out[2 * d + 1] = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
    }
    *reinterpret_cast<u32x4 *>(dst + (int64_t)n * K + p * 16) = out;
}

// Per-column weight zero-points (eq. 5-6 with z_w != 0): the activation row sums go to the scratch
// block first (one pass over A), then one tile configuration whose epilogue subtracts
// z_w[n] * rowsum[m]: the pipelined 128x128 tile when the operands are aligned, else the staged
// 64x64 tile.  No split-K (the scratch block holds the row sums).
static qnn_status run_igemm_zw(IgemmArgs &g, int a_mode, int b_mode, int vec, int kh, hipStream_t s)
{
    if (g.M * 4 > (int64_t)kSplitBytes) return QNN_EUNSUPPORTED;
    const bool capturing = stream_is_capturing(s);
    int32_t *workspace = acquire_workspace(s, capturing);
    if (!workspace) return QNN_EUNSUPPORTED; // no scratch block yet and none may be allocated during capture
    auto finish = [&](qnn_status st) {
        release_workspace(s, capturing);
        return st;
    };
    if (qnn_status st = launch_rowsum(g, a_mode, kh, workspace, s); st != QNN_OK) return finish(st);
    g.rowsum = workspace;
    const bool aligned_for_dma = vec == 16 && (g.K % 64) == 0 && g.lda < (1 << 23) && g.ldb < (1 << 23);
    if (b_mode == B_INT4 && aligned_for_dma && (int64_t)g.N * g.K <= (int64_t)kUnpackBytes) {
        int8_t *unpacked = reinterpret_cast<int8_t *>(workspace) + kSplitBytes;
        const int64_t threads = (int64_t)g.N * (g.K / 16);
        hipLaunchKernelGGL(unpack_int4_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, g.B, g.ldb / 2, g.N,
                           g.K, unpacked);
        g.B = reinterpret_cast<const uint8_t *>(unpacked), g.ldb = g.K;
        b_mode = B_INT8;
    }
    if (b_mode == B_INT8 && aligned_for_dma && ((g.M + 127) / 128) * ((g.N + 127) / 128) <= 0x7ffffff) {
        // large products: the 256x256 tile once it fills most of the chip, else 128x128
        const bool big = ((g.M + 255) / 256) * ((g.N + 255) / 256) >= 160 && g.K > 256;
        hipError_t e;
        if (big)
            e = a_mode == A_MATRIX ? launch_dma<256, 256, 4, 2, A_MATRIX, 4, false, true>(g, s)
                                   : launch_dma<256, 256, 4, 2, A_CONV, 4, false, true>(g, s);
        else
            e = a_mode == A_MATRIX ? launch_dma<128, 128, 2, 2, A_MATRIX, 4, false, true>(g, s)
                                   : launch_dma<128, 128, 2, 2, A_CONV, 4, false, true>(g, s);
        return finish(launch_status(e));
    }
    if (((g.M + 63) / 64) * ((g.N + 63) / 64) > 0x7ffffff) return finish(QNN_EINVAL);
    launch_plain_tile_zw(g, a_mode, b_mode, vec, s);
    return finish(launch_status(hipGetLastError()));
}

// Shared back end.  `vec` is the widest staging vector (in k elements) that the alignment
// of A, B and K allows.
static qnn_status run_igemm(IgemmArgs &g, int a_mode, int b_mode, int vec, hipStream_t s, int kh = 1)
{
    const int64_t max_tiles = 0x7ffffff;
    g.small_acc = g.K <= 8192 ? 2 : (g.K <= 16384 ? 1 : 0); // |acc| <= K * 2^14
    g.c_vec16 = aligned_to(g.C, 16) && (g.ldc % 16 == 0);
    g.r_vec16 = g.R != nullptr && aligned_to(g.R, 16) && (g.ldr % 16 == 0);
    if (g.zw) return run_igemm_zw(g, a_mode, b_mode, vec, kh, s);
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
    const bool mat_or_conv = a_mode == A_MATRIX;
    bool capturing = false, workspace_used = false;
    int32_t *workspace = nullptr;
    const bool aligned_for_dma = vec == 16 && (g.K % 64) == 0 && g.lda < (1 << 23) && g.ldb < (1 << 23);
    // 4-bit weights: unpack once into scratch memory, then the int8 pipelined kernel
    if (b_mode == B_INT4 && aligned_for_dma && (int64_t)g.N * g.K <= (int64_t)kUnpackBytes &&
        std::getenv("QNN_FORCE_TILE") == nullptr) {
        capturing = stream_is_capturing(s);
        workspace = acquire_workspace(s, capturing);
        if (workspace) {
            int8_t *unpacked = reinterpret_cast<int8_t *>(workspace) + kSplitBytes;
            const int64_t threads = (int64_t)g.N * (g.K / 16);
            hipLaunchKernelGGL(unpack_int4_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, g.B, g.ldb / 2,
                               g.N, g.K, unpacked);
            g.B = reinterpret_cast<const uint8_t *>(unpacked), g.ldb = g.K;
            b_mode = B_INT8;
            workspace_used = true;
        }
    }
    const bool dma_ok = b_mode == B_INT8 && aligned_for_dma;
    const Plan plan = choose_plan(g.M, g.N, g.K, dma_ok);
    const TileConfig cfg = plan.tile;
    const int64_t bm = kTileM[cfg], bn = kTileN[cfg];
    auto finish = [&](qnn_status st) { // the scratch block is free again after what was enqueued so far
        if (workspace_used) release_workspace(s, capturing);
        return st;
    };
    if (plan.splits > 1) {
        if (!workspace) {
            capturing = stream_is_capturing(s);
            workspace = acquire_workspace(s, capturing);
        }
        SplitK sk;
        sk.ksteps = (g.K / 64 + plan.splits - 1) / plan.splits;
        sk.splits = (g.K / 64 + sk.ksteps - 1) / sk.ksteps; // no empty K range
        sk.partial = workspace;
        if (sk.partial && sk.splits > 1) {
            workspace_used = true;
            hipError_t e;
            IgemmArgs plain = g; // the reduction kernel writes the product's code; the add follows
            plain.R = nullptr;
            if (cfg == TILE_DMA_128x128)
                e = mat_or_conv ? launch_dma<128, 128, 2, 2, A_MATRIX, 4, true>(plain, s, sk)
                                : launch_dma<128, 128, 2, 2, A_CONV, 4, true>(plain, s, sk);
            else
                e = mat_or_conv ? launch_dma<64, 64, 2, 2, A_MATRIX, 4, true>(plain, s, sk)
                                : launch_dma<64, 64, 2, 2, A_CONV, 4, true>(plain, s, sk);
            return finish(add_pass(launch_status(e)));
        }
    }
    if (((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn) > max_tiles) return finish(QNN_EINVAL);
    const bool mat = a_mode == A_MATRIX;
    switch (cfg) {
    case TILE_64x64:
        launch_plain_tile(false, g, a_mode, b_mode, vec, s);
        break;
    case TILE_128x128:
        launch_plain_tile(true, g, a_mode, b_mode, vec, s);
        break;
    case TILE_DMA_128x128:
        return finish(launch_status(mat ? launch_dma<128, 128, 2, 2, A_MATRIX, 4>(g, s) : launch_dma<128, 128, 2, 2, A_CONV, 4>(g, s)));
    case TILE_DMA_128x128_S3:
        return finish(launch_status(mat ? launch_dma<128, 128, 2, 2, A_MATRIX, 3>(g, s) : launch_dma<128, 128, 2, 2, A_CONV, 3>(g, s)));
    case TILE_DMA_256x256:
        return finish(launch_status(mat ? launch_dma<256, 256, 4, 2, A_MATRIX, 4>(g, s) : launch_dma<256, 256, 4, 2, A_CONV, 4>(g, s)));
    case TILE_DMA_256x64:
        return finish(launch_status(mat ? launch_dma<256, 64, 4, 1, A_MATRIX, 4>(g, s) : launch_dma<256, 64, 4, 1, A_CONV, 4>(g, s)));
    case TILE_DMA_64x64:
        return finish(launch_status(mat ? launch_dma<64, 64, 2, 2, A_MATRIX, 4>(g, s) : launch_dma<64, 64, 2, 2, A_CONV, 4>(g, s)));
    case TILE_DMA_256x128:
        return finish(launch_status(mat ? launch_dma<256, 128, 4, 2, A_MATRIX, 4>(g, s) : launch_dma<256, 128, 4, 2, A_CONV, 4>(g, s)));
    case TILE_DMA_256x64_S3:
        return finish(launch_status(mat ? launch_dma<256, 64, 4, 1, A_MATRIX, 3>(g, s) : launch_dma<256, 64, 4, 1, A_CONV, 3>(g, s)));
    default:
        return finish(QNN_EINVAL);
    }
    return finish(launch_status(hipGetLastError()));
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
                             int64_t ldc, void *stream, const uint8_t *residual, int64_t ldr, const qnn_add_params *add,
                             const int32_t *z_w = nullptr)
{
    if (!A || !B || !mult || !shift || !C) return QNN_EINVAL;
    if (M <= 0 || N <= 0 || K <= 0 || K > 65536 || N > 0x7fffffff || lda < K || ldc < N) return QNN_EINVAL;
    if (z_a < 0 || z_a > 255 || bad_out_range(z_out, act_min, act_max)) return QNN_EINVAL;
    if (weight_bits != 8 && weight_bits != 4) return QNN_EINVAL;
    if (b_layout != QNN_B_COLUMNS_CONTIGUOUS && b_layout != QNN_B_ROWS_CONTIGUOUS) return QNN_EINVAL;
    if (b_layout == QNN_B_COLUMNS_CONTIGUOUS ? ldb < K : ldb < N) return QNN_EINVAL;
    if (weight_bits == 4 && (b_layout != QNN_B_COLUMNS_CONTIGUOUS || (K % 2) || (ldb % 2))) return QNN_EINVAL;

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
    return run_igemm(g, A_MATRIX, b_mode, vec, as_stream(stream));
}


static qnn_status qconv2d_impl(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                               int kw, int weight_bits, int stride_h, int stride_w, int pad_h, int pad_w,
                               const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t z_out,
                               int32_t act_min, int32_t act_max, uint8_t *y, void *stream, const uint8_t *residual,
                               const qnn_add_params *add, const int32_t *z_w = nullptr)
{
    if (!x || !w || !mult || !shift || !y) return QNN_EINVAL;
    if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || kh <= 0 || kw <= 0) return QNN_EINVAL;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return QNN_EINVAL;
    if (H + 2 * (int64_t)pad_h < kh || W + 2 * (int64_t)pad_w < kw) return QNN_EINVAL;
    const int64_t K = (int64_t)kh * kw * Cin;
    if (K > 65536 || z_x < 0 || z_x > 255 || bad_out_range(z_out, act_min, act_max)) return QNN_EINVAL;
    if (weight_bits != 8 && weight_bits != 4) return QNN_EINVAL;
    if (weight_bits == 4 && (Cin % 2)) return QNN_EINVAL;
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
        return run_igemm(g, A_MATRIX, b_mode, pick_vec(Cin, {x, w}, {(int64_t)Cin}, weight_bits), as_stream(stream));
    }
    if (!z_w && kh == 1 && kw == 1 && pad_h == 0 && pad_w == 0 && shortk_eligible(g, b_mode, true)) // strided 1x1: rows are pixels
        return launch_shortk(g, b_mode, true, as_stream(stream));
    // pieces must not straddle a tap: the vector width divides Cin
    return run_igemm(g, A_CONV, b_mode, pick_vec(Cin, {x, w}, {(int64_t)Cin}, weight_bits), as_stream(stream), kh);
}



extern "C" {

const char *qnn_qgemm_plan(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return "";
    if (M > 64 && K <= 256 && (K % 8) == 0 && std::getenv("QNN_FORCE_TILE") == nullptr && std::getenv("QNN_NO_SHORTK") == nullptr)
        return "shortk";
    if (M <= 64 && (K % 64) == 0) return "skinny16";
    if (M >= 32768 && K > 256 && K <= 1024 && (K % 32) == 0 && N <= 256 && std::getenv("QNN_FORCE_TILE") == nullptr &&
        (std::getenv("QNN_BRES") == nullptr || std::atoi(std::getenv("QNN_BRES")) != 0))
        return "bres";
    // reported for the aligned int8 case (what the benchmark shapes are)
    const Plan plan = choose_plan(M, N, K, (K % 64) == 0);
    if (plan.splits <= 1) return kTileNames[plan.tile];
    static thread_local char name[48];
    std::snprintf(name, sizeof name, "%s/k%d", kTileNames[plan.tile], plan.splits);
    return name;
}

qnn_status qnn_qgemm(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                     int weight_bits, int64_t M, int64_t N, int64_t K, const int32_t *bias, const int32_t *mult,
                     const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *C, int64_t ldc,
                     void *stream)
{
    return qgemm_impl(A, lda, z_a, B, ldb, b_layout, weight_bits, M, N, K, bias, mult, shift, z_out, act_min, act_max, C,
                      ldc, stream, nullptr, 0, nullptr);
}

qnn_status qnn_qgemm_add(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                         int weight_bits, int64_t M, int64_t N, int64_t K, const int32_t *bias, const int32_t *mult,
                         const int32_t *shift, int32_t z_mid, int32_t mid_min, int32_t mid_max, const uint8_t *residual,
                         int64_t ldr, const qnn_add_params *add, uint8_t *C, int64_t ldc, void *stream)
{
    if (!residual || !add) return QNN_EINVAL;
    return qgemm_impl(A, lda, z_a, B, ldb, b_layout, weight_bits, M, N, K, bias, mult, shift, z_mid, mid_min, mid_max, C,
                      ldc, stream, residual, ldr, add);
}

qnn_status qnn_qgemm_asym(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                          int weight_bits, const int32_t *z_w, int64_t M, int64_t N, int64_t K, const int32_t *bias,
                          const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max,
                          uint8_t *C, int64_t ldc, void *stream)
{
    if (!z_w) return QNN_EINVAL;
    return qgemm_impl(A, lda, z_a, B, ldb, b_layout, weight_bits, M, N, K, bias, mult, shift, z_out, act_min, act_max, C,
                      ldc, stream, nullptr, 0, nullptr, z_w);
}

qnn_status qnn_qconv2d_asym(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                            int kw, int weight_bits, const int32_t *z_w, int stride_h, int stride_w, int pad_h, int pad_w,
                            const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t z_out,
                            int32_t act_min, int32_t act_max, uint8_t *y, void *stream)
{
    if (!z_w) return QNN_EINVAL;
    return qconv2d_impl(x, N, H, W, Cin, z_x, w, Cout, kh, kw, weight_bits, stride_h, stride_w, pad_h, pad_w, bias, mult,
                        shift, z_out, act_min, act_max, y, stream, nullptr, nullptr, z_w);
}

qnn_status qnn_qconv2d(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                       int kw, int weight_bits, int stride_h, int stride_w, int pad_h, int pad_w, const int32_t *bias,
                       const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max,
                       uint8_t *y, void *stream)
{
    return qconv2d_impl(x, N, H, W, Cin, z_x, w, Cout, kh, kw, weight_bits, stride_h, stride_w, pad_h, pad_w, bias, mult,
                        shift, z_out, act_min, act_max, y, stream, nullptr, nullptr);
}

qnn_status qnn_qconv2d_add(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                           int kw, int weight_bits, int stride_h, int stride_w, int pad_h, int pad_w,
                           const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t z_mid,
                           int32_t mid_min, int32_t mid_max, const uint8_t *residual, const qnn_add_params *add,
                           uint8_t *y, void *stream)
{
    if (!residual || !add) return QNN_EINVAL;
    return qconv2d_impl(x, N, H, W, Cin, z_x, w, Cout, kh, kw, weight_bits, stride_h, stride_w, pad_h, pad_w, bias, mult,
                        shift, z_mid, mid_min, mid_max, y, stream, residual, add);
}

} // extern "C"
