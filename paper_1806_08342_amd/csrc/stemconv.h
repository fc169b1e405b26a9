// Convolution with very few input channels (network stems: 3x3x3, 7x7x3), where one kernel row
// (kw * Cin bytes, at most 32) is a contiguous run of bytes in the NHWC image.
//
// The generic implicit-GEMM gather would fetch such a layer byte by byte.  Here a workgroup
// stages the kh image rows that one strip of 128 output pixels needs in LDS with aligned dword
// loads (out-of-image bytes replaced by the code z_x), and every lane cuts its 32-byte window
// (one kernel row of one output pixel; bytes past kw*Cin meet zero weights) out of LDS with
// dword reads + v_alignbyte.  K is laid out as kh sub-steps of 32: one 32x32x32 MFMA per kernel
// row and per 32 output channels.  The weights (zero-padded to 32 per kernel row) are read
// once per workgroup and stay in registers; a workgroup walks several output rows.
// Arithmetic, zero-point correction and epilogue are those of igemm.h.
#pragma once

#include "igemm.h"

namespace qnn {

struct StemArgs {
    IgemmArgs g;     // geometry, pointers, epilogue parameters (g.M = N*Ho*Wo, g.N = Cout, g.ldc = Cout)
    int kh, run;     // run = kw * Cin <= 32
    int rows_per_wg; // output rows one workgroup walks
    int strips;      // ceil(Wo / 128)
};

template <int KH, int TN>
__global__ void __launch_bounds__(256, 2) stemconv_kernel(const StemArgs s)
{
    constexpr int BM = 128, BN = 32 * TN, WM = 4, WN = 1;
    constexpr int W_BYTES = BN * KH * 32;
    constexpr int X_PITCH = 1056; // bytes per staged image row: ((128-1)*stride + kw)*Cin + 3 + 16 <= 1056 (host-checked)
    constexpr int OUT_BYTES = BM * (BN + 16);
    __shared__ __attribute__((aligned(16))) uint8_t w_lds[W_BYTES];
    __shared__ __attribute__((aligned(16))) uint8_t x_lds[KH * X_PITCH];
    __shared__ __attribute__((aligned(16))) uint8_t out_lds[OUT_BYTES];
    const IgemmArgs &g = s.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- block -> (image n, first output row, strip of 128 output columns)
    const int row_groups = (g.Ho + s.rows_per_wg - 1) / s.rows_per_wg;
    int b = blockIdx.x;
    const int strip = b % s.strips;
    b /= s.strips;
    const int rg = b % row_groups;
    const int n = b / row_groups;
    const int wo0 = strip * BM;
    const int ho_begin = rg * s.rows_per_wg;
    const int ho_end = ho_begin + s.rows_per_wg < g.Ho ? ho_begin + s.rows_per_wg : g.Ho;

    // ---- weights: [Cout][kh][run] in memory -> [BN][KH][32] in LDS, zero padded
    for (int i = tid; i < W_BYTES; i += 256) {
        const int c = i & 31, a = (i >> 5) % KH, co = i / (32 * KH);
        uint8_t v = 0;
        if (co < g.N && c < s.run) v = g.B[((int64_t)co * KH + a) * s.run + c];
        w_lds[i] = v;
    }
    const ChannelParams<TN> cparams = load_channel_params<BN, WN, TN>(g, 0);
    __syncthreads();
    const int frag_row = lane & 31, frag_half = lane >> 5;
    i32x4 fb[KH][TN];
    int32_t colsum[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) colsum[j] = 0;
#pragma unroll
    for (int a = 0; a < KH; ++a)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            fb[a][j] = *reinterpret_cast<const i32x4 *>(w_lds + ((j * 32 + frag_row) * KH + a) * 32 + frag_half * 16);
#pragma unroll
            for (int d = 0; d < 4; ++d) colsum[j] = __builtin_amdgcn_sdot4(fb[a][j][d], 0x01010101, colsum[j], false);
        }

    const int row_bytes = g.W * g.Cin;                    // one image row
    const int patch_first = (wo0 * g.sw - g.pw) * g.Cin;  // byte column (may be negative) of the strip's first tap
    const int phase = patch_first & 3;                    // staged rows start at the aligned-down byte column
    const int patch_base = patch_first - phase;
    const int pix_here = (g.Wo - wo0) < BM ? (g.Wo - wo0) : BM;
    const int patch_len = ((pix_here - 1) * g.sw) * g.Cin + 32 + phase; // bytes any lane may touch
    const int patch_dwords = (patch_len + 3) >> 2;
    const uint32_t fill = (uint32_t)g.z_a * 0x01010101u;
    const uint8_t *img = g.A + (int64_t)n * g.H * row_bytes;
    // byte offset of this lane's window inside a staged row
    const int pixel = wave * 32 + frag_row;
    const int win = phase + pixel * g.sw * g.Cin + frag_half * 16;
    const int win_dword = win & ~3, win_shift = win & 3;

    // Staged dwords this lane is responsible for (the same for every output row): LDS offset,
    // kernel row and byte column.  Image rows are a multiple of 4 bytes long and the tensor is
    // 4-byte aligned (dispatcher-checked), so a staged dword lies either fully inside or fully
    // outside an image row: the fetch is one unconditional aligned load from a clamped address
    // plus a select, with no dependent branches between the loads.
    constexpr int PF = (KH * (X_PITCH / 4) + 255) / 256;
    int pf_lds[PF], pf_col[PF], pf_a[PF];
#pragma unroll
    for (int q = 0; q < PF; ++q) {
        const int i = tid + q * 256;
        const int a = i / patch_dwords, d = i - a * patch_dwords;
        pf_a[q] = i < KH * patch_dwords ? a : -1;
        pf_lds[q] = a * X_PITCH + d * 4;
        pf_col[q] = patch_base + d * 4;
    }
    // two register sets: the rows of the next TWO output rows are in flight while one is computed
    uint32_t pre0[PF], pre1[PF];
    auto prefetch = [&](int ho, uint32_t (&pre)[PF]) {
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int hi = ho * g.sh - g.ph + pf_a[q];
            const bool ok = pf_a[q] >= 0 && hi >= 0 && hi < g.H && pf_col[q] >= 0 && pf_col[q] < row_bytes;
            const uint8_t *src = ok ? img + (int64_t)hi * row_bytes + pf_col[q] : img;
            const uint32_t v = *reinterpret_cast<const uint32_t *>(src);
            pre[q] = ok ? v : fill;
        }
    };
    prefetch(ho_begin, pre0);
    if (ho_begin + 1 < ho_end) prefetch(ho_begin + 1, pre1);

    auto output_row = [&](int ho, uint32_t (&pre)[PF]) {
        __syncthreads(); // previous row: fragment reads and output copy are done
#pragma unroll
        for (int q = 0; q < PF; ++q)
            if (pf_a[q] >= 0) *reinterpret_cast<uint32_t *>(x_lds + pf_lds[q]) = pre[q];
        __syncthreads();
        if (ho + 2 < ho_end) prefetch(ho + 2, pre);

        i32x16 acc[1][TN];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[0][j][r] = 0;
#pragma unroll
        for (int a = 0; a < KH; ++a) {
            const uint32_t *p = reinterpret_cast<const uint32_t *>(x_lds + a * X_PITCH + win_dword);
            uint32_t d[5];
#pragma unroll
            for (int e = 0; e < 5; ++e) d[e] = p[e];
            i32x4 fa;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                fa[e] = (int32_t)(__builtin_amdgcn_alignbyte(d[e + 1], d[e], (uint32_t)win_shift) ^ 0x80808080u);
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[0][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb[a][j], acc[0][j], 0, 0, 0);
        }
        // ---- epilogue on the strip: rows of the "GEMM" are the pixels of this output row
        IgemmArgs gl = g;
        const int64_t m0 = ((int64_t)n * g.Ho + ho) * g.Wo + wo0;
        gl.M = m0 + pix_here;
        int32_t cs[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) cs[j] = colsum[j];
        igemm_epilogue<BM, BN, WM, WN, false>(gl, acc, cs, cparams, out_lds, m0, 0);
    };
    for (int ho = ho_begin; ho < ho_end; ho += 2) {
        output_row(ho, pre0);
        if (ho + 1 < ho_end) output_row(ho + 1, pre1);
    }
}

} // namespace qnn
