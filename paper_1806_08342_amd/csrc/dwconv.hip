// Depthwise convolution (one kh x kw kernel per channel), NHWC uint8 -> NHWC uint8.
//
// 18 integer operations per output byte: the kernel is bound by HBM traffic and by the
// vector ALU, not by the matrix cores, so it does not use MFMA.  Channels are the
// contiguous axis: one lane owns 4 consecutive channels (one dword of activations, one
// dword of weights per tap) and a small patch of output pixels, so that the input window is
// loaded and unpacked once and reused by every output of the patch; consecutive lanes own
// consecutive channel groups, which makes every load and store of a wave a contiguous run
// of channels.
//
//   acc[c] = sum_{a,b} (x[hi][wi][c] - z_x) * w[a][b][c]    taps outside the image skipped
//   out    = clamp(z_out + RESCALE(acc + bias[c]; mult[c], shift[c]))            (eq. 4-6, z_w = 0)
#include <cstdlib>
#include <type_traits>

#include "qnn_device.h"
#include "tuning.h"

namespace qnn {

struct DwArgs {
    const uint8_t *x;
    const int8_t *w;
    uint8_t *y;
    const int32_t *bias, *mult, *shift;
    const int32_t *zw; // per-channel weight zero-points, or nullptr (generic kernel only)
    int N, H, W, C, Ho, Wo, kh, kw, sh, sw, ph, pw;
    int32_t z_x, z_out, lo_rel, hi_rel;
    int64_t total_work; // lanes of work
    int wruns, hruns;   // patches of RW x RH output pixels per image row / column
    uint32_t magic_cgroups, shift_cgroups; // x / (C/4) = umulhi(x, magic) >> shift for x < 2^31
};

__device__ __forceinline__ int32_t sbyte(uint32_t v, int j) { return (int32_t)(int8_t)(v >> (8 * j)); }
__device__ __forceinline__ int32_t ubyte(uint32_t v, int j) { return (int32_t)((v >> (8 * j)) & 0xffu); }

// 3x3 kernel, stride S (same in h and w).  One lane owns 4 consecutive channels and an
// RH x RW patch of output pixels; the ((RH-1)S+3) x ((RW-1)S+3) input window is loaded once
// (one dword = 4 channels per pixel), each byte is unpacked once and multiplied into every
// output of the patch that uses it.  The accumulators start at bias - z_x * sum(w) and taps
// outside the image read as the code z_x, which is the expansion of eq. 5-6 (z_w = 0) with
// the border padded by the code of real zero.
template <int S, int RH, int RW>
__global__ void __launch_bounds__(256) dwconv3x3_kernel(const DwArgs g)
{
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= g.total_work) return;
    const int cgroups = g.C >> 2;
    const int cg = (int)(gid % cgroups);
    int64_t t = gid / cgroups;
    const int pw = (int)(t % g.wruns);
    t /= g.wruns;
    const int ph = (int)(t % g.hruns);
    const int n = (int)(t / g.hruns);
    const int c0 = cg * 4;
    const int ho0 = ph * RH, wo0 = pw * RW;

    // weights as sign-extended ints, and their per-channel sums
    int32_t wt[3][3][4];
    int32_t wsum[4] = {0, 0, 0, 0};
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            const uint32_t wv = *reinterpret_cast<const uint32_t *>(g.w + ((int64_t)a * 3 + b) * g.C + c0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                wt[a][b][j] = sbyte(wv, j);
                wsum[j] += wt[a][b][j];
            }
        }
    int32_t acc[RH][RW][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int32_t init = (g.bias ? g.bias[c0 + j] : 0) - g.z_x * wsum[j];
#pragma unroll
        for (int r = 0; r < RH; ++r)
#pragma unroll
            for (int p = 0; p < RW; ++p) acc[r][p][j] = init;
    }

    constexpr int ROWS = (RH - 1) * S + 3, COLS = (RW - 1) * S + 3;
    const int hi0 = ho0 * S - g.ph, wi0 = wo0 * S - g.pw;
    const uint8_t *img = g.x + (int64_t)n * g.H * g.W * g.C + c0;
    const uint32_t fill = (uint32_t)g.z_x * 0x01010101u;
#pragma unroll
    for (int row = 0; row < ROWS; ++row) {
        const int hi = hi0 + row;
        const bool row_ok = hi >= 0 && hi < g.H;
        const uint8_t *line = img + (int64_t)hi * g.W * g.C;
        uint32_t v[COLS];
#pragma unroll
        for (int col = 0; col < COLS; ++col) {
            const int wi = wi0 + col;
            v[col] = fill;
            if (row_ok && wi >= 0 && wi < g.W) v[col] = *reinterpret_cast<const uint32_t *>(line + (int64_t)wi * g.C);
        }
#pragma unroll
        for (int col = 0; col < COLS; ++col) {
            int32_t xv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) xv[j] = ubyte(v[col], j);
#pragma unroll
            for (int r = 0; r < RH; ++r) {
                const int a = row - r * S; // kernel row of this input row for output row r
                if (a < 0 || a > 2) continue;
#pragma unroll
                for (int p = 0; p < RW; ++p) {
                    const int b = col - p * S;
                    if (b < 0 || b > 2) continue;
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[r][p][j] += xv[j] * wt[a][b][j];
                }
            }
        }
    }

    RescaleParams rp[4];
    FusedRescale fr[4];
    bool fused_ok = true;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int32_t mu = g.mult[c0 + j], sf = g.shift[c0 + j];
        rp[j] = make_rescale(mu, sf);
        fused_ok = fused_ok && sf >= 1 && sf <= 20;
        fr[j] = make_fused(mu, sf, 0, g.z_out, g.lo_rel + g.z_out, g.hi_rel + g.z_out);
    }
    // |acc| <= |bias| + 2 * 9 * 255 * 128: the fused form needs |acc| < 2^29, i.e. a sane bias
    if (g.bias) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int32_t b = g.bias[c0 + j];
            fused_ok = fused_ok && b > -(1 << 28) && b < (1 << 28);
        }
    }
    const bool fused = __all(fused_ok);
#pragma unroll
    for (int r = 0; r < RH; ++r) {
        if (ho0 + r >= g.Ho) break;
        uint8_t *out = g.y + (((int64_t)n * g.Ho + ho0 + r) * g.Wo + wo0) * g.C + c0;
#pragma unroll
        for (int p = 0; p < RW; ++p) {
            if (wo0 + p >= g.Wo) break;
            uint32_t packed = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int32_t y;
                if (fused) y = rescale_fused(acc[r][p][j], fr[j]);
                else y = clamp_i32(g.lo_rel, g.hi_rel, rescale_general(acc[r][p][j], rp[j])) + g.z_out;
                packed |= (uint32_t)y << (8 * j);
            }
            *reinterpret_cast<uint32_t *>(out + (int64_t)p * g.C) = packed;
        }
    }
}

// Same layer, multiply-accumulates on the 4-way int8 dot product instruction.
//
// In NHWC a dword holds 4 channels of one pixel, but the sum of a depthwise kernel runs over
// pixels of ONE channel.  Each input row of the window is therefore transposed in registers
// (byte permutes) into per-channel dwords of 4 consecutive pixels, x - 128 as signed bytes.
// One kernel row of one channel is the signed byte vector [w0, w1, w2, 0]: its dot product with
// pixels (p, p+1, p+2, p+3) is the row's contribution to output p, and the same vector shifted by
// one byte gives output p+1 from the same dword, so a row of 4 outputs costs 5 (stride 1) or
// 6 (stride 2) instructions per channel and kernel row instead of 12 multiply-adds plus the
// byte unpacking.  acc starts at bias + (128 - z_x) * sum(w); taps outside the image read as
// the code z_x.  One lane: 4 channels x RH x 4 outputs.
//
// Launch: grid.x covers (patch along W, channel group) lanes, grid.y the patches along H, grid.z
// the images, so that the image and the input rows of a workgroup are wave-uniform: row
// addresses and row bounds live in scalar registers, and a lane only keeps the byte offset and
// the in-image flag of its COLS window columns.  Every load is unconditional (from a clamped
// address) followed by a select of the padding code: no branches around memory operations.
template <int S, int RH>
__global__ void __launch_bounds__(256) dwconv3x3_dot_kernel(const DwArgs g)
{
    constexpr int RW = 4;
    constexpr int ROWS = (RH - 1) * S + 3, COLS = (RW - 1) * S + 3; // 6 or 9 input pixels per window row
    const uint32_t lane_x = blockIdx.x * 256u + threadIdx.x;
    const uint32_t cgroups = (uint32_t)g.C >> 2;
    const uint32_t pw = cgroups == 1 ? lane_x : __umulhi(lane_x, g.magic_cgroups) >> g.shift_cgroups; // lane_x / cgroups
    const uint32_t cg = lane_x - pw * cgroups;
    if (pw >= (uint32_t)g.wruns) return;
    const int n = blockIdx.z, ph = blockIdx.y; // wave-uniform
    const int c0 = (int)cg * 4;
    const int ho0 = ph * RH, wo0 = (int)pw * RW;

    // ---- weights: wa[a][j] = [w(a,0), w(a,1), w(a,2), 0] of channel c0 + j
    uint32_t wa[3][4];
    int32_t wsum[4] = {0, 0, 0, 0};
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        uint32_t wv[3];
#pragma unroll
        for (int b = 0; b < 3; ++b) wv[b] = *reinterpret_cast<const uint32_t *>(g.w + (a * 3 + b) * g.C + c0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t t01 = __builtin_amdgcn_perm(wv[1], wv[0], 0x0c0c0000u | ((4u + j) << 8) | (uint32_t)j);
            wa[a][j] = __builtin_amdgcn_perm(wv[2], t01, 0x0c000100u | ((4u + j) << 16));
            wsum[j] = __builtin_amdgcn_sdot4((int)wa[a][j], 0x01010101, wsum[j], false);
        }
    }
    int32_t acc[RH][RW][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int32_t init = (g.bias ? g.bias[c0 + j] : 0) + (128 - g.z_x) * wsum[j];
#pragma unroll
        for (int r = 0; r < RH; ++r)
#pragma unroll
            for (int p = 0; p < RW; ++p) acc[r][p][j] = init;
    }

    const int hi0 = ho0 * S - g.ph, wi0 = wo0 * S - g.pw;
    const uint8_t *img = g.x + (int64_t)n * g.H * g.W * g.C; // scalar
    const uint32_t fill = (uint32_t)g.z_x * 0x01010101u;
    // byte offset inside an image row and in-image flag of each window column (the dispatcher
    // guarantees W * C < 2^31)
    uint32_t col_off[COLS]; // unsigned: scalar base + 32-bit lane offset addressing
    bool col_ok[COLS];
#pragma unroll
    for (int col = 0; col < COLS; ++col) {
        const int wi = wi0 + col;
        col_ok[col] = wi >= 0 && wi < g.W;
        col_off[col] = (uint32_t)((col_ok[col] ? wi : 0) * g.C + c0);
    }
    // 4 pixel dwords (4 channels each) -> 4 channel dwords (4 pixels each)
    auto transpose4 = [](const uint32_t *v, uint32_t (&x)[4]) {
        const uint32_t lo01 = __builtin_amdgcn_perm(v[1], v[0], 0x05010400u), hi01 = __builtin_amdgcn_perm(v[1], v[0], 0x07030602u);
        const uint32_t lo23 = __builtin_amdgcn_perm(v[3], v[2], 0x05010400u), hi23 = __builtin_amdgcn_perm(v[3], v[2], 0x07030602u);
        x[0] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
        x[1] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
        x[2] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
        x[3] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
    };
    const uint32_t fill_s = fill ^ 0x80808080u;
#pragma unroll
    for (int row = 0; row < ROWS; ++row) {
        const int hi = hi0 + row;                       // scalar
        const bool row_ok = hi >= 0 && hi < g.H;        // scalar
        const uint8_t *line = img + (int64_t)(row_ok ? hi : 0) * g.W * g.C; // scalar, always inside the image
        uint32_t v[COLS];
#pragma unroll
        for (int col = 0; col < COLS; ++col) v[col] = *reinterpret_cast<const uint32_t *>(line + col_off[col]);
#pragma unroll
        for (int col = 0; col < COLS; ++col) v[col] = (row_ok && col_ok[col]) ? (v[col] ^ 0x80808080u) : fill_s; // signed (code - 128)
        uint32_t x0[4], x1[4], x2[4] = {0u, 0u, 0u, 0u};
        transpose4(v, x0);
        if constexpr (S == 1) { // pixels 4, 5 -> [p4, p5, 0, 0]
#pragma unroll
            for (int j = 0; j < 4; ++j) x1[j] = __builtin_amdgcn_perm(v[5], v[4], 0x0c0c0000u | ((4u + j) << 8) | (uint32_t)j);
        } else { // pixels 4..7, and pixel 8 alone
            transpose4(v + 4, x1);
#pragma unroll
            for (int j = 0; j < 4; ++j) x2[j] = (v[8] >> (8 * j)) & 0xffu;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // stride 1: pixels (2, 3, 4, 5) as one dword
            const uint32_t y = S == 1 ? __builtin_amdgcn_alignbyte(x1[j], x0[j], 2) : 0u;
#pragma unroll
            for (int r = 0; r < RH; ++r) {
                const int a = row - r * S; // kernel row of this input row for output row r
                if (a < 0 || a > 2) continue;
                const uint32_t w = wa[a][j];
                if constexpr (S == 1) {
                    acc[r][0][j] = __builtin_amdgcn_sdot4((int)x0[j], (int)w, acc[r][0][j], false);
                    acc[r][1][j] = __builtin_amdgcn_sdot4((int)x0[j], (int)(w << 8), acc[r][1][j], false);
                    acc[r][2][j] = __builtin_amdgcn_sdot4((int)y, (int)w, acc[r][2][j], false);
                    acc[r][3][j] = __builtin_amdgcn_sdot4((int)y, (int)(w << 8), acc[r][3][j], false);
                } else { // output p uses pixels 2p, 2p+1, 2p+2
                    acc[r][0][j] = __builtin_amdgcn_sdot4((int)x0[j], (int)w, acc[r][0][j], false);
                    acc[r][1][j] = __builtin_amdgcn_sdot4((int)x0[j], (int)(w << 16), acc[r][1][j], false);
                    acc[r][1][j] = __builtin_amdgcn_sdot4((int)x1[j], (int)(w >> 16), acc[r][1][j], false);
                    acc[r][2][j] = __builtin_amdgcn_sdot4((int)x1[j], (int)w, acc[r][2][j], false);
                    acc[r][3][j] = __builtin_amdgcn_sdot4((int)x1[j], (int)(w << 16), acc[r][3][j], false);
                    acc[r][3][j] = __builtin_amdgcn_sdot4((int)x2[j], (int)(w >> 16), acc[r][3][j], false);
                }
            }
        }
    }

    // ---- epilogue: exact rescale in its cheapest form when every channel of the wave allows it
    // (see the comment at rescale_fused; here clamped before the final shift so that the shift
    // writes its byte into the packed dword), else the general form
    int32_t mu[4], cc[4], n1[4], lo[4], hi_[4], sf[4];
    bool fused_ok = true;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        mu[j] = g.mult[c0 + j], sf[j] = g.shift[c0 + j];
        const int32_t b = g.bias ? g.bias[c0 + j] : 0;
        fused_ok = fused_ok && sf[j] >= 1 && sf[j] <= 20 && b > -(1 << 28) && b < (1 << 28);
        const int nn = (sf[j] >= 1 && sf[j] <= 20) ? sf[j] : 1;
        n1[j] = nn + 1;
        cc[j] = 2 * ((1 << (nn - 1)) + (g.z_out << nn)) + 1;
        lo[j] = (g.lo_rel + g.z_out) << (nn + 1);
        hi_[j] = ((g.hi_rel + g.z_out + 1) << (nn + 1)) - 1;
    }
    const bool fused = __all(fused_ok);
    uint8_t *const out_img = g.y + (int64_t)n * g.Ho * g.Wo * g.C; // scalar
    const uint32_t out_off = (uint32_t)(wo0 * g.C + c0);            // inside an output row (Wo * C < 2^31)
    auto finish = [&](auto fused_tag) {
#pragma unroll
        for (int r = 0; r < RH; ++r) {
            if (ho0 + r >= g.Ho) break; // scalar
            uint8_t *out = out_img + (int64_t)(ho0 + r) * g.Wo * g.C; // scalar
#pragma unroll
            for (int p = 0; p < RW; ++p) {
                uint32_t packed = 0;
                if constexpr (decltype(fused_tag)::value > 0) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int32_t tt = __mulhi((int32_t)((uint32_t)acc[r][p][j] << 2), mu[j]);
                        const int32_t w = fused_w_from_t<decltype(fused_tag)::value == 1>(tt, cc[j]); // 2: without the tie term
                        packed = shift_into_byte(packed, med3_i32(w, lo[j], hi_[j]), n1[j], j);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int32_t y = clamp_i32(g.lo_rel, g.hi_rel, rescale_general(acc[r][p][j], make_rescale(mu[j], sf[j]))) + g.z_out;
                        packed |= (uint32_t)y << (8 * j);
                    }
                }
                if (wo0 + p < g.Wo) *reinterpret_cast<uint32_t *>(out + (out_off + (uint32_t)(p * g.C))) = packed;
            }
        }
    };
    if (!fused) finish(std::integral_constant<int, 0>{});
    else if (g.lo_rel < 0) finish(std::integral_constant<int, 1>{});
    else finish(std::integral_constant<int, 2>{}); // act_min >= z_out: the clamp absorbs the tie term
}

// any kernel size / stride / channel count: one lane per output element
__global__ void __launch_bounds__(256) dwconv_generic_kernel(const DwArgs g)
{
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= g.total_work) return;
    const int c = (int)(gid % g.C);
    int64_t t = gid / g.C;
    const int wo = (int)(t % g.Wo);
    t /= g.Wo;
    const int ho = (int)(t % g.Ho);
    const int n = (int)(t / g.Ho);
    int32_t acc = g.bias ? g.bias[c] : 0;
    const int32_t zw = g.zw ? g.zw[c] : 0;
    for (int a = 0; a < g.kh; ++a) {
        const int hi = ho * g.sh - g.ph + a;
        if (hi < 0 || hi >= g.H) continue;
        for (int b = 0; b < g.kw; ++b) {
            const int wi = wo * g.sw - g.pw + b;
            if (wi < 0 || wi >= g.W) continue;
            const int32_t xv = (int32_t)g.x[(((int64_t)n * g.H + hi) * g.W + wi) * g.C + c] - g.z_x;
            acc += xv * ((int32_t)g.w[((int64_t)a * g.kw + b) * g.C + c] - zw); // eq. 4 taken literally
        }
    }
    const RescaleParams rp = make_rescale(g.mult[c], g.shift[c]);
    g.y[gid] = (uint8_t)(clamp_i32(g.lo_rel, g.hi_rel, rescale_general(acc, rp)) + g.z_out);
}

} // namespace qnn

using namespace qnn;

static qnn_status qdwconv2d_impl(const uint8_t *x, int N, int H, int W, int C, int32_t z_x, const int8_t *w, int kh, int kw,
                                 int stride_h, int stride_w, int pad_h, int pad_w, const int32_t *bias, const int32_t *mult,
                                 const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *y,
                                 void *stream, const int32_t *z_w)
{
    if (!x || !w || !mult || !shift || !y) return QNN_EINVAL;
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || kh <= 0 || kw <= 0 || kh > 7 || kw > 7) return QNN_EINVAL;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return QNN_EINVAL;
    if (H + 2 * (int64_t)pad_h < kh || W + 2 * (int64_t)pad_w < kw) return QNN_EINVAL;
    if (z_x < 0 || z_x > 255 || bad_out_range(z_out, act_min, act_max)) return QNN_EINVAL;
    DwArgs g = {};
    g.x = x, g.w = w, g.y = y, g.bias = bias, g.mult = mult, g.shift = shift, g.zw = z_w;
    g.N = N, g.H = H, g.W = W, g.C = C, g.kh = kh, g.kw = kw;
    g.sh = stride_h, g.sw = stride_w, g.ph = pad_h, g.pw = pad_w;
    g.Ho = (H + 2 * pad_h - kh) / stride_h + 1;
    g.Wo = (W + 2 * pad_w - kw) / stride_w + 1;
    g.z_x = z_x, g.z_out = z_out, g.lo_rel = act_min - z_out, g.hi_rel = act_max - z_out;
    const hipStream_t s = as_stream(stream);
    auto al4 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3) == 0; };
    // (weight zero-points: the one-lane-per-output kernel, which evaluates the defining sum directly)
    const bool c4 = !z_w && (C % 4 == 0) && al4(x) && al4(w) && al4(y) && kh == 3 && kw == 3 && stride_h == stride_w &&
                    (stride_h == 1 || stride_h == 2);
    constexpr int RH = 2, RW = 4;
    if (c4) {
        g.wruns = (g.Wo + RW - 1) / RW;
        g.hruns = (g.Ho + RH - 1) / RH;
        g.total_work = (int64_t)N * g.hruns * g.wruns * (C / 4);
    } else {
        g.total_work = (int64_t)N * g.Ho * g.Wo * C;
    }
    const int64_t blocks = (g.total_work + 255) / 256;
    if (blocks > 0x7fffffff) return QNN_EINVAL;
    const bool old_form = tuning().dw_mad != 0; // tuning aid: the multiply-add form
    const int64_t lanes_x = (int64_t)g.wruns * (C / 4);
    const bool dot_ok = c4 && !old_form && N <= 65535 && g.hruns <= 65535 && lanes_x < (1ll << 31) - 256 &&
                        (int64_t)W * C < (1ll << 31) && (int64_t)g.Wo * C < (1ll << 31);
    if (dot_ok) {
        // division by the number of channel groups d >= 2 as multiply-high + shift: with
        // l = ceil(log2 d), m = ceil(2^(31+l) / d) < 2^32, x / d = (x * m) >> (31 + l) for x < 2^31
        const uint32_t d = (uint32_t)(C / 4);
        uint32_t l = 0;
        while ((1u << l) < d) ++l;
        g.shift_cgroups = l > 0 ? l - 1 : 0;
        g.magic_cgroups = d > 1 ? (uint32_t)((((uint64_t)1 << (31 + l)) + d - 1) / d) : 0u;
        // taller patches (4 output rows per lane) reuse more of the window, but need enough lanes to
        // give the chip something to do (tiny layers keep 2-row patches: twice the lanes)
        const int tall_env = tuning().dw_rh; // tuning aid: 2 or 4 forces the patch height
        const int64_t lanes_tall = lanes_x * ((g.Ho + 3) / 4) * N;
        const bool tall = tall_env ? tall_env == 4 : lanes_tall >= 16384;
        if (tall) g.hruns = (g.Ho + 3) / 4;
        const dim3 grid((unsigned)((lanes_x + 255) / 256), (unsigned)g.hruns, (unsigned)N);
        if (tall && stride_h == 1) hipLaunchKernelGGL((dwconv3x3_dot_kernel<1, 4>), grid, dim3(256), 0, s, g);
        else if (tall) hipLaunchKernelGGL((dwconv3x3_dot_kernel<2, 4>), grid, dim3(256), 0, s, g);
        else if (stride_h == 1) hipLaunchKernelGGL((dwconv3x3_dot_kernel<1, RH>), grid, dim3(256), 0, s, g);
        else hipLaunchKernelGGL((dwconv3x3_dot_kernel<2, RH>), grid, dim3(256), 0, s, g);
    } else if (c4 && stride_h == 1)
        hipLaunchKernelGGL((dwconv3x3_kernel<1, RH, RW>), dim3((unsigned)blocks), dim3(256), 0, s, g);
    else if (c4)
        hipLaunchKernelGGL((dwconv3x3_kernel<2, RH, RW>), dim3((unsigned)blocks), dim3(256), 0, s, g);
    else
        hipLaunchKernelGGL(dwconv_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s, g);
    return launch_status(hipGetLastError());
}

extern "C" qnn_status qnn_qdwconv2d(const uint8_t *x, int N, int H, int W, int C, int32_t z_x, const int8_t *w, int kh,
                                    int kw, int stride_h, int stride_w, int pad_h, int pad_w, const int32_t *bias,
                                    const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min,
                                    int32_t act_max, uint8_t *y, void *stream)
{
    return qdwconv2d_impl(x, N, H, W, C, z_x, w, kh, kw, stride_h, stride_w, pad_h, pad_w, bias, mult, shift, z_out, act_min,
                          act_max, y, stream, nullptr);
}

extern "C" qnn_status qnn_qdwconv2d_asym(const uint8_t *x, int N, int H, int W, int C, int32_t z_x, const int8_t *w, int kh,
                                         int kw, const int32_t *z_w, int stride_h, int stride_w, int pad_h, int pad_w,
                                         const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t z_out,
                                         int32_t act_min, int32_t act_max, uint8_t *y, void *stream)
{
    if (!z_w) return QNN_EINVAL;
    return qdwconv2d_impl(x, N, H, W, C, z_x, w, kh, kw, stride_h, stride_w, pad_h, pad_w, bias, mult, shift, z_out, act_min,
                          act_max, y, stream, z_w);
}
