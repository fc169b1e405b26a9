// Depthwise convolution (one kh x kw kernel per channel), NHWC uint8 -> NHWC uint8.
//
// 18 integer operations per output byte: the kernel is bound by HBM traffic and by the
// vector ALU, not by the matrix cores, so it does not use MFMA.  Channels are the
// contiguous axis: one lane owns 4 consecutive channels (one dword of activations, one
// dword of weights per tap) and a run of RW consecutive output pixels along W, so that the
// kh x (RW*stride + kw - stride) input window is loaded once and reused by all RW outputs;
// consecutive lanes own consecutive channel groups, which makes every load and store of a
// wave a contiguous run of channels.
//
//   acc[c] = sum_{a,b} (x[hi][wi][c] - z_x) * w[a][b][c]    taps outside the image skipped
//   out    = clamp(z_out + RESCALE(acc + bias[c]; mult[c], shift[c]))            (eq. 4-6, z_w = 0)
#include "qnn_device.h"

namespace qnn {

struct DwArgs {
    const uint8_t *x;
    const int8_t *w;
    uint8_t *y;
    const int32_t *bias, *mult, *shift;
    int N, H, W, C, Ho, Wo, kh, kw, sh, sw, ph, pw;
    int32_t z_x, z_out, lo_rel, hi_rel;
    int64_t total_work; // lanes of work
    int wruns;          // runs of RW output pixels per output row
};

__device__ __forceinline__ int32_t sbyte(uint32_t v, int j) { return (int32_t)(int8_t)(v >> (8 * j)); }
__device__ __forceinline__ int32_t ubyte(uint32_t v, int j) { return (int32_t)((v >> (8 * j)) & 0xffu); }

// KH x KW kernel, stride S (same in h and w), RW outputs per lane, 4 channels per lane
template <int KH, int KW, int S, int RW>
__global__ void __launch_bounds__(256) dwconv_c4_kernel(const DwArgs g)
{
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= g.total_work) return;
    const int cgroups = g.C >> 2;
    const int cg = (int)(gid % cgroups);
    int64_t t = gid / cgroups;
    const int run = (int)(t % g.wruns);
    t /= g.wruns;
    const int ho = (int)(t % g.Ho);
    const int n = (int)(t / g.Ho);
    const int c0 = cg * 4;
    const int wo0 = run * RW;

    // per-channel constants
    int32_t wt[KH][KW][4];
#pragma unroll
    for (int a = 0; a < KH; ++a)
#pragma unroll
        for (int b = 0; b < KW; ++b) {
            const uint32_t wv = *reinterpret_cast<const uint32_t *>(g.w + ((int64_t)a * KW + b) * g.C + c0);
#pragma unroll
            for (int j = 0; j < 4; ++j) wt[a][b][j] = sbyte(wv, j);
        }
    int32_t acc[RW][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int32_t b = g.bias ? g.bias[c0 + j] : 0;
#pragma unroll
        for (int p = 0; p < RW; ++p) acc[p][j] = b;
    }

    constexpr int COLS = (RW - 1) * S + KW;
    const int hi0 = ho * S - g.ph, wi0 = wo0 * S - g.pw;
    const uint8_t *img = g.x + (int64_t)n * g.H * g.W * g.C + c0;
#pragma unroll
    for (int a = 0; a < KH; ++a) {
        const int hi = hi0 + a;
        const bool row_ok = hi >= 0 && hi < g.H;
#pragma unroll
        for (int col = 0; col < COLS; ++col) {
            const int wi = wi0 + col;
            int32_t xv[4] = {0, 0, 0, 0}; // (x - z_x); a tap outside the image contributes 0
            if (row_ok && wi >= 0 && wi < g.W) {
                const uint32_t v = *reinterpret_cast<const uint32_t *>(img + ((int64_t)hi * g.W + wi) * g.C);
#pragma unroll
                for (int j = 0; j < 4; ++j) xv[j] = ubyte(v, j) - g.z_x;
            }
#pragma unroll
            for (int p = 0; p < RW; ++p) {
                const int b = col - p * S;
                if (b >= 0 && b < KW) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[p][j] += xv[j] * wt[a][b][j];
                }
            }
        }
    }

    RescaleParams rp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) rp[j] = make_rescale(g.mult[c0 + j], g.shift[c0 + j]);
    uint8_t *out = g.y + (((int64_t)n * g.Ho + ho) * g.Wo + wo0) * g.C + c0;
#pragma unroll
    for (int p = 0; p < RW; ++p) {
        if (wo0 + p >= g.Wo) break;
        uint32_t packed = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int32_t v = clamp_i32(g.lo_rel, g.hi_rel, rescale_general(acc[p][j], rp[j])) + g.z_out;
            packed |= (uint32_t)v << (8 * j);
        }
        *reinterpret_cast<uint32_t *>(out + (int64_t)p * g.C) = packed;
    }
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
    for (int a = 0; a < g.kh; ++a) {
        const int hi = ho * g.sh - g.ph + a;
        if (hi < 0 || hi >= g.H) continue;
        for (int b = 0; b < g.kw; ++b) {
            const int wi = wo * g.sw - g.pw + b;
            if (wi < 0 || wi >= g.W) continue;
            const int32_t xv = (int32_t)g.x[(((int64_t)n * g.H + hi) * g.W + wi) * g.C + c] - g.z_x;
            acc += xv * (int32_t)g.w[((int64_t)a * g.kw + b) * g.C + c];
        }
    }
    const RescaleParams rp = make_rescale(g.mult[c], g.shift[c]);
    g.y[gid] = (uint8_t)(clamp_i32(g.lo_rel, g.hi_rel, rescale_general(acc, rp)) + g.z_out);
}

} // namespace qnn

using namespace qnn;

extern "C" qnn_status qnn_qdwconv2d(const uint8_t *x, int N, int H, int W, int C, int32_t z_x, const int8_t *w, int kh,
                                    int kw, int stride_h, int stride_w, int pad_h, int pad_w, const int32_t *bias,
                                    const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min,
                                    int32_t act_max, uint8_t *y, void *stream)
{
    if (!x || !w || !mult || !shift || !y) return QNN_EINVAL;
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || kh <= 0 || kw <= 0 || kh > 7 || kw > 7) return QNN_EINVAL;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return QNN_EINVAL;
    if (H + 2 * (int64_t)pad_h < kh || W + 2 * (int64_t)pad_w < kw) return QNN_EINVAL;
    if (z_x < 0 || z_x > 255 || bad_out_range(z_out, act_min, act_max)) return QNN_EINVAL;
    DwArgs g = {};
    g.x = x, g.w = w, g.y = y, g.bias = bias, g.mult = mult, g.shift = shift;
    g.N = N, g.H = H, g.W = W, g.C = C, g.kh = kh, g.kw = kw;
    g.sh = stride_h, g.sw = stride_w, g.ph = pad_h, g.pw = pad_w;
    g.Ho = (H + 2 * pad_h - kh) / stride_h + 1;
    g.Wo = (W + 2 * pad_w - kw) / stride_w + 1;
    g.z_x = z_x, g.z_out = z_out, g.lo_rel = act_min - z_out, g.hi_rel = act_max - z_out;
    const hipStream_t s = as_stream(stream);
    auto al4 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3) == 0; };
    const bool c4 = (C % 4 == 0) && al4(x) && al4(w) && al4(y) && kh == 3 && kw == 3 && stride_h == stride_w &&
                    (stride_h == 1 || stride_h == 2);
    constexpr int RW = 4;
    if (c4) {
        g.wruns = (g.Wo + RW - 1) / RW;
        g.total_work = (int64_t)N * g.Ho * g.wruns * (C / 4);
    } else {
        g.total_work = (int64_t)N * g.Ho * g.Wo * C;
    }
    const int64_t blocks = (g.total_work + 255) / 256;
    if (blocks > 0x7fffffff) return QNN_EINVAL;
    if (c4 && stride_h == 1)
        hipLaunchKernelGGL((dwconv_c4_kernel<3, 3, 1, RW>), dim3((unsigned)blocks), dim3(256), 0, s, g);
    else if (c4)
        hipLaunchKernelGGL((dwconv_c4_kernel<3, 3, 2, RW>), dim3((unsigned)blocks), dim3(256), 0, s, g);
    else
        hipLaunchKernelGGL(dwconv_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s, g);
    return launch_status(hipGetLastError());
}
