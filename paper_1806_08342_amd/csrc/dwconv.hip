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
    int xcd_remap;      // renumber the workgroups (see xcd_neighbours)
};

// The hardware deals workgroups to the 8 XCDs (each with a private L2) round-robin by linear
// id, so spatial neighbours -- which re-read each other's halo rows and columns -- end up behind
// eight different L2s and every halo byte is fetched from the fabric twice.  This renumbering
// gives XCD k the k-th contiguous eighth of the (x fastest, then y, then z) order instead:
// workgroup lin runs on XCD lin % 8 as its (lin / 8)-th, and takes the place
// k * (total / 8) + min(k, total % 8) + lin / 8, a bijection of 0 .. total - 1.
__device__ __forceinline__ void xcd_neighbours(bool on, uint32_t &bx, uint32_t &by, uint32_t &bz)
{
    bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    if (!on) return;
    const uint32_t gx = gridDim.x, gy = gridDim.y;
    const uint32_t total = gx * gy * gridDim.z; // the dispatcher keeps this below 2^31
    const uint32_t lin = bx + gx * (by + gy * bz);
    const uint32_t xcd = lin & 7u, per = total >> 3, rem = total & 7u;
    const uint32_t id = xcd * per + (xcd < rem ? xcd : rem) + (lin >> 3);
    const uint32_t t = id / gx;
    bx = id - t * gx;
    bz = t / gy;
    by = t - bz * gy;
}

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
    uint32_t bx, by, bz;
    xcd_neighbours(g.xcd_remap != 0, bx, by, bz);
    const uint32_t lane_x = bx * 256u + threadIdx.x;
    const uint32_t cgroups = (uint32_t)g.C >> 2;
    const uint32_t pw = cgroups == 1 ? lane_x : __umulhi(lane_x, g.magic_cgroups) >> g.shift_cgroups; // lane_x / cgroups
    const uint32_t cg = lane_x - pw * cgroups;
    if (pw >= (uint32_t)g.wruns) return;
    const int n = (int)bz, ph = (int)by; // wave-uniform
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

// Depthwise 3x3 with the multiplies on the matrix unit.
//
// The layer moves 2-5 bytes per output, and on the vector ALU it costs about 16 instructions per
// output byte (the dot products need pixels in the bytes of a dword while NHWC puts channels there,
// so every input byte goes through byte permutes first): the vector ALU, not HBM, sets the pace.
// v_mfma_i32_32x32x32_i8 takes the transposition away.  For a block of 32 channels and one kernel tap,
//   D[pixel][c] += sum_c' A[pixel][c'] * B[c'][c],   B[c'][c] = w[tap][c] if c' == c else 0
// is that tap's contribution to 32 pixels x 32 channels.  A's fragment is what NHWC memory holds:
// lane (pixel, half) takes the 16 contiguous channel bytes of its pixel -- no byte shuffling at all;
// B's fragment is a diagonal matrix built once per wave from the weights.  The unit runs at 1/32
// of its density and that is fine: nine of these instructions per output row of a wave take fewer
// issue cycles than the rescale of the same outputs, and they run beside it.  The layer stays
// HBM-bound and is graded against HBM; the matrix unit only replaces the byte transposition.
//
// A wave owns TP = 30 output pixels of one image row x 32 channels and walks down a segment of output
// rows.  Its input rows -- 32 pixels (stride 1) or 64 pixels (stride 2) x 32 channel bytes, one or
// two 1 KB copies -- go straight from global memory into a ring of LDS rows that belongs to the wave
// alone (global_load_lds_dwordx4, RING - 1 rows ahead of the row in use; no barrier anywhere: waves
// share nothing).  A row is read back three times as fragments (window columns 0, 1, 2 = the same
// pixels shifted by one); it is kernel row 0, 1 and 2 of three consecutive output rows (stride 1;
// stride 2: two rows per output row, the odd one shared), whose accumulators form a ring of their
// own.  An output row that has received its last kernel row is rescaled (all 16 values of a lane
// belong to ONE channel, so the constants are per lane), its bytes are transposed across the four
// lanes of a quad into NHWC order and stored.  acc starts at bias + (128 - z_x) * sum(w); codes are
// offset by 128 (xor) to be signed; taps outside the image hold the code z_x.
//
// vmcnt bookkeeping: every wave issues exactly DPW copies per input row, rows
// past the end of the segment repeat the last one, "at most (RING - 2) x DPW outstanding" means
// the oldest row has landed, and the output stores can only make that wait stricter.
// (Measured: a wait that also allows for the stores issued since -- possible in the steady state, where their
// number is known -- and even no wait at all leave the time of a launch unchanged.)
using dw_i32x4 = int32_t __attribute__((ext_vector_type(4)));
using dw_i32x16 = int32_t __attribute__((ext_vector_type(16)));

template <int S, int MODE>
__global__ void __launch_bounds__(256, 2) dwconv3x3_mfma_kernel(const DwArgs g, const int seg_rows, const int tiles_w,
                                                                const int cblocks)
{
    constexpr int SLOTS = S == 1 ? 3 : 2, TP = 30, DPW = S, ROW_BYTES = DPW * 1024, RING = S == 1 ? 12 : 8, D = RING - 1;
    __shared__ __attribute__((aligned(16))) uint8_t lds[4 * RING * ROW_BYTES];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    uint32_t bx, by, bz;
    xcd_neighbours(g.xcd_remap != 0, bx, by, bz);
    const int wave_lin = (int)bx * 4 + wave; // scalar
    const int tile_w = wave_lin / cblocks, cblk = wave_lin - tile_w * cblocks;
    if (tile_w >= tiles_w) return; // whole wave; waves share nothing
    uint8_t *const ring = lds + wave * (RING * ROW_BYTES);
    const int n = (int)bz;
    const int hb = (int)by * seg_rows;
    const int rows = (g.Ho - hb) < seg_rows ? (g.Ho - hb) : seg_rows;
    const int li = lane & 31, half = lane >> 5;
    const int w0 = tile_w * TP;

    // ---- input rows: copy j of a row moves, per lane, 16 channel bytes of pixel wi0 + (j * 64 + lane) / 2
    // (clamped into the image row; pixels outside are replaced after the read-back) to LDS offset
    // (j * 64 + lane) * 16, i.e. an LDS row is [pixel][32 channel bytes]
    const int wi0 = w0 * S - g.pw;
    const int64_t row_bytes = (int64_t)g.W * g.C;
    const uint8_t *img = g.x + (int64_t)n * g.H * row_bytes;    // scalar
    uint32_t src_off[DPW];
#pragma unroll
    for (int j = 0; j < DPW; ++j) {
        int wi = wi0 + ((j * 64 + lane) >> 1);
        wi = wi < 0 ? 0 : (wi >= g.W ? g.W - 1 : wi);
        int c16 = cblk * 32 + 16 * (lane & 1);
        c16 = c16 + 16 <= g.C ? c16 : g.C - 16; // blocks that stick out of C: any valid bytes (B is zero there)
        src_off[j] = (uint32_t)(wi * g.C + c16);
    }
    // ---- the row pipeline: input row t of the segment is image row hi_first + t, t = 0 .. steps - 1
    const int hi_first = hb * S - g.ph;
    const int steps = S == 1 ? rows + 2 : 2 * rows + 1;
    int issue_t = 0, issue_slot = 0; // next row to copy and the ring row it goes to (scalar)
    int read_t = 0, read_slot = 0;   // next row to consume
    auto issue_row = [&]() __attribute__((always_inline)) {
        const int t = issue_t < steps ? issue_t : steps - 1; // past the end: repeat the last row (nobody reads that ring row)
        int hi = hi_first + t;
        hi = hi < 0 ? 0 : (hi >= g.H ? g.H - 1 : hi);        // rows outside the image: any row inside (replaced by the padding code)
        const uint8_t *line = img + (int64_t)hi * row_bytes;
        uint8_t *dst = ring + issue_slot * ROW_BYTES;
#pragma unroll
        for (int j = 0; j < DPW; ++j)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(line + src_off[j]),
                                             (__attribute__((address_space(3))) void *)(dst + j * 1024), 16, 0, 0);
        ++issue_t;
        issue_slot = issue_slot + 1 == RING ? 0 : issue_slot + 1;
    };
    for (int d = 0; d < D; ++d) issue_row(); // D rows in flight before anything else: their latency covers the set-up below

    // ---- B fragments: the diagonal of tap (a, b) for the channels of this block.  Lane (column li, half)
    // holds rows k = 16 half .. 16 half + 15 of column li: only row k = li is non-zero.
    const int ch = cblk * 32 + li;                  // the channel this lane accumulates and rescales
    const bool ch_ok = ch < g.C;
    const bool diag_here = ch_ok && (li >> 4) == half;
    dw_i32x4 wq[3][3];
    int32_t wsum = 0;
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            const int32_t w = ch_ok ? (int32_t)g.w[(a * 3 + b) * g.C + ch] : 0;
            wsum += w;
            const uint32_t placed = diag_here ? ((uint32_t)(w & 0xff) << (8 * (li & 3))) : 0u;
            const int d = (li >> 2) & 3;
            wq[a][b] = dw_i32x4{d == 0 ? (int32_t)placed : 0, d == 1 ? (int32_t)placed : 0, d == 2 ? (int32_t)placed : 0,
                                d == 3 ? (int32_t)placed : 0};
        }
    const int32_t bias = (ch_ok && g.bias) ? g.bias[ch] : 0;
    const int32_t init = bias + (128 - g.z_x) * wsum;

    // ---- epilogue constants of this lane's channel (see rescale_fused_w)
    const int32_t mu = ch_ok ? g.mult[ch] : 0, sf = ch_ok ? g.shift[ch] : 1;
    const bool fused_ok = sf >= 1 && sf <= 20 && bias > -(1 << 28) && bias < (1 << 28);
    const int nn = (sf >= 1 && sf <= 20) ? sf : 1;
    const int32_t n1 = nn + 1;
    const int32_t cc = 2 * ((1 << (nn - 1)) + (g.z_out << nn)) + 1;
    const int32_t lo = (g.lo_rel + g.z_out) << (nn + 1);
    const int32_t hi_ = ((g.hi_rel + g.z_out + 1) << (nn + 1)) - 1;
    const bool fused = MODE != 0 && __all(fused_ok); // wave-uniform

    // read-back of window column b: pixel li * S + b of the LDS row, 16 channel bytes of this lane's half
    uint32_t l_off[3];
    bool a_ok[3], all_ok = true;
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        const int wi = wi0 + li * S + b;
        a_ok[b] = wi >= 0 && wi < g.W;
        all_ok = all_ok && a_ok[b];
        const int lp = li < TP ? li : TP - 1; // lanes 30, 31 own no output pixel: they re-read the last one, inside the row
        l_off[b] = (uint32_t)((lp * S + b) * 32 + 16 * half);
    }
    const bool wave_interior = __all(all_ok);
    const int32_t fill_s = (int32_t)(((uint32_t)g.z_x * 0x01010101u) ^ 0x80808080u);

    // ---- output addressing: after the quad transposition lane (li, half) stores, for q = 0..3, the 4 channels
    // (li & ~3) .. + 3 of pixel w0 + 8q + 4 half + (li & 3)
    const int quad_lane = li & 3;
    const uint32_t sel1 = (quad_lane & 1) ? 0x03070105u : 0x06020400u;
    const uint32_t sel2 = (quad_lane & 2) ? 0x03020706u : 0x05040100u;
    const int64_t out_row_bytes = (int64_t)g.Wo * g.C;
    int64_t out_row = ((int64_t)n * g.Ho + hb) * out_row_bytes; // scalar: byte offset of the output row that finishes next
    const int out_c = cblk * 32 + (li & ~3);
    uint32_t o_off[4];
    bool o_ok[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int p = 8 * q + 4 * half + quad_lane; // pixel of the tile
        const int wo = w0 + p;
        o_ok[q] = p < TP && wo < g.Wo && out_c < g.C;
        o_off[q] = (uint32_t)((o_ok[q] ? wo : 0) * g.C + (out_c < g.C ? out_c : 0));
    }

    // accumulators start at zero (an inline constant of the matrix instruction); bias and zero-point term join in
    // the rescale, inside the add-and-shift that the 32-bit form needs anyway
    dw_i32x16 acc[SLOTS];
    auto reset = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[slot][r] = 0;
    };
    auto finish = [&](int slot) __attribute__((always_inline)) {
        // wave-uniform row base (scalar registers) + 32-bit lane offsets
        const int64_t row_off = ((int64_t)__builtin_amdgcn_readfirstlane((int)(out_row >> 32)) << 32) |
                                (uint32_t)__builtin_amdgcn_readfirstlane((int)out_row);
        uint8_t *out = g.y + row_off;
        uint32_t x[4];
        if (fused) { // one test per output row; the general form below is the rare case
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                x[q] = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int32_t tt = __mulhi((int32_t)(((uint32_t)acc[slot][4 * q + e] + (uint32_t)init) << 2), mu);
                    x[q] = shift_into_byte(x[q], med3_i32(fused_w_from_t<MODE == 1>(tt, cc), lo, hi_), n1, e);
                }
            }
        } else {
            const RescaleParams rp = make_rescale(mu, sf);
#pragma nounroll
            for (int q = 0; q < 4; ++q) {
                x[q] = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int32_t y = clamp_i32(g.lo_rel, g.hi_rel, rescale_general(acc[slot][4 * q + e] + init, rp)) + g.z_out;
                    x[q] |= (uint32_t)y << (8 * e);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // 4 pixels of one channel -> 4 channels of one pixel, across the quad (two exchanges + byte permutes)
            uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)x[q], 0xB1, 0xF, 0xF, true);
            uint32_t v = __builtin_amdgcn_perm(o, x[q], sel1);
            o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);
            v = __builtin_amdgcn_perm(o, v, sel2);
            if (o_ok[q]) *reinterpret_cast<uint32_t *>(out + o_off[q]) = v;
        }
        out_row += out_row_bytes;
    };

    dw_i32x4 fa[3], fn[3];
    // requests the LDS read-back of input row read_t into fn (after its copy has landed) and the copy of row read_t + D
    auto fetch_row = [&]() __attribute__((always_inline)) {
        constexpr int N = (D - 1) * DPW;
        __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8)); // vmcnt only
        asm volatile("" ::: "memory");
        const uint8_t *src = ring + read_slot * ROW_BYTES;
#pragma unroll
        for (int b = 0; b < 3; ++b) fn[b] = *reinterpret_cast<const dw_i32x4 *>(src + l_off[b]);
        asm volatile("" ::: "memory");
        issue_row(); // into the ring row that was consumed one step ago
    };
    // fn (raw codes of row read_t) -> fa (signed, padding replaced)
    auto take_row = [&]() __attribute__((always_inline)) {
        const int hi = hi_first + read_t;
        const bool row_ok = hi >= 0 && hi < g.H; // scalar
        if (!row_ok) {
#pragma unroll
            for (int b = 0; b < 3; ++b) fa[b] = dw_i32x4{fill_s, fill_s, fill_s, fill_s};
        } else if (wave_interior) { // the common case: twelve xors
#pragma unroll
            for (int b = 0; b < 3; ++b) fa[b] = fn[b] ^ (int32_t)0x80808080; // signed (code - 128)
        } else {
#pragma unroll
            for (int b = 0; b < 3; ++b) {
                const dw_i32x4 t = fn[b] ^ (int32_t)0x80808080;
                const bool ok = a_ok[b];
                fa[b] = dw_i32x4{ok ? t.x : fill_s, ok ? t.y : fill_s, ok ? t.z : fill_s, ok ? t.w : fill_s};
            }
        }
        ++read_t;
        read_slot = read_slot + 1 == RING ? 0 : read_slot + 1;
    };
    // one window column of the current row into one accumulator set (the caller interleaves the sets, so that
    // consecutive matrix instructions do not depend on each other)
    auto mac1 = [&](int a, int b, int slot) __attribute__((always_inline)) {
        acc[slot] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[b], wq[a][b], acc[slot], 0, 0, 0);
    };

    // Steady state of the row pipeline, free of run-time conditions: every output row involved exists and every
    // input row lies inside the image, so a step is LDS read-back, sign flip (EDGE: plus the padding selects of
    // the window columns that stick out of the image), nine matrix instructions -- the first one of a new output
    // row takes the constant zero as its accumulator input, which replaces the reset -- and one rescale.
    const dw_i32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    auto take_inside = [&](auto edge) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            const dw_i32x4 t = fn[b] ^ (int32_t)0x80808080;
            if constexpr (decltype(edge)::value) {
                const bool ok = a_ok[b];
                fa[b] = dw_i32x4{ok ? t.x : fill_s, ok ? t.y : fill_s, ok ? t.z : fill_s, ok ? t.w : fill_s};
            } else {
                fa[b] = t;
            }
        }
        ++read_t;
        read_slot = read_slot + 1 == RING ? 0 : read_slot + 1;
    };
    auto mac0 = [&](int b, int slot) __attribute__((always_inline)) { // kernel row 0: window column 0 opens the accumulator set
        acc[slot] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[b], wq[0][b], b == 0 ? zero16 : acc[slot], 0, 0, 0);
    };

    if constexpr (S == 1) {
        // row t is kernel row 0 of output k = t, kernel row 1 of k = t - 1, kernel row 2 of k = t - 2; output k lives
        // in accumulator set k % 3
        auto steady3 = [&](auto edge) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                fetch_row();
                take_inside(edge);
#pragma unroll
                for (int b = 0; b < 3; ++b) {
                    mac1(2, b, (u + 1) % 3);
                    mac1(1, b, (u + 2) % 3);
                    mac0(b, u);
                }
                finish((u + 1) % 3);
            }
        };
        for (int t0 = 0; t0 < steps; t0 += 3) {
            // rows t0 .. t0 + 2: all three outputs of every step exist and all three input rows are inside the image
            if (t0 >= 2 && t0 + 2 < rows && hi_first + t0 >= 0 && hi_first + t0 + 2 < g.H) { // scalar
                if (wave_interior) steady3(std::false_type{});
                else steady3(std::true_type{});
                continue;
            }
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const int t = t0 + u;
                if (t >= steps) break; // scalar
                fetch_row();
                take_row();
                const bool has0 = t < rows, has1 = t >= 1 && t - 1 < rows, has2 = t >= 2; // scalar
                if (has0) reset(u);
#pragma unroll
                for (int b = 0; b < 3; ++b) {
                    if (has2) mac1(2, b, (u + 1) % 3);
                    if (has1) mac1(1, b, (u + 2) % 3);
                    if (has0) mac1(0, b, u);
                }
                if (has2) finish((u + 1) % 3);
            }
        }
    } else {
        // output k uses rows 2k, 2k + 1, 2k + 2 of the segment; row 2k + 2 is also the first row of output k + 1;
        // output k lives in accumulator set k % 2
        fetch_row();
        take_row();
        reset(0);
#pragma unroll
        for (int b = 0; b < 3; ++b) mac1(0, b, 0);
        auto steady2 = [&](auto edge) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                fetch_row();
                take_inside(edge);
#pragma unroll
                for (int b = 0; b < 3; ++b) mac1(1, b, u);
                fetch_row();
                take_inside(edge);
#pragma unroll
                for (int b = 0; b < 3; ++b) {
                    mac1(2, b, u);
                    mac0(b, u ^ 1);
                }
                finish(u);
            }
        };
        for (int k0 = 0; k0 < rows; k0 += 2) {
            // outputs k0, k0 + 1 and k0 + 2 exist and input rows 2 k0 + 1 .. 2 k0 + 4 are inside the image
            if (k0 + 2 < rows && hi_first + 2 * k0 + 1 >= 0 && hi_first + 2 * k0 + 4 < g.H) { // scalar
                if (wave_interior) steady2(std::false_type{});
                else steady2(std::true_type{});
                continue;
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int k = k0 + u;
                if (k >= rows) break; // scalar
                fetch_row();
                take_row();
#pragma unroll
                for (int b = 0; b < 3; ++b) mac1(1, b, u);
                fetch_row();
                take_row();
                const bool more = k + 1 < rows; // scalar
                if (more) reset(u ^ 1);
#pragma unroll
                for (int b = 0; b < 3; ++b) {
                    mac1(2, b, u);
                    if (more) mac1(0, b, u ^ 1);
                }
                finish(u);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8)); // vmcnt(0): no copy may land in LDS after the wave is gone
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
    if (N < 0 || H <= 0 || W <= 0 || C <= 0 || kh <= 0 || kw <= 0 || kh > 7 || kw > 7) return QNN_EINVAL;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return QNN_EINVAL;
    if (H + 2 * (int64_t)pad_h < kh || W + 2 * (int64_t)pad_w < kw) return QNN_EINVAL;
    if (z_x < 0 || z_x > 255 || bad_out_range(z_out, act_min, act_max)) return QNN_EINVAL;
    if (N == 0) return QNN_OK; // an empty batch: nothing to compute, no pointer is looked at
    if (!x || !w || !mult || !shift || !y) return QNN_EINVAL;
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
        const int variant = tuning().dw_variant; // tuning aid: 0 = patch kernel, 3 = matrix-unit kernel, -1 = by shape
        // matrix-unit kernel: whole 16-byte channel chunks, rows of at least 24 outputs (narrower images waste
        // most of the 32-pixel tile and stay with the patch kernel)
        if ((variant == 3 || variant < 0) && (C % 16) == 0 && (reinterpret_cast<uintptr_t>(x) % 16) == 0 &&
            (int64_t)H * W * C < (1ll << 31) && (int64_t)g.Ho * g.Wo * C < (1ll << 31) &&
            // measured: ahead of the patch kernel on stride-2 layers from 56 x 56 inputs up (+15 % at 112 x 112 and
            // at 56 x 56), by 5 % on stride-1 layers at least 48 pixels wide, and once a launch has more than ~10^8 outputs
            // (+25 %: 0.40 against 0.32 of HBM); behind it on the small layers, whose image rows fill less than
            // half of the 30-pixel tile
            // (and never below 2^21 outputs: a few dozen waves walking their segments row by row take longer than the
            // patch kernel's thousands of independent lanes -- 9 against 4 us on one 112 x 112 x 32 image)
            (variant == 3 ||
             ((int64_t)N * g.Ho * g.Wo * C >= (1ll << 21) && ((stride_h == 2 && g.Wo >= 24) || (stride_h == 1 && g.Wo >= 48))) ||
             (int64_t)N * g.Ho * g.Wo * C >= (100ll << 20))) {
            const int tiles_w = (g.Wo + 29) / 30, cblocks = (C + 31) / 32; // 30 output pixels per wave
            const int64_t waves_x = (int64_t)tiles_w * cblocks;
            int seg_rows = tuning().dw_rh > 0 ? tuning().dw_rh : 0;
            if (seg_rows <= 0) {
                const int64_t target = 2048; // waves: 2 per SIMD of the chip
                int64_t segs = (target + waves_x * N - 1) / (waves_x * N);
                const int64_t most = (g.Ho + 7) / 8; // at least 8 output rows per segment (each re-reads 2 input rows)
                segs = segs < 1 ? 1 : (segs > most ? most : segs);
                seg_rows = (int)((g.Ho + segs - 1) / segs);
            }
            if (seg_rows > g.Ho) seg_rows = g.Ho;
            const int segs = (g.Ho + seg_rows - 1) / seg_rows;
            const dim3 grid((unsigned)((waves_x + 3) / 4), (unsigned)segs, (unsigned)N);
            g.xcd_remap = tuning().dw_xcd != 0 && (int64_t)grid.x * grid.y * grid.z < (1ll << 31);
            const int mode = g.lo_rel >= 0 ? 2 : 1;
            if (stride_h == 1 && mode == 2) hipLaunchKernelGGL((dwconv3x3_mfma_kernel<1, 2>), grid, dim3(256), 0, s, g, seg_rows, tiles_w, cblocks);
            else if (stride_h == 1) hipLaunchKernelGGL((dwconv3x3_mfma_kernel<1, 1>), grid, dim3(256), 0, s, g, seg_rows, tiles_w, cblocks);
            else if (mode == 2) hipLaunchKernelGGL((dwconv3x3_mfma_kernel<2, 2>), grid, dim3(256), 0, s, g, seg_rows, tiles_w, cblocks);
            else hipLaunchKernelGGL((dwconv3x3_mfma_kernel<2, 1>), grid, dim3(256), 0, s, g, seg_rows, tiles_w, cblocks);
            return launch_status(hipGetLastError());
        }
        // taller patches (4 output rows per lane) reuse more of the window, but need enough lanes to
        // give the chip something to do (tiny layers keep 2-row patches: twice the lanes)
        const int tall_env = tuning().dw_rh; // tuning aid: 2 or 4 forces the patch height
        const int64_t lanes_tall = lanes_x * ((g.Ho + 3) / 4) * N;
        const bool tall = tall_env ? tall_env == 4 : lanes_tall >= 16384;
        if (tall) g.hruns = (g.Ho + 3) / 4;
        const dim3 grid((unsigned)((lanes_x + 255) / 256), (unsigned)g.hruns, (unsigned)N);
        g.xcd_remap = tuning().dw_xcd != 0 && (int64_t)grid.x * grid.y * grid.z < (1ll << 31);
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
