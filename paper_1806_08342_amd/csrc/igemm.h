// Implicit-GEMM kernel for the dense quantized layers (GEMM / fully connected, 1x1, 3x3, 7x7
// convolutions) on gfx950 int8 MFMA.
//
//   acc[m][n] = sum_k xs[m][k] * w[k][n],  xs = x - 128 (the MFMA int8 operands are signed)
//   a         = acc + bias[n] + (128 - z_x) * sum_k w[k][n]          (eq. 5-6 with z_w = 0)
//   out       = clamp(z_out + RESCALE(a))
//
// m runs over output pixels (n, ho, wo) and k over (kh, kw, ci), gathered on the fly from
// the NHWC image; taps outside the image are filled with the code z_x, so the single
// column-sum correction is valid at the border too.  The weight column sums are formed
// from the B fragments while they stream through the registers (v_dot4 with a vector of
// ones), not in a separate pass.
//
// Tile: BM x BN outputs per workgroup, K in steps of 64; WM x WN waves, each owning a
// (BM/WM) x (BN/WN) sub-tile built from 32x32x32 MFMAs.  Both operands are staged in LDS as
// rows of 64 bytes whose four 16-byte chunks are XOR-swizzled with the row index, so that
// the 16-byte fragment reads of 32 consecutive rows and the 16-byte staging writes are both
// bank-conflict free.
#pragma once

#include <type_traits>

#include "qnn_device.h"

namespace qnn {

using i32x4 = int32_t __attribute__((ext_vector_type(4)));
using i32x16 = int32_t __attribute__((ext_vector_type(16)));
using u32x4 = uint32_t __attribute__((ext_vector_type(4)));
using u32x2 = uint32_t __attribute__((ext_vector_type(2)));

enum { A_MATRIX = 0, A_CONV = 1 };
enum { B_INT8 = 0, B_INT4 = 1, B_INT8_ROWS = 2 };

struct IgemmArgs {
    const uint8_t *A;
    int64_t lda; // A_MATRIX: row pitch
    // A_CONV geometry
    int H, W, Cin, Ho, Wo, kw, sh, sw, ph, pw;
    uint32_t magic_cin, magic_kw; // ceil(2^32 / d): floor(k / d) = mulhi(k, magic) for k < 2^16
    const uint8_t *B;
    int64_t ldb; // elements
    int64_t M;
    int32_t N, K;
    int32_t z_a;
    const int32_t *bias, *mult, *shift;
    int32_t z_out, lo_rel, hi_rel; // clamp range relative to z_out
    uint8_t *C;
    int64_t ldc;
    int32_t c_vec16;  // C and ldc are 16-byte aligned
    int32_t small_acc; // 2: |acc| and the zero-point correction are each below 2^27; 1: below 2^28; 0: unknown
    // optional per-column weight zero-points (eq. 5-6 with z_w != 0): zw[n] and the row sums
    // rowsum[m] = sum_k (A[m][k] - z_a) over the taps inside the image (both int32, device); nullptr: z_w = 0
    const int32_t *zw, *rowsum;
    // optional rescaling add behind the product: C = ADD(code of the product, R); R == nullptr: none
    const uint8_t *R;
    int64_t ldr;
    int32_t r_vec16; // R and ldr are 16-byte aligned
    AddParams add;
};

__device__ __forceinline__ uint32_t fast_div(uint32_t k, uint32_t d, uint32_t magic)
{
    return d == 1 ? k : __umulhi(k, magic);
}

// XOR swizzle of the four 16-byte chunks of a 64-byte tile row.  A 16-byte LDS read serves the
// 64 lanes in four cycles of 16 lanes, 256 bytes (64 banks) each, and the lanes that share a
// cycle are {0-3, 12-15, 20-23, 24-27}, {4-11, 16-19, 28-31} and the same sets + 32 (measured).
// A fragment read has lane = tile row (mod 32): within one such set row / 4 takes four values
// whose low two bits differ, so XOR-ing the chunk index with (row / 4) % 4 gives every lane of
// a cycle its own 16-byte bank group.
__device__ __forceinline__ int lds_swizzle(int row) { return (row >> 2) & 3; }

// swizzled byte offset of 16-byte chunk c (0..3) of a 64-byte tile row
__device__ __forceinline__ int lds_chunk_offset(int row, int c)
{
    return row * 64 + (((c ^ lds_swizzle(row)) & 3) << 4);
}

template <int VEC> struct PieceLoader;
template <> struct PieceLoader<16> {
    static __device__ __forceinline__ void load(const uint8_t *p, uint32_t *w, int piece)
    {
        (void)piece;
        u32x4 v = *reinterpret_cast<const u32x4 *>(p);
        w[0] = v.x, w[1] = v.y, w[2] = v.z, w[3] = v.w;
    }
};
template <> struct PieceLoader<8> {
    static __device__ __forceinline__ void load(const uint8_t *p, uint32_t *w, int piece)
    {
        u32x2 v = *reinterpret_cast<const u32x2 *>(p);
        w[2 * piece] = v.x, w[2 * piece + 1] = v.y;
    }
};
template <> struct PieceLoader<4> {
    static __device__ __forceinline__ void load(const uint8_t *p, uint32_t *w, int piece)
    {
        w[piece] = *reinterpret_cast<const uint32_t *>(p);
    }
};
template <> struct PieceLoader<1> {
    static __device__ __forceinline__ void load(const uint8_t *p, uint32_t *w, int piece)
    {
        const int sh = (piece & 3) * 8;
        w[piece >> 2] = (w[piece >> 2] & ~(0xffu << sh)) | ((uint32_t)(*p) << sh);
    }
};

struct ARow {
    const uint8_t *base; // A_MATRIX: row start; A_CONV: image start
    int hi0, wi0;
    bool valid;
};

// 16 consecutive k (one chunk) of one A row, as 4 dwords of uint8 codes
template <int A_MODE, int VEC>
__device__ __forceinline__ void load_a_chunk(const IgemmArgs &g, const ARow &r, int kc, uint32_t fill, uint32_t *w)
{
    w[0] = w[1] = w[2] = w[3] = fill;
    if (!r.valid) return;
#pragma unroll
    for (int p = 0; p < 16 / VEC; ++p) {
        const int k = kc + p * VEC;
        if (k >= g.K) break;
        if constexpr (A_MODE == A_MATRIX) {
            PieceLoader<VEC>::load(r.base + k, w, p);
        } else {
            const uint32_t tap = fast_div((uint32_t)k, (uint32_t)g.Cin, g.magic_cin);
            const int ci = k - (int)tap * g.Cin;
            const uint32_t ta = fast_div(tap, (uint32_t)g.kw, g.magic_kw);
            const int tb = (int)tap - (int)ta * g.kw;
            const int hi = r.hi0 + (int)ta, wi = r.wi0 + tb;
            if (hi >= 0 && hi < g.H && wi >= 0 && wi < g.W)
                PieceLoader<VEC>::load(r.base + ((int64_t)hi * g.W + wi) * g.Cin + ci, w, p);
            // else: stays at the fill code z_x
        }
    }
}

// 16 consecutive k of one B column as 4 dwords of int8 (B_INT4: the values times 16)
template <int B_MODE, int VEC>
__device__ __forceinline__ void load_b_chunk(const IgemmArgs &g, int n, int kc, uint32_t *w)
{
    w[0] = w[1] = w[2] = w[3] = 0u;
    if (n >= g.N) return;
    if constexpr (B_MODE == B_INT8) {
        const uint8_t *col = g.B + (int64_t)n * g.ldb;
#pragma unroll
        for (int p = 0; p < 16 / VEC; ++p) {
            const int k = kc + p * VEC;
            if (k >= g.K) break;
            PieceLoader<VEC>::load(col + k, w, p);
        }
    } else if constexpr (B_MODE == B_INT8_ROWS) {
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int k = kc + p;
            if (k >= g.K) break;
            PieceLoader<1>::load(g.B + (int64_t)k * g.ldb + n, w, p);
        }
    } else { // nibble pairs, element 2j in the low nibble of byte j
        const uint8_t *col = g.B + (((int64_t)n * g.ldb) >> 1);
        if constexpr (VEC >= 8) {
            uint32_t raw[4] = {0u, 0u, 0u, 0u}; // VEC elements = VEC/2 bytes per piece
#pragma unroll
            for (int p = 0; p < 16 / VEC; ++p) {
                const int k = kc + p * VEC;
                if (k >= g.K) break;
                PieceLoader<VEC / 2>::load(col + (k >> 1), raw, p);
            }
#pragma unroll
            for (int d = 0; d < 2; ++d) { // raw[d] holds elements 8d .. 8d+7
                const uint32_t even = (raw[d] << 4) & 0xF0F0F0F0u; // e0 e2 e4 e6, each times 16
                const uint32_t odd = raw[d] & 0xF0F0F0F0u;          // e1 e3 e5 e7
                w[2 * d] = (even & 0xFFu) | ((odd & 0xFFu) << 8) | ((even & 0xFF00u) << 8) | ((odd & 0xFF00u) << 16);
                w[2 * d + 1] = ((even >> 16) & 0xFFu) | (((odd >> 16) & 0xFFu) << 8) | (((even >> 24) & 0xFFu) << 16) |
                               ((odd >> 24) << 24);
            }
        } else {
#pragma unroll
            for (int p = 0; p < 16; ++p) {
                const int k = kc + p;
                if (k >= g.K) break;
                const uint32_t byte = col[k >> 1];
                const uint32_t v = ((byte >> ((k & 1) * 4)) & 0xFu) << 4;
                w[p >> 2] |= v << ((p & 3) * 8);
            }
        }
    }
}


// Epilogue shared by the dense kernels: zero-point correction (eq. 5-6), bias, fixed-point
// rescale, clamp; the uint8 tile is staged in LDS so that the global stores are 16-byte
// rows.  `so` must not be read by anyone else any more (callers synchronise before).
// Per-channel epilogue parameters of the TN column tiles a lane owns; fetched at kernel start
// so that their global-memory latency is hidden behind the main loop.
template <int TN> struct ChannelParams {
    int32_t bias[TN], mult[TN], shift[TN], zw[TN];
};

template <int BN, int WN, int TN>
__device__ __forceinline__ ChannelParams<TN> load_channel_params(const IgemmArgs &g, int n0)
{
    constexpr int WTN = BN / WN;
    const int lane = threadIdx.x & 63, wave_n = (threadIdx.x >> 6) % WN;
    ChannelParams<TN> p;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wave_n * WTN + j * 32 + (lane & 31);
        p.bias[j] = 0, p.mult[j] = 0, p.shift[j] = 1, p.zw[j] = 0;
        if (n < g.N) {
            p.bias[j] = g.bias ? g.bias[n] : 0;
            p.zw[j] = g.zw ? g.zw[n] : 0;
            p.mult[j] = g.mult[n];
            p.shift[j] = g.shift[n];
        }
    }
    return p;
}

// ZW: per-column weight zero-points; the term - z_w[n] * rowsum[m] joins every accumulator (the
// tile's row sums are staged in LDS behind the add tables)
template <int BM, int BN, int WM, int WN, bool WEIGHTS_X16, bool ZW, int TM, int TN>
__device__ __forceinline__ void igemm_epilogue_impl(const IgemmArgs &g, i32x16 (&acc)[TM][TN], int32_t (&colsum)[TN],
                                                    const ChannelParams<TN> &cp, uint8_t *so, int64_t m0, int n0)
{
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int OUT_PITCH = BN + 16;
    constexpr int ADD_TABLE_OFFSET = BM * OUT_PITCH + 4 * WM * WN * TN * 64; // behind the tile and the column-sum partials
    constexpr int ROWSUM_OFFSET = ADD_TABLE_OFFSET + 2048;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / WN, wave_n = wave % WN;
    const int frag_row = lane & 31, frag_half = lane >> 5;
    // with weight zero-points |z_w * rowsum| <= 2^15 * K joins the sum: the 32-bit forms stay exact for K <= 2048
    bool fast_ok = g.small_acc >= 1 && (!ZW || g.K <= 4096), fused_ok = g.small_acc >= 2 && (!ZW || g.K <= 2048);
    int32_t corr[TN];
    RescaleParams rp[TN];
    FusedRescale fr[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int32_t cs = colsum[j] + __shfl_xor(colsum[j], 32);
        if (WEIGHTS_X16) cs >>= 4;
        const int32_t b = cp.bias[j], mu = cp.mult[j], sf = cp.shift[j];
        corr[j] = b + (128 - g.z_a) * cs;
        rp[j] = make_rescale(mu, sf);
        // |acc + corr| < 2^30 for the 64-bit fast form, < 2^29 for the fused 32-bit form
        fast_ok = fast_ok && sf >= 0 && b > -(1 << 28) && b < (1 << 28);
        fused_ok = fused_ok && sf >= 1 && sf <= 20 && b > -(1 << 27) && b < (1 << 27);
        fr[j] = make_fused(mu, sf, corr[j], g.z_out, g.lo_rel + g.z_out, g.hi_rel + g.z_out);
    }
    const bool fast = __all(fast_ok), fused = __all(fused_ok);
    // A lane holds, for one column, the rows 8q + 4*half + {0,1,2,3} (q = 0..3) of each 32x32
    // tile.  The four bytes of a row group are packed into a dword and the 4x4 byte blocks are
    // transposed across the four lanes of a quad (two DPP exchanges + byte permutes), so that
    // every lane ends up with 4 consecutive columns of ONE row and the LDS tile is written
    // with conflict-free dword stores instead of byte stores.
    const int quad_lane = lane & 3;
    const uint32_t sel1 = (quad_lane & 1) ? 0x03070105u : 0x06020400u;
    const uint32_t sel2 = (quad_lane & 2) ? 0x03020706u : 0x05040100u;
    auto store_group = [&](int i, int j, int q, uint32_t x) { // x: the 4 bytes of rows 8q + 4*half + {0,1,2,3}
        // exchange with lane ^ 1, then with lane ^ 2 (quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E)
        uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true);
        x = __builtin_amdgcn_perm(o, x, sel1);
        o = (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, true);
        x = __builtin_amdgcn_perm(o, x, sel2);
        const int row = wave_m * WTM + i * 32 + 8 * q + 4 * frag_half + quad_lane;
        const int col = wave_n * WTN + j * 32 + (frag_row & ~3);
        *reinterpret_cast<uint32_t *>(so + row * OUT_PITCH + col) = x;
    };
    int32_t *const rs_lds = reinterpret_cast<int32_t *>(so + ROWSUM_OFFSET);
    if constexpr (ZW) { // the caller has synchronised: the operand ring is free
        for (int r = tid; r < BM; r += NT) rs_lds[r] = m0 + r < g.M ? g.rowsum[m0 + r] : 0;
        __syncthreads();
    }
    auto run = [&](auto pack4) {
#pragma clang loop unroll(full)
        for (int i = 0; i < TM; ++i)
#pragma clang loop unroll(full)
            for (int j = 0; j < TN; ++j)
#pragma clang loop unroll(full)
                for (int q = 0; q < 4; ++q) {
                    int32_t a[4];
                    i32x4 rs4 = {0, 0, 0, 0};
                    if constexpr (ZW) // rows 8q + 4*half + {0,1,2,3} of this 32-row tile
                        rs4 = *reinterpret_cast<const i32x4 *>(rs_lds + wave_m * WTM + i * 32 + 8 * q + 4 * frag_half);
#pragma clang loop unroll(full)
                    for (int e = 0; e < 4; ++e) {
                        a[e] = acc[i][j][4 * q + e];
                        if (WEIGHTS_X16) a[e] >>= 4; // weights were staged times 16; exact
                        if constexpr (ZW) a[e] = (int32_t)((uint32_t)a[e] - (uint32_t)cp.zw[j] * (uint32_t)rs4[e]); // wraps like the sum it is part of
                    }
                    store_group(i, j, q, pack4(a, j));
                }
    };
    auto pack_values = [&](const int32_t (&y)[4]) {
        return (uint32_t)y[0] | ((uint32_t)y[1] << 8) | ((uint32_t)y[2] << 16) | ((uint32_t)y[3] << 24);
    };
    if (fused && g.lo_rel >= 0) { // act_min >= z_out: the clamp absorbs the tie term
        run([&](const int32_t (&a)[4], int j) {
            uint32_t x = 0;
#pragma clang loop unroll(full)
            for (int e = 0; e < 4; ++e) x = shift_into_byte(x, rescale_fused_w<false>(a[e], fr[j]), fr[j].n1, e);
            return x;
        });
    } else if (fused) {
        run([&](const int32_t (&a)[4], int j) {
            uint32_t x = 0;
#pragma clang loop unroll(full)
            for (int e = 0; e < 4; ++e) x = shift_into_byte(x, rescale_fused_w<true>(a[e], fr[j]), fr[j].n1, e);
            return x;
        });
    } else if (fast) {
        run([&](const int32_t (&a)[4], int j) {
            int32_t y[4];
#pragma clang loop unroll(full)
            for (int e = 0; e < 4; ++e) y[e] = clamp_i32(g.lo_rel, g.hi_rel, rescale_fast(a[e] + corr[j], rp[j])) + g.z_out;
            return pack_values(y);
        });
    } else {
        run([&](const int32_t (&a)[4], int j) {
            int32_t y[4];
#pragma clang loop unroll(full)
            for (int e = 0; e < 4; ++e) y[e] = clamp_i32(g.lo_rel, g.hi_rel, rescale_general(a[e] + corr[j], rp[j])) + g.z_out;
            return pack_values(y);
        });
    }
    // optional rescaling add: tables of the 2 x 256 rescaled codes behind the output tile and the
    // column-sum partials (the operand ring is free by now)
    const bool add = g.R != nullptr; // uniform
    int32_t *const add_tab = reinterpret_cast<int32_t *>(so + ADD_TABLE_OFFSET);
    if (add) add_fill_tables(add_tab, g.add, tid, NT);
    __syncthreads();

    constexpr int ROW_CHUNKS = BN / 16;
    if (!add) {
        for (int q = tid; q < BM * ROW_CHUNKS; q += NT) {
            const int row = q / ROW_CHUNKS, cc = q % ROW_CHUNKS;
            const int64_t m = m0 + row;
            const int n = n0 + cc * 16;
            if (m >= g.M || n >= g.N) continue;
            uint8_t *dst = g.C + m * g.ldc + n;
            const uint8_t *src = so + row * OUT_PITCH + cc * 16;
            if (g.c_vec16 && n + 16 <= g.N) {
                *reinterpret_cast<u32x4 *>(dst) = *reinterpret_cast<const u32x4 *>(src);
            } else {
                for (int e = 0; e < 16 && n + e < g.N; ++e) dst[e] = src[e];
            }
        }
        return;
    }
    const AddOut ao = make_add_out(g.add);
    auto add_tile = [&](auto fused_tag) {
        constexpr bool FUSED = decltype(fused_tag)::value;
        for (int q = tid; q < BM * ROW_CHUNKS; q += NT) {
            const int row = q / ROW_CHUNKS, cc = q % ROW_CHUNKS;
            const int64_t m = m0 + row;
            const int n = n0 + cc * 16;
            if (m >= g.M || n >= g.N) continue;
            uint8_t *dst = g.C + m * g.ldc + n;
            const uint8_t *res = g.R + m * g.ldr + n;
            const uint8_t *src = so + row * OUT_PITCH + cc * 16;
            if (g.c_vec16 && g.r_vec16 && n + 16 <= g.N) {
                const u32x4 r = *reinterpret_cast<const u32x4 *>(res);
                const u32x4 v = *reinterpret_cast<const u32x4 *>(src);
                u32x4 y;
#pragma unroll
                for (int d = 0; d < 4; ++d) y[d] = add_codes4<FUSED>(v[d], r[d], add_tab, ao);
                *reinterpret_cast<u32x4 *>(dst) = y;
            } else {
                for (int e = 0; e < 16 && n + e < g.N; ++e) dst[e] = (uint8_t)add_code1<FUSED>(src[e], res[e], add_tab, ao);
            }
        }
    };
    if (ao.fused) add_tile(std::true_type{});
    else add_tile(std::false_type{});
}

template <int BM, int BN, int WM, int WN, bool WEIGHTS_X16, bool ZW = false, int TM, int TN>
__device__ __forceinline__ void igemm_epilogue(const IgemmArgs &g, i32x16 (&acc)[TM][TN], int32_t (&colsum)[TN],
                                               const ChannelParams<TN> &cp, uint8_t *so, int64_t m0, int n0)
{
    igemm_epilogue_impl<BM, BN, WM, WN, WEIGHTS_X16, ZW, TM, TN>(g, acc, colsum, cp, so, m0, n0);
}

template <int BM, int BN, int WM, int WN, int A_MODE, int B_MODE, int VEC, bool ZW = false>
__global__ void __launch_bounds__(WM *WN * 64) igemm_kernel(const IgemmArgs g)
{
    constexpr int NT = WM * WN * 64;
    constexpr int BK = 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int A_CHUNKS = BM * 4 / NT, B_CHUNKS = BN * 4 / NT;
    static_assert(BM * 4 % NT == 0 && BN * 4 % NT == 0, "staging assumes whole chunks per thread");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of 32x32 MFMA tiles");
    constexpr int OUT_PITCH = BN + 16;
    constexpr int STAGE_BYTES = (BM + BN) * BK;
    constexpr int OUT_BYTES = BM * OUT_PITCH + 4 * WM * WN * TN * 64 + 2048 + 4 * BM; // tile, column-sum partials, add tables, row sums
    constexpr int SMEM_BYTES = (2 * STAGE_BYTES > OUT_BYTES) ? 2 * STAGE_BYTES : OUT_BYTES;
    __shared__ __attribute__((aligned(16))) uint8_t smem[SMEM_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / WN, wave_n = wave % WN;

    const int tiles_n = (g.N + BN - 1) / BN;
    const int64_t tile = blockIdx.x;
    const int64_t m0 = (tile / tiles_n) * BM;
    const int n0 = (int)(tile % tiles_n) * BN;

    // ---- rows of A and columns of B this thread stages (the same ones at every k step)
    const int chunk_c = tid & 3;
    ARow arow[A_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
        const int64_t m = m0 + (tid >> 2) + i * (NT / 4);
        arow[i].valid = m < g.M;
        arow[i].hi0 = arow[i].wi0 = 0;
        if (A_MODE == A_MATRIX) {
            arow[i].base = g.A + m * g.lda;
        } else {
            const int64_t img = m / ((int64_t)g.Ho * g.Wo);
            const int rem = (int)(m - img * ((int64_t)g.Ho * g.Wo));
            const int ho = rem / g.Wo, wo = rem - ho * g.Wo;
            arow[i].base = g.A + img * ((int64_t)g.H * g.W * g.Cin);
            arow[i].hi0 = ho * g.sh - g.ph;
            arow[i].wi0 = wo * g.sw - g.pw;
        }
    }
    const uint32_t fill_a = (uint32_t)g.z_a * 0x01010101u;
    const ChannelParams<TN> cparams = load_channel_params<BN, WN, TN>(g, n0);

    uint32_t stage_a[A_CHUNKS][4], stage_b[B_CHUNKS][4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) load_a_chunk<A_MODE, VEC>(g, arow[i], k0 + chunk_c * 16, fill_a, stage_a[i]);
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i)
            load_b_chunk<B_MODE, VEC>(g, n0 + (tid >> 2) + i * (NT / 4), k0 + chunk_c * 16, stage_b[i]);
    };
    auto commit = [&](int buf) {
        uint8_t *sa = smem + buf * STAGE_BYTES;
        uint8_t *sb = sa + BM * BK;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int row = (tid >> 2) + i * (NT / 4);
            u32x4 v = {stage_a[i][0] ^ 0x80808080u, stage_a[i][1] ^ 0x80808080u, stage_a[i][2] ^ 0x80808080u,
                       stage_a[i][3] ^ 0x80808080u}; // uint8 code -> signed code - 128
            *reinterpret_cast<u32x4 *>(sa + lds_chunk_offset(row, chunk_c)) = v;
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            const int row = (tid >> 2) + i * (NT / 4);
            u32x4 v = {stage_b[i][0], stage_b[i][1], stage_b[i][2], stage_b[i][3]};
            *reinterpret_cast<u32x4 *>(sb + lds_chunk_offset(row, chunk_c)) = v;
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
    fetch(0);
    commit(0);
    __syncthreads();

    const int frag_row = lane & 31, frag_half = lane >> 5;
    for (int kt = 0; kt < ktiles; ++kt) {
        const bool more = kt + 1 < ktiles;
        if (more) fetch((kt + 1) * BK);
        const uint8_t *sa = smem + (kt & 1) * STAGE_BYTES;
        const uint8_t *sb = sa + BM * BK;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            i32x4 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const i32x4 *>(
                    sa + lds_chunk_offset(wave_m * WTM + i * 32 + frag_row, ks * 2 + frag_half));
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                fb[j] = *reinterpret_cast<const i32x4 *>(
                    sb + lds_chunk_offset(wave_n * WTN + j * 32 + frag_row, ks * 2 + frag_half));
#pragma unroll
                for (int d = 0; d < 4; ++d) colsum[j] = __builtin_amdgcn_sdot4(fb[j][d], 0x01010101, colsum[j], false);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (more) commit((kt + 1) & 1);
        __syncthreads();
    }

    // the last __syncthreads above guarantees nobody still reads the operand tiles
    igemm_epilogue<BM, BN, WM, WN, B_MODE == B_INT4, ZW>(g, acc, colsum, cparams, smem, m0, n0);
}

} // namespace qnn
