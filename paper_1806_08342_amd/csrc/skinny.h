// Quantized GEMM with very few rows (M <= 64: a fully connected layer at small batch).
//
// The product is bound by streaming the weights from HBM once (K*N bytes, half of that for
// 4-bit weights), so the kernel is organised around memory-level parallelism, not MFMA rate:
// one workgroup owns 16 output columns, its 8 waves split K between them, and every lane
// fetches its own MFMA fragments straight from global memory with 16-byte loads (several
// K-steps in flight), no LDS staging.  The roles of the operands are swapped with respect to
// the big kernel: the weights are the A operand of v_mfma_i32_16x16x64_i8 (16 columns n x 64 k)
// and the activations the B operand (16 rows m), so a lane ends up with 4 consecutive output
// columns of one row m: one dword store, no transposition.  4-bit weights are unpacked in
// registers (kept times 16 in int8, accumulators shifted back exactly).  The partial sums of
// the 8 waves are combined through LDS; arithmetic and rescale as in igemm.h.
#pragma once

#include "igemm.h"

namespace qnn {

template <int MT, bool INT4>
__global__ void __launch_bounds__(512) skinny_gemm_kernel(const IgemmArgs g)
{
    constexpr int NW = 8, BN = 16, BK = 64, UNROLL = 4;
    __shared__ int32_t part[NW][MT][4][64]; // [wave][m tile][register][lane]
    __shared__ int32_t csum[NW][BN];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = blockIdx.x * BN;
    const int frow = lane & 15, fk = (lane >> 4) * 16; // fragment row / column, k offset inside a K-step

    // weight row (output column) and activation rows of this lane's fragments, clamped
    int nw = n0 + frow;
    nw = nw < g.N ? nw : g.N - 1;
    const uint8_t *brow = INT4 ? g.B + (((int64_t)nw * g.ldb) >> 1) : g.B + (int64_t)nw * g.ldb;
    const uint8_t *arow[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        int64_t m = t * 16 + frow;
        m = m < g.M ? m : g.M - 1;
        arow[t] = g.A + m * g.lda;
    }

    i32x4 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = i32x4{0, 0, 0, 0};
    int32_t colsum = 0;
    const bool need_colsum = g.z_a != 128;

    const int ksteps = g.K / BK; // K % 64 == 0 (dispatcher)
    // 4-bit weights, wide form: a lane fetches 16 bytes = 32 consecutive weights per load, so that as many weight
    // bytes are in flight as with 8-bit weights (the kernel lives on memory-level parallelism).  The 32 weights
    // feed two matrix instructions; the reduction index is renumbered for that -- quarter q of the lanes takes
    // k = 128 s + 32 q + 16 h + (0..15) in instruction h of step s, on both operands alike, and a sum does not care
    // about the order of its terms.
    bool wide = false;
    if constexpr (INT4) wide = (g.K & 127) == 0 && (g.ldb & 31) == 0 && (reinterpret_cast<uintptr_t>(g.B) & 15) == 0;
    if constexpr (INT4) {
        if (wide) {
            constexpr int UW = MT >= 4 ? 2 : 4;
            const int steps2 = g.K / 128, kq = (lane >> 4) * 32;
            for (int s0 = wave; s0 < steps2; s0 += NW * UW) {
                u32x4 raw[UW];
                i32x4 fa[UW][2][MT];
#pragma unroll
                for (int u = 0; u < UW; ++u) {
                    const int st = s0 + u * NW;
                    const int k = (st < steps2 ? st : steps2 - 1) * 128 + kq; // past the end: re-read, ignored below
                    raw[u] = *reinterpret_cast<const u32x4 *>(brow + (k >> 1));
#pragma unroll
                    for (int t = 0; t < MT; ++t) {
                        fa[u][0][t] = *reinterpret_cast<const i32x4 *>(arow[t] + k);
                        fa[u][1][t] = *reinterpret_cast<const i32x4 *>(arow[t] + k + 16);
                    }
                }
#pragma unroll
                for (int u = 0; u < UW; ++u) {
                    if (s0 + u * NW >= steps2) break;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        i32x4 fb; // dword d of raw holds weights 8d .. 8d+7, two per byte, low nibble first; kept times 16
#pragma unroll
                        for (int d = 0; d < 2; ++d) {
                            const uint32_t r = raw[u][2 * h + d];
                            const uint32_t even = (r << 4) & 0xF0F0F0F0u, odd = r & 0xF0F0F0F0u;
                            fb[2 * d] = (int32_t)__builtin_amdgcn_perm(odd, even, 0x05010400u);
                            fb[2 * d + 1] = (int32_t)__builtin_amdgcn_perm(odd, even, 0x07030602u);
                        }
                        if (need_colsum) {
#pragma unroll
                            for (int d = 0; d < 4; ++d) colsum = __builtin_amdgcn_sdot4(fb[d], 0x01010101, colsum, false);
                        }
#pragma unroll
                        for (int t = 0; t < MT; ++t) {
                            const i32x4 xs = fa[u][h][t] ^ (int32_t)0x80808080;
                            acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fb, xs, acc[t], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }
    for (int ks0 = wave; ks0 < (wide ? 0 : ksteps); ks0 += NW * UNROLL) {
        i32x4 fb[UNROLL];       // weights
        i32x4 fa[UNROLL][MT];   // activations
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int ks = ks0 + u * NW;
            const int k = (ks < ksteps ? ks : ksteps - 1) * BK + fk; // past the end: re-read, ignored below
            if constexpr (INT4) {
                const u32x2 raw = *reinterpret_cast<const u32x2 *>(brow + (k >> 1));
                const uint32_t r2[2] = {raw.x, raw.y};
#pragma unroll
                for (int d = 0; d < 2; ++d) { // r2[d] holds elements 8d .. 8d+7, two per byte
                    const uint32_t even = (r2[d] << 4) & 0xF0F0F0F0u, odd = r2[d] & 0xF0F0F0F0u;
                    fb[u][2 * d] = (int32_t)((even & 0xFFu) | ((odd & 0xFFu) << 8) | ((even & 0xFF00u) << 8) |
                                             ((odd & 0xFF00u) << 16));
                    fb[u][2 * d + 1] = (int32_t)(((even >> 16) & 0xFFu) | (((odd >> 16) & 0xFFu) << 8) |
                                                 (((even >> 24) & 0xFFu) << 16) | ((odd >> 24) << 24));
                }
            } else {
                fb[u] = *reinterpret_cast<const i32x4 *>(brow + k);
            }
#pragma unroll
            for (int t = 0; t < MT; ++t) fa[u][t] = *reinterpret_cast<const i32x4 *>(arow[t] + k);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (ks0 + u * NW >= ksteps) break;
            if (need_colsum) {
#pragma unroll
                for (int d = 0; d < 4; ++d) colsum = __builtin_amdgcn_sdot4(fb[u][d], 0x01010101, colsum, false);
            }
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const i32x4 xs = fa[u][t] ^ (int32_t)0x80808080; // uint8 code -> signed (code - 128)
                acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fb[u], xs, acc[t], 0, 0, 0);
            }
        }
    }

    // ---- combine the waves
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) part[wave][t][e][lane] = acc[t][e];
    colsum += __shfl_xor(colsum, 16);
    colsum += __shfl_xor(colsum, 32);
    if (lane < BN) csum[wave][lane] = colsum;
    __syncthreads();

    // ---- epilogue: thread -> (m tile, lane of the accumulator layout): row m = 16t + (l & 15),
    // columns n0 + 4*(l >> 4) + {0,1,2,3}
    for (int item = tid; item < MT * 64; item += NW * 64) {
        const int t = item >> 6, l = item & 63;
        const int64_t m = t * 16 + (l & 15);
        const int nb = n0 + 4 * (l >> 4);
        if (m >= g.M || nb >= g.N) continue;
        uint32_t packed = 0;
        int valid = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int n = nb + e;
            if (n >= g.N) break;
            int32_t a = 0, cs = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                a += part[w][t][e][l];
                cs += csum[w][4 * (l >> 4) + e];
            }
            if (INT4) {
                a >>= 4; // weights were kept times 16; exact
                cs >>= 4;
            }
            a += (g.bias ? g.bias[n] : 0) + (128 - g.z_a) * cs;
            const RescaleParams rp = make_rescale(g.mult[n], g.shift[n]);
            const int32_t y = clamp_i32(g.lo_rel, g.hi_rel, rescale_general(a, rp)) + g.z_out;
            packed |= (uint32_t)y << (8 * e);
            ++valid;
        }
        uint8_t *dst = g.C + m * g.ldc + nb;
        if (valid == 4 && (reinterpret_cast<uintptr_t>(dst) & 3) == 0) {
            *reinterpret_cast<uint32_t *>(dst) = packed;
        } else {
            for (int e = 0; e < valid; ++e) dst[e] = (uint8_t)(packed >> (8 * e));
        }
    }
}

} // namespace qnn
