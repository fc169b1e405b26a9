// Dense quantized layer with a medium reduction (256 < K <= ~1200) and few output channels:
// 1x1 convolutions / GEMMs with K = 512 .. 1024 and 3x3 convolutions over 64 .. 128 channels.
// By bytes these layers are bound by HBM; with output tiles, every tile pays its own pipeline
// fill and epilogue around a K loop of only 8 - 18 steps.
//
// Weight-resident: a workgroup (8 waves) owns up to 128 output columns and keeps ALL K rows of
// them in LDS for its whole life, already laid out as MFMA B fragments (fragment (ks, j) = 1 KB,
// lane l at byte 16*l: linear, conflict-free reads; 4-bit weights are unpacked while filling).
// After that one barrier the waves never synchronise again: each walks over blocks of 32 output
// rows (pixels), fetches its A fragments straight from global memory (16 bytes per lane; for a
// convolution the tap of a 32-deep K sub-step is wave-uniform, only the bounds test is per
// lane; taps outside the image read as the code z_x), in chunks of KC K sub-steps with the next
// two chunks in flight, one LDS read per MFMA, and finishes a block with the epilogue of shortk.h
// (constants in registers, wave-private LDS tile, 16-byte row stores issued one block late).
// Arithmetic as in igemm.h (eq. 4-6 with z_w = 0, bias, RESCALE, clamp).
#pragma once

#include <type_traits>

#include "fill_table.h"
#include "igemm.h"

namespace qnn {

struct BResArgs {
    IgemmArgs g;         // A_MATRIX fields or the convolution geometry (Cin % 32 == 0, kw in g.kw)
    int col_groups;      // ceil(N / (32 * NB))
    int groups_walkers;  // workgroups that share one column group
};

// KC: K sub-steps (of 32) per chunk; CONV: rows of A are gathered pixels; PAD: K / 32 is not a multiple of KC
template <int NB, int KC, bool INT4, bool CONV, bool PAD>
__global__ void __launch_bounds__(512, 2) bres_kernel(const BResArgs s)
{
    constexpr int NW = 8;                     // waves per workgroup
    constexpr int PITCH = 32 * NB + 32;       // staged output row (see shortk.h)
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const IgemmArgs &g = s.g;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int frow = lane & 31, fhalf = lane >> 5;
    const int KS = g.K / 32;                  // the dispatcher guarantees K % 32 == 0
    uint8_t *const bfrag = smem;                                   // KS * NB fragments of 1 KB
    uint8_t *const stage = smem + KS * NB * 1024 + wave * 32 * PITCH;

    const int cg = blockIdx.x % s.col_groups, wg_walker = blockIdx.x / s.col_groups;
    const int n0 = cg * 32 * NB;
    const int blocks_here = (g.N - n0 + 31) / 32 < NB ? (g.N - n0 + 31) / 32 : NB;

    // ---- weights -> LDS, in fragment order
    for (int f = wave; f < KS * NB; f += NW) {
        const int ks = f / NB, j = f - ks * NB;
        int n = n0 + j * 32 + frow;
        n = n < g.N ? n : g.N - 1;
        const int k = ks * 32 + fhalf * 16;
        u32x4 v;
        if constexpr (INT4) {
            const u32x2 raw = *reinterpret_cast<const u32x2 *>(g.B + (((int64_t)n * g.ldb + k) >> 1));
            const uint32_t r2[2] = {raw.x, raw.y};
#pragma unroll
            for (int d = 0; d < 2; ++d) { // two nibbles per byte, low nibble first; sign-extend to int8
                uint32_t lo = r2[d] & 0x0F0F0F0Fu, hi = (r2[d] >> 4) & 0x0F0F0F0Fu;
                lo |= ((lo >> 3) & 0x01010101u) * 0xF0u;
                hi |= ((hi >> 3) & 0x01010101u) * 0xF0u;
                v[2 * d] = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
                v[2 * d + 1] = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
            }
        } else {
            v = *reinterpret_cast<const u32x4 *>(g.B + (int64_t)n * g.ldb + k);
        }
        *reinterpret_cast<u32x4 *>(bfrag + f * 1024 + lane * 16) = v;
    }
    __syncthreads(); // the only workgroup barrier

    // ---- per-column epilogue constants (as in shortk.h)
    int32_t c_mult[NB], c_corr[NB], c_c[NB], c_n1[NB], c_lo[NB], c_hi[NB], c_shift[NB];
    bool fused_ok = g.small_acc >= 2;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        int n = n0 + j * 32 + frow;
        n = n < g.N ? n : g.N - 1;
        int32_t colsum = 0;
        if (g.z_a != 128) {
            for (int ks = 0; ks < KS; ++ks) {
                const i32x4 b = *reinterpret_cast<const i32x4 *>(bfrag + (ks * NB + j) * 1024 + lane * 16);
#pragma unroll
                for (int d = 0; d < 4; ++d) colsum = __builtin_amdgcn_sdot4(b[d], 0x01010101, colsum, false);
            }
            colsum += __shfl_xor(colsum, 32);
        }
        const int32_t b = g.bias ? g.bias[n] : 0, mu = g.mult[n], sf = g.shift[n];
        fused_ok = fused_ok && sf >= 1 && sf <= 20 && b > -(1 << 27) && b < (1 << 27);
        const int nn = (sf >= 1 && sf <= 20) ? sf : 1;
        c_mult[j] = mu;
        c_corr[j] = b + (128 - g.z_a) * colsum;
        c_n1[j] = nn + 1;
        c_c[j] = 2 * ((1 << (nn - 1)) + (g.z_out << nn)) + 1;
        c_lo[j] = (g.lo_rel + g.z_out) << (nn + 1);
        c_hi[j] = ((g.hi_rel + g.z_out + 1) << (nn + 1)) - 1;
        c_shift[j] = sf;
    }
    const bool fused = __all(fused_ok);

    // ---- rows (the dispatcher guarantees M < 2^31 and 32-bit offsets inside one image / matrix)
    const int M = (int)g.M;
    const int row_blocks = (M + 31) / 32;
    const int walkers = s.groups_walkers * NW;
    const int walker = wg_walker * NW + wave;

    // where the row (pixel) of this lane starts, for the row block being loaded
    const uint8_t *row_base = g.A;
    int row_hi0 = 0, row_wi0 = 0;
    auto set_rows = [&](int rb) {
        int m = rb * 32 + frow;
        m = m < M ? m : M - 1;
        if constexpr (CONV) {
            const uint32_t per_image = (uint32_t)g.Ho * (uint32_t)g.Wo;
            const uint32_t img = (uint32_t)m / per_image, rem = (uint32_t)m - img * per_image;
            const uint32_t ho = rem / (uint32_t)g.Wo, wo = rem - ho * (uint32_t)g.Wo;
            row_hi0 = (int)ho * g.sh - g.ph;
            row_wi0 = (int)wo * g.sw - g.pw;
            // address of tap (0,0), channel 0 of this pixel's window (may lie outside the image: only
            // dereferenced after the bounds test)
            row_base = g.A + ((int64_t)img * g.H * g.W + (int64_t)row_hi0 * g.W + row_wi0) * g.Cin + fhalf * 16;
        } else {
            row_base = g.A + (int64_t)m * g.lda + fhalf * 16;
        }
    };
    // The 16 bytes of the next K sub-step of the load stream.  The stream walks the sub-steps of a
    // block in order, so its kernel row / column and its byte offset from tap (0,0) are kept in
    // scalar registers and advanced by compare-and-select.  A tap outside the image is read from a
    // constant chunk holding the code z_x instead (an address select, no data select behind the
    // load).  Sub-steps past the end of K (padded last chunk) read some valid address; their MFMA
    // operand is zeroed at use.
    const uint8_t *const fill_chunk = &g_fill_table.v[g.z_a][0];
    int t_a = 0, t_b = 0, t_ci = 0, t_off = 0, t_ks = 0;
    auto restart_stream = [&] { t_a = t_b = t_ci = t_off = t_ks = 0; };
    auto load_piece = [&]() -> i32x4 {
        i32x4 v;
        if constexpr (CONV) {
            const int hi = row_hi0 + t_a, wi = row_wi0 + t_b;
            const bool ok = (unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W;
            const uint8_t *p = ok ? row_base + t_off : fill_chunk;
            v = *reinterpret_cast<const i32x4 *>(p);
            t_ci += 32, t_off += 32;
            const bool next_tap = t_ci >= g.Cin; // the offset already points at the next pixel then
            t_ci = next_tap ? 0 : t_ci;
            t_b += next_tap ? 1 : 0;
            const bool next_row = t_b >= g.kw;
            t_b = next_row ? 0 : t_b;
            t_a += next_row ? 1 : 0;
            t_off += next_row ? (g.W - g.kw) * g.Cin : 0;
        } else {
            const int ks = t_ks < KS ? t_ks : KS - 1;
            v = *reinterpret_cast<const i32x4 *>(row_base + ks * 32);
            ++t_ks;
        }
        return v;
    };
    auto load_chunk = [&](i32x4 (&fa)[KC]) {
#pragma unroll
        for (int u = 0; u < KC; ++u) fa[u] = load_piece();
    };

    // lane-invariant parts of the output addresses (as in shortk.h)
    int st_lds[NB], st_row[NB];
    bool st_col_ok[NB];
    int64_t st_off[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int idx = i * 64 + lane;
        st_row[i] = idx / (2 * NB);
        const int col0 = n0 + (idx % (2 * NB)) * 16;
        st_col_ok[i] = col0 < g.N;
        st_lds[i] = st_row[i] * PITCH + (idx % (2 * NB)) * 16;
        st_off[i] = (int64_t)st_row[i] * g.ldc + col0;
    }
    const int put_base = (4 * fhalf + (lane & 3)) * PITCH + (frow & ~3);
    const bool chunks_whole = g.c_vec16 && ((g.N & 15) == 0 || n0 + 32 * NB <= g.N);
    const int quad_lane = lane & 3;
    const uint32_t sel1 = (quad_lane & 1) ? 0x03070105u : 0x06020400u;
    const uint32_t sel2 = (quad_lane & 2) ? 0x03020706u : 0x05040100u;

    auto wave_sync = [] { // orders the wave's own LDS traffic for the compiler; the hardware keeps it in order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    auto store_block = [&](int rbx) {
        wave_sync();
        uint8_t *const c_block = g.C + (int64_t)rbx * 32 * g.ldc;
        if (chunks_whole) {
            const bool whole_rows = rbx * 32 + 32 <= M;
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (st_col_ok[i] && (whole_rows || rbx * 32 + st_row[i] < M))
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
        wave_sync();
    };

    auto walk = [&](auto fused_tag) {
        constexpr bool FUSED = decltype(fused_tag)::value > 0, TIES = decltype(fused_tag)::value == 1; // 2: without the tie term
        const int chunks = (KS + KC - 1) / KC;
        i32x4 fa0[KC], fa1[KC], fa2[KC]; // the chunk being computed and the next two, in flight
        i32x16 acc[NB];
        int rb_stored = -1;
        int rb = walker, chunk = 0; // position of the chunk held in the "current" set
        if (rb >= row_blocks) return;
        auto advance = [&](int &r, int &c) {
            if (++c == chunks) r += walkers, c = 0;
        };
        set_rows(rb);
        restart_stream();
        load_chunk(fa0);
        {
            int r1 = rb, c1 = 0;
            advance(r1, c1);
            if (r1 < row_blocks) {
                if (c1 == 0) set_rows(r1), restart_stream();
                load_chunk(fa1);
            }
        }
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = 0;
        // one step: request the chunk two after (rb, chunk) into `nxt`, compute (rb, chunk) from `cur`
        auto step = [&](i32x4 (&cur)[KC], i32x4 (&nxt)[KC]) {
            int rb_1 = rb, chunk_1 = chunk;
            advance(rb_1, chunk_1);
            int rb_n = rb_1, chunk_n = chunk_1;
            advance(rb_n, chunk_n);
            // Order matters for the memory counter (loads and stores share it, and a wait with both
            // kinds pending drains everything): first consume the current chunk's loads (the XOR
            // below waits for them while only loads are in flight), then issue the previous block's
            // stores, then the loads of the chunk two ahead, piece by piece between the MFMAs.
            i32x4 xs[KC];
#pragma unroll
            for (int u = 0; u < KC; ++u) {
                xs[u] = cur[u] ^ (int32_t)0x80808080; // uint8 code -> signed (code - 128)
                if constexpr (PAD) {
                    if (chunk * KC + u >= KS) xs[u] = i32x4{0, 0, 0, 0}; // wave-uniform; a zero operand adds nothing
                }
            }
            if (chunk == 0 && rb_stored >= 0) {
                store_block(rb_stored);
                rb_stored = -1;
            }
            // past the last block the stream just runs on: its loads stay inside the image / row
            if (chunk_n == 0 && rb_n < row_blocks) set_rows(rb_n);
            if (chunk_n == 0) restart_stream();
            const int ks0 = chunk * KC;
            auto b_frag = [&](int u, int j) {
                int ks = ks0 + u;
                ks = ks < KS ? ks : KS - 1;
                return *reinterpret_cast<const i32x4 *>(bfrag + (ks * NB + j) * 1024 + lane * 16);
            };
            i32x4 bq[3][NB]; // B fragments of the sub-step at the MFMAs and of the two after it
#pragma unroll
            for (int j = 0; j < NB; ++j) bq[0][j] = b_frag(0, j);
            if (KC > 1) {
#pragma unroll
                for (int j = 0; j < NB; ++j) bq[1][j] = b_frag(1, j);
            }
#pragma unroll
            for (int u = 0; u < KC; ++u) {
                if (u + 2 < KC) {
#pragma unroll
                    for (int j = 0; j < NB; ++j) bq[(u + 2) % 3][j] = b_frag(u + 2, j);
                }
#pragma unroll
                for (int j = 0; j < NB; ++j) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xs[u], bq[u % 3][j], acc[j], 0, 0, 0);
                nxt[u] = load_piece();
            }
            if (chunk == chunks - 1) { // the block is complete: epilogue into the wave's LDS tile
                auto put = [&](int j, int q, uint32_t x) {
                    uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true);
                    x = __builtin_amdgcn_perm(o, x, sel1);
                    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, true);
                    x = __builtin_amdgcn_perm(o, x, sel2);
                    *reinterpret_cast<uint32_t *>(stage + put_base + q * 8 * PITCH + j * 32) = x;
                };
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    if (j >= blocks_here) break;
                    const RescaleParams rp = make_rescale(c_mult[j], c_shift[j]);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        uint32_t x = 0;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int32_t a = acc[j][4 * q + e];
                            if constexpr (FUSED) {
                                const int32_t t = __mulhi((int32_t)((uint32_t)(a + c_corr[j]) << 2), c_mult[j]);
                                const int32_t w = fused_w_from_t<TIES>(t, c_c[j]);
                                x = shift_into_byte(x, med3_i32(w, c_lo[j], c_hi[j]), c_n1[j], e);
                            } else {
                                const int32_t y = clamp_i32(g.lo_rel, g.hi_rel, rescale_general(a + c_corr[j], rp)) + g.z_out;
                                x |= (uint32_t)y << (8 * e);
                            }
                        }
                        put(j, q, x);
                    }
                }
                wave_sync();
                rb_stored = rb;
#pragma unroll
                for (int j = 0; j < NB; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[j][r] = 0;
            }
            rb = rb_1, chunk = chunk_1;
        };
        while (rb < row_blocks) {
            step(fa0, fa2);
            if (rb < row_blocks) step(fa1, fa0);
            if (rb < row_blocks) step(fa2, fa1);
        }
        if (rb_stored >= 0) store_block(rb_stored);
    };
    if (!fused) walk(std::integral_constant<int, 0>{});
    else if (g.lo_rel < 0) walk(std::integral_constant<int, 1>{});
    else walk(std::integral_constant<int, 2>{}); // act_min >= z_out: the clamp absorbs the tie term
}

} // namespace qnn
