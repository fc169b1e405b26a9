// Network stems (3x3x3, 7x7x3: very few input channels), barrier-free variant of stemconv.h.
//
// One wave owns 32 consecutive output pixels of an output row, all (<= 64) output channels, and
// walks down a segment of output rows.  As in stemconv.h one kernel row (kw * Cin <= 32 bytes) is
// a contiguous byte run of the NHWC image and is one 32-deep K sub-step: K is laid out as kh
// sub-steps, the weights (zero-padded to 32 per kernel row) stay in registers as MFMA B
// fragments.  The image rows the strip needs (at most 256 bytes each: one dword per lane) live in
// a wave-private LDS ring of 8 rows; going from one output row to the next only stride_h new
// image rows are fetched (aligned dword loads, out-of-image dwords replaced by the code z_x; the
// loads for the next output row are in flight while the current one is computed; the row stride
// is a template parameter so that these fetches are straight-line code).  Each lane
// cuts its 32-byte window out of the ring with dword reads + v_alignbyte (the codes are stored
// in the ring already offset to signed bytes).  After the weights are staged (once per
// workgroup, two barriers) nothing in the kernel synchronises waves with each other.  Epilogue as in shortk.h.
#pragma once

#include <type_traits>

#include "fill_table.h"
#include "igemm.h"

namespace qnn {

struct StemWaveArgs {
    IgemmArgs g;       // geometry, pointers, epilogue parameters (g.N = Cout, g.ldc = Cout)
    int kh, run;       // run = kw * Cin <= 32
    int strips;        // ceil(Wo / 32)
    int segments;      // an image column of strips is cut into this many row segments
    int rows_per_seg;  // ceil(Ho / segments)
    int64_t waves;     // N * strips * segments
};

template <int KH, int NB, int SH> // kernel rows, blocks of 32 output channels, row stride (compile-time: the row fetches are unrolled)
__global__ void __launch_bounds__(256) stemwave_kernel(const StemWaveArgs s)
{
    constexpr int NEW = SH < KH ? SH : KH; // image rows that enter the window per output row
    constexpr int PITCH = 32 * NB + 32; // staged output row (see shortk.h)
    constexpr int RING = 8, ROW_BYTES = 256 + 32; // ring rows; a little slack behind a row for the window reads
    static_assert(KH <= RING, "the rows of one output row must fit the ring");
    // one LDS block: the raw filter bank while the fragments are built, then the waves' rings and output tiles
    constexpr int RING_ALL = 4 * RING * ROW_BYTES, WORK = RING_ALL + 4 * 32 * PITCH;
    static_assert(NB * 32 * KH * 32 + 32 <= WORK, "the raw weights must fit the block they borrow");
    __shared__ __attribute__((aligned(16))) uint8_t work[WORK];
    __shared__ __attribute__((aligned(16))) uint8_t wfrag[KH * NB * 1024]; // B fragments: (kernel row, column block) x lane x 16
    const IgemmArgs &g = s.g;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint8_t *const ring = work + wave * (RING * ROW_BYTES), *const stage = work + RING_ALL + wave * (32 * PITCH);
    const int frow = lane & 31, fhalf = lane >> 5;

    // ---- weights, once per workgroup: [Cout][kh][run] bytes -> LDS with coalesced loads, then each
    // wave cuts a share of the MFMA B fragments (kernel row, column block; rows zero padded to 32)
    // out of it and leaves them in LDS for all four waves
    {
        const int total = g.N * KH * s.run;
        if ((reinterpret_cast<uintptr_t>(g.B) & 3) == 0) {
            for (int i = threadIdx.x; i * 4 + 4 <= total; i += 256)
                reinterpret_cast<uint32_t *>(work)[i] = reinterpret_cast<const uint32_t *>(g.B)[i];
            if ((int)threadIdx.x < (total & 3)) work[(total & ~3) + threadIdx.x] = g.B[(total & ~3) + threadIdx.x];
        } else {
            for (int i = threadIdx.x; i < total; i += 256) work[i] = g.B[i];
        }
        __syncthreads();
        for (int p = wave; p < KH * NB; p += 4) { // p = a * NB + j, wave-uniform
            const int a = p / NB, j = p % NB;
            int co = j * 32 + frow;
            co = co < g.N ? co : g.N - 1;
            const int addr = (co * KH + a) * s.run + fhalf * 16;
            const uint32_t *src = reinterpret_cast<const uint32_t *>(work + (addr & ~3));
            uint32_t d[5];
#pragma unroll
            for (int e = 0; e < 5; ++e) d[e] = src[e];
            u32x4 f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int valid = s.run - fhalf * 16 - e * 4; // bytes of this dword that belong to the kernel row
                valid = valid < 0 ? 0 : (valid > 4 ? 4 : valid);
                const uint32_t mask = valid >= 4 ? 0xffffffffu : ((1u << (8 * valid)) - 1u);
                f[e] = __builtin_amdgcn_alignbyte(d[e + 1], d[e], (uint32_t)(addr & 3)) & mask;
            }
            *reinterpret_cast<u32x4 *>(wfrag + p * 1024 + lane * 16) = f;
        }
        __syncthreads(); // the only workgroup barriers: from here on the waves run independently
    }

    // ---- wave -> (image, strip of 32 output columns, segment of output rows); all wave-uniform
    int64_t w = (int64_t)blockIdx.x * 4 + wave;
    if (w >= s.waves) return;
    const int strip = (int)(w % s.strips);
    w /= s.strips;
    const int seg = (int)(w % s.segments);
    const int n = (int)(w / s.segments);
    const int wo0 = strip * 32;
    const int ho_begin = seg * s.rows_per_seg;
    const int ho_end = ho_begin + s.rows_per_seg < g.Ho ? ho_begin + s.rows_per_seg : g.Ho;
    if (ho_begin >= ho_end) return;

    i32x4 fb[KH][NB];
    int32_t c_mult[NB], c_corr[NB], c_c[NB], c_n1[NB], c_lo[NB], c_hi[NB], c_shift[NB];
    bool fused_ok = true;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        int co = j * 32 + frow;
        co = co < g.N ? co : g.N - 1;
        int32_t colsum = 0;
#pragma unroll
        for (int a = 0; a < KH; ++a) {
            fb[a][j] = *reinterpret_cast<const i32x4 *>(wfrag + (a * NB + j) * 1024 + lane * 16);
#pragma unroll
            for (int d = 0; d < 4; ++d) colsum = __builtin_amdgcn_sdot4(fb[a][j][d], 0x01010101, colsum, false);
        }
        colsum += __shfl_xor(colsum, 32);
        const int32_t b = g.bias ? g.bias[co] : 0, mu = g.mult[co], sf = g.shift[co];
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

    // ---- the strip's patch of an image row: 64 aligned dwords starting at the aligned-down byte
    // column of the first tap; lane l owns dword l.  Image rows are a multiple of 4 bytes long and
    // the tensor is 4-byte aligned (dispatcher-checked), so a dword lies fully inside or outside.
    const int row_bytes = g.W * g.Cin;
    const int patch_first = (wo0 * g.sw - g.pw) * g.Cin; // may be negative
    const int phase = patch_first & 3;
    const int my_col = patch_first - phase + lane * 4;
    const bool col_inside = my_col >= 0 && my_col < row_bytes;
    const uint32_t fill = (uint32_t)g.z_a * 0x01010101u;
    const uint8_t *const img = g.A + (int64_t)n * g.H * row_bytes;
    const uint32_t my_off = (uint32_t)(col_inside ? my_col : 0);
    const uint8_t *const fill_chunk = &g_fill_table.v[g.z_a][0];
    // hi is wave-uniform: a row outside the image is read from the fill table (scalar base, no branch);
    // columns outside are replaced when the dword goes into the ring, not behind the load
    auto fetch_row = [&](int hi) -> uint32_t {
        const bool row_inside = hi >= 0 && hi < g.H;
        const uint8_t *base = row_inside ? img + (int64_t)hi * row_bytes : fill_chunk;
        const uint32_t off = row_inside ? my_off : 0u;
        return *reinterpret_cast<const __attribute__((address_space(1))) uint32_t *>((uintptr_t)(base + off));
    };
    auto ring_slot = [&](int hi) { return ring + ((hi + 64) & (RING - 1)) * ROW_BYTES; };
    // this lane's window inside a staged row
    const int win = phase + frow * g.sw * g.Cin + fhalf * 16;
    const int win_dword = win & ~3, win_shift = win & 3;

    // lane-invariant parts of the output addresses (as in shortk.h)
    int st_lds[NB], st_row[NB];
    bool st_col_ok[NB];
    uint32_t st_off[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int idx = i * 64 + lane;
        st_row[i] = idx / (2 * NB);
        const int col0 = (idx % (2 * NB)) * 16;
        st_col_ok[i] = col0 < g.N && wo0 + st_row[i] < g.Wo;
        st_lds[i] = st_row[i] * PITCH + (idx % (2 * NB)) * 16;
        st_off[i] = (uint32_t)(st_row[i] * g.N + col0);
    }
    const int put_base = (4 * fhalf + (lane & 3)) * PITCH + (frow & ~3);
    const bool chunks_whole = g.c_vec16 && (g.N & 15) == 0;
    const int quad_lane = lane & 3;
    const uint32_t sel1 = (quad_lane & 1) ? 0x03070105u : 0x06020400u;
    const uint32_t sel2 = (quad_lane & 2) ? 0x03020706u : 0x05040100u;
    auto wave_sync = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    auto store_row = [&](int ho) { // the 32 x Cout tile of output row ho, from the wave's LDS tile
        wave_sync();
        uint8_t *const out = g.C + (((int64_t)n * g.Ho + ho) * g.Wo + wo0) * g.N; // wave-uniform
        if (chunks_whole) {
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (st_col_ok[i]) *reinterpret_cast<u32x4 *>(out + st_off[i]) = *reinterpret_cast<const u32x4 *>(stage + st_lds[i]);
        } else {
#pragma nounroll
            for (int i = 0; i < NB; ++i) {
                const int idx = i * 64 + lane;
                const int row = idx / (2 * NB), ch = idx % (2 * NB);
                if (wo0 + row >= g.Wo || ch * 16 >= g.N) continue;
                uint8_t *dst = out + (int64_t)row * g.N + ch * 16;
                const uint8_t *src = stage + row * PITCH + ch * 16;
#pragma nounroll
                for (int e = 0; e < 16 && ch * 16 + e < g.N; ++e) dst[e] = src[e];
            }
        }
        wave_sync();
    };

    auto walk = [&](auto fused_tag) {
        constexpr bool FUSED = decltype(fused_tag)::value > 0, TIES = decltype(fused_tag)::value == 1; // 2: without the tie term
        // the first output row of the segment needs all KH image rows; afterwards NEW new ones
        uint32_t fresh[NEW];
        {
            uint32_t first[KH];
            const int hi0 = ho_begin * SH - g.ph;
#pragma unroll
            for (int a = 0; a < KH; ++a) first[a] = fetch_row(hi0 + a);
#pragma unroll
            for (int a = 0; a < KH - NEW; ++a)
                *reinterpret_cast<uint32_t *>(ring_slot(hi0 + a) + lane * 4) = (col_inside ? first[a] : fill) ^ 0x80808080u;
#pragma unroll
            for (int a = 0; a < NEW; ++a) fresh[a] = first[KH - NEW + a];
        }
        int ho_stored = -1;
        for (int ho = ho_begin; ho < ho_end; ++ho) {
            // ---- the newest image rows into the ring (the window reads of the previous output row are
            // done: LDS operations of one wave complete in order)
            const int fresh_first = ho * SH - g.ph + KH - NEW;
#pragma unroll
            for (int a = 0; a < NEW; ++a)
                *reinterpret_cast<uint32_t *>(ring_slot(fresh_first + a) + lane * 4) = (col_inside ? fresh[a] : fill) ^ 0x80808080u;
            wave_sync();
            // ---- previous output row's stores, then the loads for the next output row (see shortk.h);
            // behind the last row of the segment the loads repeat a row already seen (in bounds, unused)
            if (ho_stored >= 0) store_row(ho_stored);
            {
                const int next_first = (ho + 1 < ho_end ? ho + 1 : ho) * SH - g.ph + KH - NEW;
#pragma unroll
                for (int a = 0; a < NEW; ++a) fresh[a] = fetch_row(next_first + a);
            }
            // ---- one MFMA per kernel row and column block
            i32x16 acc[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[j][r] = 0;
            const int hi0 = ho * SH - g.ph;
#pragma unroll
            for (int a = 0; a < KH; ++a) {
                const uint32_t *p = reinterpret_cast<const uint32_t *>(ring_slot(hi0 + a) + win_dword);
                uint32_t d[5];
#pragma unroll
                for (int e = 0; e < 5; ++e) d[e] = p[e];
                i32x4 fa;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    fa[e] = (int32_t)__builtin_amdgcn_alignbyte(d[e + 1], d[e], (uint32_t)win_shift);
#pragma unroll
                for (int j = 0; j < NB; ++j) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb[a][j], acc[j], 0, 0, 0);
            }
            // ---- epilogue into the wave's LDS tile
            auto put = [&](int j, int q, uint32_t x) {
                uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true);
                x = __builtin_amdgcn_perm(o, x, sel1);
                o = (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, true);
                x = __builtin_amdgcn_perm(o, x, sel2);
                *reinterpret_cast<uint32_t *>(stage + put_base + q * 8 * PITCH + j * 32) = x;
            };
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const RescaleParams rp = make_rescale(c_mult[j], c_shift[j]);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint32_t x = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int32_t a = acc[j][4 * q + e];
                        if constexpr (FUSED) {
                            const int32_t t = __mulhi((int32_t)((uint32_t)(a + c_corr[j]) << 2), c_mult[j]);
                            const int32_t wv = fused_w_from_t<TIES>(t, c_c[j]);
                            x = shift_into_byte(x, med3_i32(wv, c_lo[j], c_hi[j]), c_n1[j], e);
                        } else {
                            const int32_t y = clamp_i32(g.lo_rel, g.hi_rel, rescale_general(a + c_corr[j], rp)) + g.z_out;
                            x |= (uint32_t)y << (8 * e);
                        }
                    }
                    put(j, q, x);
                }
            }
            wave_sync();
            ho_stored = ho;
        }
        if (ho_stored >= 0) store_row(ho_stored);
    };
    if (!fused) walk(std::integral_constant<int, 0>{});
    else if (g.lo_rel < 0) walk(std::integral_constant<int, 1>{});
    else walk(std::integral_constant<int, 2>{}); // act_min >= z_out: the clamp absorbs the tie term
}

} // namespace qnn
