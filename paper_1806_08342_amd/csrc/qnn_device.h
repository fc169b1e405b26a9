// Shared device-side pieces of the gfx950 kernels: launch checking and the exact
// fixed-point rescale that every epilogue uses.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/qnn.h"

namespace qnn {

// records the HIP error text for qnn_last_error() and maps it to QNN_ELAUNCH
qnn_status launch_status(hipError_t e);
// text that qnn_last_error() returns on this thread until the next failing call
void set_last_error(const char *text);

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline bool bad_out_range(int32_t z_out, int32_t act_min, int32_t act_max)
{
    return act_min < 0 || act_max > 255 || act_min > act_max || z_out < 0 || z_out > 255;
}

// Per-channel constants of the rescale, prepared once per lane and reused for
// every accumulator of that channel.
struct RescaleParams {
    int32_t mult;
    int32_t rshift;   // max(shift, 0)
    int32_t lshift;   // max(-shift, 0)
    int32_t half;     // 2^(rshift-1), 0 when rshift == 0
    int32_t sgn_mask; // -1 when rshift > 0 else 0
};

__device__ __forceinline__ RescaleParams make_rescale(int32_t mult, int32_t shift)
{
    RescaleParams p;
    p.mult = mult;
    // per-channel parameters live in device memory and cannot be validated by the host: keep the shift
    // counts below inside what a 32-bit shift defines
    shift = shift < -31 ? -31 : (shift > 31 ? 31 : shift);
    p.rshift = shift > 0 ? shift : 0;
    p.lshift = shift < 0 ? -shift : 0;
    p.half = p.rshift ? (1 << (p.rshift - 1)) : 0;
    p.sgn_mask = p.rshift ? -1 : 0;
    return p;
}

// General form: any int32 a, any mult, shift in [-31, 31].
__device__ __forceinline__ int32_t rescale_general(int32_t a, const RescaleParams &p)
{
    if (p.lshift) {
        int64_t t = (int64_t)a << p.lshift;
        t = t > INT32_MAX ? INT32_MAX : t;
        t = t < INT32_MIN ? INT32_MIN : t;
        a = (int32_t)t;
    }
    // nearest(a*mult / 2^31), ties toward +inf: floor((a*mult + 2^30) / 2^31) in exact 64-bit
    int64_t prod = (int64_t)a * (int64_t)p.mult + (int64_t(1) << 30);
    int32_t h = (int32_t)(prod >> 31);
    if (a == INT32_MIN && p.mult == INT32_MIN) h = INT32_MAX;
    // nearest(h / 2^n), ties away from zero: (h + 2^(n-1) - [h < 0]) >> n, in 64 bits
    int64_t t = (int64_t)h + (int64_t)p.half + (int64_t)((h >> 31) & p.sgn_mask);
    return (int32_t)(t >> p.rshift);
}

// Fast form, valid when shift >= 0 and |a| < 2^30: then |h| <= |a| < 2^30 and
// h + 2^(n-1) cannot leave int32, so the second stage runs in 32 bits.
__device__ __forceinline__ int32_t rescale_fast(int32_t a, const RescaleParams &p)
{
    int64_t prod = (int64_t)a * (int64_t)p.mult + (int64_t(1) << 30);
    int32_t h = (int32_t)(prod >> 31);
    int32_t t = h + p.half + ((h >> 31) & p.sgn_mask);
    return t >> p.rshift;
}

// Fused fast form used by the conv / GEMM epilogues, valid when 1 <= shift <= 20,
// |acc + corr| < 2^29 and 0 <= act_min <= act_max <= 255.  With a = acc + corr, n = shift:
//   T = hi32(4a * mult) = floor(a*mult / 2^30)     so  nearest(a*mult/2^31), ties up  = (T + 1) >> 1
//   s = T >> 31 (0 or -1)                          and z_out + nearest(h/2^n), ties away from zero,
//   w = T + 2s + c,  c = 2*(2^(n-1) + (z_out << n)) + 1            is  w >> (n + 1)
// (two nested floor divisions by powers of two collapse into one; taking the sign from T
// instead of T + 1 changes nothing, the two differ only at T = -1 where both give z_out).
// The clamp is applied to w, against act_min << (n+1) and ((act_max + 1) << (n+1)) - 1, so
// that the final shift can write its byte straight into a packed dword (shift_into_byte).
// Only full-rate 32-bit operations.
struct FusedRescale {
    int32_t mult, corr4, c, n1, lo, hi; // corr4 = 4*corr, n1 = n + 1, lo / hi = clamp bounds of w
};

__device__ __forceinline__ FusedRescale make_fused(int32_t mult, int32_t shift, int32_t corr, int32_t z_out,
                                                  int32_t act_min, int32_t act_max)
{
    const int nn = (shift >= 1 && shift <= 20) ? shift : 1; // callers check the range; keep shifts defined
    FusedRescale f;
    f.mult = mult;
    f.corr4 = (int32_t)((uint32_t)corr << 2);
    f.c = 2 * ((1 << (nn - 1)) + (z_out << nn)) + 1;
    f.n1 = nn + 1;
    f.lo = act_min << (nn + 1);
    f.hi = ((act_max + 1) << (nn + 1)) - 1;
    return f;
}

// w of the comment above from T.  TIES = false drops the term 2s (two instructions fewer).  That
// is exact whenever act_min >= z_out (every ReLU-like output range): the term only acts for T < 0,
// where both T + c and T - 2 + c stay below (z_out + 1) << (n+1) <= (act_min + 1) << (n+1), so
// after the clamp from below the shifted result is act_min either way.
template <bool TIES> __device__ __forceinline__ int32_t fused_w_from_t(int32_t t, int32_t c)
{
    if constexpr (TIES) return (int32_t)(((uint32_t)(t >> 31) << 1) + (uint32_t)t + (uint32_t)c);
    else return (int32_t)((uint32_t)t + (uint32_t)c);
}

// w of the comment above, clamped; the caller shifts it right by n1
__device__ __forceinline__ int32_t med3_i32(int32_t v, int32_t lo, int32_t hi);
template <bool TIES = true> __device__ __forceinline__ int32_t rescale_fused_w(int32_t acc, const FusedRescale &p)
{
    const int32_t a4 = (int32_t)(((uint32_t)acc << 2) + (uint32_t)p.corr4);
    const int32_t t = __mulhi(a4, p.mult);
    return med3_i32(fused_w_from_t<TIES>(t, p.c), p.lo, p.hi);
}

// complete value (already clamped to [act_min, act_max])
__device__ __forceinline__ int32_t rescale_fused(int32_t acc, const FusedRescale &p)
{
    return rescale_fused_w(acc, p) >> p.n1;
}

// arithmetic shift right whose result byte lands in byte `byte` of `packed` (sub-dword addressing)
__device__ __forceinline__ uint32_t shift_into_byte(uint32_t packed, int32_t x, int32_t n1, int byte)
{
    // packed.byte[byte] = (x >> n1) & 0xff, other bytes kept (byte 0: cleared): one sub-dword-addressed shift
    switch (byte) {
    case 0: asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:DWORD" : "=v"(packed) : "v"(n1), "v"(x)); break; // other bytes cleared
    case 1: asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(packed) : "v"(n1), "v"(x)); break;
    case 2: asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(packed) : "v"(n1), "v"(x)); break;
    default: asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(packed) : "v"(n1), "v"(x)); break;
    }
    return packed;
}

// median of three = clamp(lo, hi, v) for lo <= hi, one instruction
__device__ __forceinline__ int32_t med3_i32(int32_t v, int32_t lo, int32_t hi)
{
    int32_t r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}

__device__ __forceinline__ int32_t clamp_i32(int32_t lo, int32_t hi, int32_t v)
{
    return v < lo ? lo : (v > hi ? hi : v);
}

// ---- rescaling add behind a product (the residual connection of Sec. 3.2.1 fused into the
// producing layer, as Sec. 3.2.1 and the operator-fusion recommendation of Sec. 7 advise).  The product's uint8
// code m (its own scale and zero-point) and the residual's code r are brought to a common scale
// and summed: RESCALE_o(RESCALE_m((m - z_m) << L) + RESCALE_r((r - z_r) << L)) + z_out, clamped.
// The two inner values depend only on an 8-bit code: 2 x 256 entries, tabulated once per workgroup.
struct AddParams {
    int32_t z_m, mult_m, shift_m; // the product's code enters the add with these
    int32_t z_r, mult_r, shift_r; // the residual operand
    int32_t left_shift, mult_o, shift_o, z_out, act_min, act_max;
};

// tab[0..255]: codes of the product, tab[256..511]: codes of the residual (LDS, 2 KB)
__device__ __forceinline__ void add_fill_tables(int32_t *tab, const AddParams &p, int tid, int nthreads)
{
    for (int v = tid; v < 512; v += nthreads) {
        const bool res = v >= 256;
        const int32_t d = (v & 255) - (res ? p.z_r : p.z_m);
        tab[v] = rescale_general(d * (1 << p.left_shift), make_rescale(res ? p.mult_r : p.mult_m, res ? p.shift_r : p.shift_m));
    }
}

struct AddOut {
    FusedRescale fo;
    RescaleParams po;
    int32_t z_out, lo_rel, hi_rel;
    bool fused; // both table ranges below 2^28 and 1 <= shift_o <= 20: the 32-bit form is exact
};

__device__ __forceinline__ AddOut make_add_out(const AddParams &p)
{
    AddOut o;
    o.fo = make_fused(p.mult_o, p.shift_o, 0, p.z_out, p.act_min, p.act_max);
    o.po = make_rescale(p.mult_o, p.shift_o);
    o.z_out = p.z_out, o.lo_rel = p.act_min - p.z_out, o.hi_rel = p.act_max - p.z_out;
    o.fused = p.shift_o >= 1 && p.shift_o <= 20 && p.shift_m >= 0 && p.shift_r >= 0 && p.left_shift <= 20;
    return o;
}

// one code of the product + one of the residual -> one output code
template <bool FUSED> __device__ __forceinline__ uint32_t add_code1(uint32_t m, uint32_t r, const int32_t *tab, const AddOut &o)
{
    const int32_t tm = tab[m], tr = tab[256 + r];
    if constexpr (FUSED) {
        return (uint32_t)rescale_fused(tm + tr, o.fo);
    } else {
        int64_t u = (int64_t)tm + (int64_t)tr;
        u = u > INT32_MAX ? INT32_MAX : (u < INT32_MIN ? INT32_MIN : u);
        return (uint32_t)(clamp_i32(o.lo_rel, o.hi_rel, rescale_general((int32_t)u, o.po)) + o.z_out);
    }
}

// four codes of the product (bytes of m) + four of the residual (bytes of r) -> four output codes
template <bool FUSED> __device__ __forceinline__ uint32_t add_codes4(uint32_t m, uint32_t r, const int32_t *tab, const AddOut &o)
{
    uint32_t x = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int32_t tm = tab[(m >> (8 * e)) & 0xffu], tr = tab[256 + ((r >> (8 * e)) & 0xffu)];
        if constexpr (FUSED) {
            x = shift_into_byte(x, rescale_fused_w(tm + tr, o.fo), o.fo.n1, e);
        } else {
            int64_t u = (int64_t)tm + (int64_t)tr;
            u = u > INT32_MAX ? INT32_MAX : (u < INT32_MIN ? INT32_MIN : u);
            x |= (uint32_t)(clamp_i32(o.lo_rel, o.hi_rel, rescale_general((int32_t)u, o.po)) + o.z_out) << (8 * e);
        }
    }
    return x;
}

// y[m][n] = ADD(y[m][n], r[m][n]) in place (elementwise.hip): the second pass of the kernels that
// do not apply the add themselves
qnn_status launch_add_inplace(uint8_t *y, int64_t ldy, const uint8_t *r, int64_t ldr, int64_t M, int32_t N,
                              const AddParams &p, hipStream_t s);

} // namespace qnn
