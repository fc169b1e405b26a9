// Streaming (HBM-bound) kernels: affine quantize / de-quantize (Sec. 2.1 eq. 1-3),
// stand-alone rescale of int32 accumulators, rescaling add (Sec. 3.2.1), weight transpose.
//
// All of them move each byte once: 16-byte loads per lane, consecutive lanes on
// consecutive addresses, grid sized to a few waves per SIMD and a grid-stride loop.
#include "qnn_device.h"

namespace qnn {

constexpr int kThreads = 256;

using f32x4 = float __attribute__((ext_vector_type(4)));
using u32x4 = uint32_t __attribute__((ext_vector_type(4)));
using i32x4 = int32_t __attribute__((ext_vector_type(4)));

static int grid_for(size_t work_items, int per_block, int max_blocks = 256 * 16)
{
    size_t b = (work_items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > (size_t)max_blocks) b = max_blocks;
    return (int)b;
}

// ------------------------------------------------------------------ quantize

__device__ __forceinline__ uint32_t quantize_one(float x, float scale, float lo, float hi, int32_t z)
{
    float t = __fdiv_rn(x, scale);   // one correctly rounded binary32 division
    float r = roundf(t);             // ties away from zero
    r = (t != t) ? 0.0f : r;         // NaN behaves like 0.0
    r = r < lo ? lo : r;
    r = r > hi ? hi : r;
    return (uint32_t)((int32_t)r + z);
}

// VEC = 4: x is 16-byte aligned, q 4-byte aligned; VEC = 1: anything.
template <int VEC>
__global__ void __launch_bounds__(kThreads) quantize_kernel(const float *__restrict__ x, uint8_t *__restrict__ q,
                                                            size_t n, float scale, int32_t z, float lo, float hi)
{
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    if (VEC == 4) {
        const size_t nvec = n / 4;
        const f32x4 *xv = reinterpret_cast<const f32x4 *>(x);
        uint32_t *qv = reinterpret_cast<uint32_t *>(q);
        size_t v = tid;
        // four independent 16-byte loads in flight per lane
        for (; v + 3 * nthreads < nvec; v += 4 * nthreads) {
            f32x4 a[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) a[u] = __builtin_nontemporal_load(&xv[v + u * nthreads]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                uint32_t p = quantize_one(a[u].x, scale, lo, hi, z) | (quantize_one(a[u].y, scale, lo, hi, z) << 8) |
                             (quantize_one(a[u].z, scale, lo, hi, z) << 16) |
                             (quantize_one(a[u].w, scale, lo, hi, z) << 24);
                __builtin_nontemporal_store(p, &qv[v + u * nthreads]);
            }
        }
        for (; v < nvec; v += nthreads) {
            f32x4 a = xv[v];
            qv[v] = quantize_one(a.x, scale, lo, hi, z) | (quantize_one(a.y, scale, lo, hi, z) << 8) |
                    (quantize_one(a.z, scale, lo, hi, z) << 16) | (quantize_one(a.w, scale, lo, hi, z) << 24);
        }
        for (size_t i = nvec * 4 + tid; i < n; i += nthreads) q[i] = (uint8_t)quantize_one(x[i], scale, lo, hi, z);
    } else {
        for (size_t i = tid; i < n; i += nthreads) q[i] = (uint8_t)quantize_one(x[i], scale, lo, hi, z);
    }
}

// ------------------------------------------- ranges on the device, dynamic quantization

// Sec. 2.5: activation ranges come from the minimum and maximum of the tensor (their moving average
// across batches during training); Sec. 2.1 turns a range into (scale, zero_point).  Everything stays on
// the device: a reduction with one atomic pair per workgroup on order-preserving integer keys, a
// one-lane kernel that updates the range and derives the parameters in double precision exactly as
// qnn_choose_qparams does on the host, and a quantize kernel that reads them from memory.
__device__ __forceinline__ uint32_t float_key(float v) // monotonic: a < b  <=>  key(a) < key(b)
{
    const uint32_t b = __float_as_uint(v);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ float key_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ void minmax_init_kernel(qnn_dyn_qparams *st)
{
    st->key_min = 0xffffffffu;
    st->key_max = 0u;
}

__global__ void __launch_bounds__(kThreads) minmax_kernel(const float *__restrict__ x, size_t n, qnn_dyn_qparams *st)
{
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    float lo = INFINITY, hi = -INFINITY; // values that are not finite take no part in the range
    auto take = [&](float v) {
        if (__builtin_isfinite(v)) lo = fminf(lo, v), hi = fmaxf(hi, v);
    };
    if ((reinterpret_cast<uintptr_t>(x) & 15) == 0) {
        const size_t nvec = n / 4;
        const f32x4 *xv = reinterpret_cast<const f32x4 *>(x);
        size_t v = tid;
        for (; v + 3 * nthreads < nvec; v += 4 * nthreads) { // four independent 16-byte loads in flight per lane
            f32x4 a[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) a[u] = xv[v + u * nthreads]; // plain loads: the quantize pass reads x again
#pragma unroll
            for (int u = 0; u < 4; ++u) take(a[u].x), take(a[u].y), take(a[u].z), take(a[u].w);
        }
        for (; v < nvec; v += nthreads) {
            const f32x4 a = xv[v];
            take(a.x), take(a.y), take(a.z), take(a.w);
        }
        for (size_t i = nvec * 4 + tid; i < n; i += nthreads) take(x[i]);
    } else {
        for (size_t i = tid; i < n; i += nthreads) take(x[i]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
    }
    __shared__ float s_lo[kThreads / 64], s_hi[kThreads / 64];
    if ((threadIdx.x & 63) == 0) s_lo[threadIdx.x >> 6] = lo, s_hi[threadIdx.x >> 6] = hi;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) lo = fminf(lo, s_lo[w]), hi = fmaxf(hi, s_hi[w]);
        if (lo <= hi) { // at least one finite value in this block
            // atomics on one address serialise across the chip: skip them when the value seen so far is
            // already as good (a stale read only costs an atomic that changes nothing)
            const uint32_t klo = float_key(lo), khi = float_key(hi);
            if (klo < __hip_atomic_load(&st->key_min, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMin(&st->key_min, klo);
            if (khi > __hip_atomic_load(&st->key_max, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(&st->key_max, khi);
        }
    }
}

__device__ __forceinline__ double nearest_away_dev(double v) { return v < 0.0 ? -floor(-v + 0.5) : floor(v + 0.5); }

// range update (momentum 0: the batch range; else moving average) and quantizer parameters
__global__ void range_finalize_kernel(qnn_dyn_qparams *st, float momentum, int bits)
{
    float bmin = 0.0f, bmax = 0.0f;
    if (st->key_min <= st->key_max) bmin = key_float(st->key_min), bmax = key_float(st->key_max);
    if (momentum != 0.0f) { // m * old + (1 - m) * batch, each operation rounded once in double, then to binary32
        const double m = (double)momentum, om = __dsub_rn(1.0, m);
        bmin = (float)__dadd_rn(__dmul_rn(m, (double)st->xmin), __dmul_rn(om, (double)bmin));
        bmax = (float)__dadd_rn(__dmul_rn(m, (double)st->xmax), __dmul_rn(om, (double)bmax));
    }
    st->xmin = bmin, st->xmax = bmax;
    const double lo = fmin((double)bmin, 0.0), hi = fmax((double)bmax, 0.0);
    const double steps = (double)((1 << bits) - 1);
    if (hi - lo == 0.0) {
        st->scale = 1.0f, st->zero_point = 0;
        return;
    }
    const float sc = (float)__ddiv_rn(__dsub_rn(hi, lo), steps);
    double z = nearest_away_dev(__ddiv_rn(-lo, (double)sc));
    z = fmin(fmax(z, 0.0), steps);
    st->scale = sc, st->zero_point = (int32_t)z;
}

// quantize with parameters that live in device memory (8-bit codes)
__global__ void __launch_bounds__(kThreads) quantize_with_kernel(const float *__restrict__ x, uint8_t *__restrict__ q, size_t n,
                                                                 const qnn_dyn_qparams *__restrict__ st)
{
    const float scale = st->scale;
    const int32_t z = st->zero_point;
    const float lo = (float)(0 - z), hi = (float)(255 - z);
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    if (((reinterpret_cast<uintptr_t>(x) & 15) | (reinterpret_cast<uintptr_t>(q) & 3)) == 0) {
        const size_t nvec = n / 4;
        const f32x4 *xv = reinterpret_cast<const f32x4 *>(x);
        uint32_t *qv = reinterpret_cast<uint32_t *>(q);
        size_t v = tid;
        for (; v + 3 * nthreads < nvec; v += 4 * nthreads) {
            f32x4 a[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) a[u] = __builtin_nontemporal_load(&xv[v + u * nthreads]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t p = quantize_one(a[u].x, scale, lo, hi, z) | (quantize_one(a[u].y, scale, lo, hi, z) << 8) |
                                   (quantize_one(a[u].z, scale, lo, hi, z) << 16) |
                                   (quantize_one(a[u].w, scale, lo, hi, z) << 24);
                __builtin_nontemporal_store(p, &qv[v + u * nthreads]);
            }
        }
        for (; v < nvec; v += nthreads) {
            const f32x4 a = xv[v];
            qv[v] = quantize_one(a.x, scale, lo, hi, z) | (quantize_one(a.y, scale, lo, hi, z) << 8) |
                    (quantize_one(a.z, scale, lo, hi, z) << 16) | (quantize_one(a.w, scale, lo, hi, z) << 24);
        }
        for (size_t i = nvec * 4 + tid; i < n; i += nthreads) q[i] = (uint8_t)quantize_one(x[i], scale, lo, hi, z);
    } else {
        for (size_t i = tid; i < n; i += nthreads) q[i] = (uint8_t)quantize_one(x[i], scale, lo, hi, z);
    }
}

// ------------------------------------------------- simulated quantization (training side)

// Sec. 2.4: SimQuant = quantizer followed by de-quantizer (eq. 12-13); in the backward pass the
// quantizer is replaced by a clamp to the representable range, i.e. the incoming gradient passes
// where x_min <= x <= x_max and is zero elsewhere (straight-through estimator, eq. 14-15).
__global__ void __launch_bounds__(kThreads) simquant_kernel(const float *__restrict__ x, float *__restrict__ y, size_t n,
                                                            float scale, int32_t z, float lo, float hi)
{
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += nthreads) {
        const int32_t code = (int32_t)quantize_one(x[i], scale, lo, hi, z);
        y[i] = __fmul_rn((float)(code - z), scale);
    }
}

__global__ void __launch_bounds__(kThreads) simquant_backward_kernel(const float *__restrict__ x, const float *__restrict__ gy,
                                                                     float *__restrict__ gx, size_t n, float xmin, float xmax)
{
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += nthreads) {
        const float v = x[i];
        gx[i] = (v >= xmin && v <= xmax) ? gy[i] : 0.0f; // NaN fails both comparisons: no gradient
    }
}

// 16-bit codes (Sec. 3.3 compares activation precisions of 4, 8 and 16 bits): the same arithmetic with
// uint16 storage.  A lane handles 4 consecutive elements (16 bytes in, 8 bytes out) when the pointers
// allow it.
using u32x2 = uint32_t __attribute__((ext_vector_type(2)));

template <int VEC>
__global__ void __launch_bounds__(kThreads) quantize_u16_kernel(const float *__restrict__ x, uint16_t *__restrict__ q,
                                                                size_t n, float scale, int32_t z, float lo, float hi)
{
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    size_t done = 0;
    if (VEC == 4) {
        const size_t nvec = n / 4;
        const f32x4 *xv = reinterpret_cast<const f32x4 *>(x);
        u32x2 *qv = reinterpret_cast<u32x2 *>(q);
        for (size_t v = tid; v < nvec; v += nthreads) {
            const f32x4 a = __builtin_nontemporal_load(&xv[v]);
            u32x2 p;
            p.x = quantize_one(a.x, scale, lo, hi, z) | (quantize_one(a.y, scale, lo, hi, z) << 16);
            p.y = quantize_one(a.z, scale, lo, hi, z) | (quantize_one(a.w, scale, lo, hi, z) << 16);
            __builtin_nontemporal_store(p, &qv[v]);
        }
        done = nvec * 4;
    }
    for (size_t i = done + tid; i < n; i += nthreads) q[i] = (uint16_t)quantize_one(x[i], scale, lo, hi, z);
}

template <int VEC>
__global__ void __launch_bounds__(kThreads) dequantize_u16_kernel(const uint16_t *__restrict__ q, float *__restrict__ x,
                                                                  size_t n, float scale, int32_t z)
{
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    size_t done = 0;
    if (VEC == 4) {
        const size_t nvec = n / 4;
        const u32x2 *qv = reinterpret_cast<const u32x2 *>(q);
        f32x4 *xv = reinterpret_cast<f32x4 *>(x);
        for (size_t v = tid; v < nvec; v += nthreads) {
            const u32x2 p = __builtin_nontemporal_load(&qv[v]);
            f32x4 o;
            o.x = __fmul_rn((float)((int32_t)(p.x & 0xffffu) - z), scale);
            o.y = __fmul_rn((float)((int32_t)(p.x >> 16) - z), scale);
            o.z = __fmul_rn((float)((int32_t)(p.y & 0xffffu) - z), scale);
            o.w = __fmul_rn((float)((int32_t)(p.y >> 16) - z), scale);
            __builtin_nontemporal_store(o, &xv[v]);
        }
        done = nvec * 4;
    }
    for (size_t i = done + tid; i < n; i += nthreads) x[i] = __fmul_rn((float)((int32_t)q[i] - z), scale);
}

// ---------------------------------------------------------------- dequantize

template <int VEC>
__global__ void __launch_bounds__(kThreads) dequantize_kernel(const uint8_t *__restrict__ q, float *__restrict__ x,
                                                              size_t n, float scale, int32_t z)
{
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    if (VEC == 4) {
        const size_t nvec = n / 4;
        const uint32_t *qv = reinterpret_cast<const uint32_t *>(q);
        f32x4 *xv = reinterpret_cast<f32x4 *>(x);
        size_t v = tid;
        for (; v + 3 * nthreads < nvec; v += 4 * nthreads) {
            uint32_t p[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) p[u] = __builtin_nontemporal_load(&qv[v + u * nthreads]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                f32x4 o;
                o.x = __fmul_rn((float)((int32_t)(p[u] & 0xffu) - z), scale);
                o.y = __fmul_rn((float)((int32_t)((p[u] >> 8) & 0xffu) - z), scale);
                o.z = __fmul_rn((float)((int32_t)((p[u] >> 16) & 0xffu) - z), scale);
                o.w = __fmul_rn((float)((int32_t)(p[u] >> 24) - z), scale);
                __builtin_nontemporal_store(o, &xv[v + u * nthreads]);
            }
        }
        for (; v < nvec; v += nthreads) {
            uint32_t p = qv[v];
            f32x4 o;
            o.x = __fmul_rn((float)((int32_t)(p & 0xffu) - z), scale);
            o.y = __fmul_rn((float)((int32_t)((p >> 8) & 0xffu) - z), scale);
            o.z = __fmul_rn((float)((int32_t)((p >> 16) & 0xffu) - z), scale);
            o.w = __fmul_rn((float)((int32_t)(p >> 24) - z), scale);
            xv[v] = o;
        }
        for (size_t i = nvec * 4 + tid; i < n; i += nthreads) x[i] = __fmul_rn((float)((int32_t)q[i] - z), scale);
    } else {
        for (size_t i = tid; i < n; i += nthreads) x[i] = __fmul_rn((float)((int32_t)q[i] - z), scale);
    }
}

// ---------------------------------------------------------------- requantize

// VEC = 4: acc 16-byte aligned, y 4-byte aligned, channels % 4 == 0 (so four consecutive
// elements never straddle a row).  One lane rescales 4 accumulators and stores 4 bytes.
template <int VEC, bool PER_CHANNEL>
__global__ void __launch_bounds__(kThreads)
    requantize_kernel(const int32_t *__restrict__ acc, uint8_t *__restrict__ y, size_t total, uint32_t channels,
                      const int32_t *__restrict__ mult, const int32_t *__restrict__ shift, int32_t z_out,
                      int32_t act_min, int32_t act_max)
{
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    RescaleParams uni = make_rescale(mult[0], shift[0]);
    const int32_t uni_shift = shift[0];
    if (VEC == 4) {
        const size_t nvec = total / 4;
        const i32x4 *av = reinterpret_cast<const i32x4 *>(acc);
        uint32_t *yv = reinterpret_cast<uint32_t *>(y);
        // four accumulators of one lane -> four codes.  When every lane of the wave has 1 <= shift <= 20 and
        // |acc| < 2^29 the rescale runs in its 7-operation 32-bit form, else in the general 64-bit form.
        auto four = [&](const i32x4 a, uint32_t c) -> uint32_t {
            i32x4 m4 = {uni.mult, uni.mult, uni.mult, uni.mult}, s4 = {uni_shift, uni_shift, uni_shift, uni_shift};
            if (PER_CHANNEL) {
                m4 = *reinterpret_cast<const i32x4 *>(mult + c);
                s4 = *reinterpret_cast<const i32x4 *>(shift + c);
            }
            bool ok = true;
#pragma unroll
            for (int j = 0; j < 4; ++j) ok = ok && s4[j] >= 1 && s4[j] <= 20 && a[j] > -(1 << 29) && a[j] < (1 << 29);
            uint32_t packed = 0;
            if (__all(ok)) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int32_t n1 = s4[j] + 1;
                    FusedRescale f;
                    f.mult = m4[j], f.corr4 = 0, f.n1 = n1;
                    f.c = (1 << s4[j]) + (z_out << n1) + 1;
                    f.lo = act_min << n1;
                    f.hi = ((act_max + 1) << n1) - 1;
                    packed = shift_into_byte(packed, rescale_fused_w(a[j], f), n1, j);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const RescaleParams p = make_rescale(m4[j], s4[j]);
                    // clamp before adding z_out: the rescaled value may sit at the int32 limits
                    const int32_t r = clamp_i32(act_min - z_out, act_max - z_out, rescale_general(a[j], p)) + z_out;
                    packed |= (uint32_t)r << (8 * j);
                }
            }
            return packed;
        };
        // channel of a lane's first element, advanced without a 64-bit division per step (rows are a
        // multiple of 4 long, so a vector never straddles a row)
        const uint32_t step = PER_CHANNEL ? (uint32_t)((nthreads * 4) % channels) : 0u;
        uint32_t c = PER_CHANNEL ? (uint32_t)((tid * 4) % channels) : 0u;
        auto advance = [&](uint32_t ch) {
            ch += step;
            return ch >= channels ? ch - channels : ch;
        };
        size_t v = tid;
        for (; v + 3 * nthreads < nvec; v += 4 * nthreads) { // four independent 16-byte loads in flight per lane
            i32x4 a[4];
            uint32_t cs[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                a[u] = __builtin_nontemporal_load(&av[v + u * nthreads]);
                cs[u] = c;
                c = advance(c);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(four(a[u], cs[u]), &yv[v + u * nthreads]);
        }
        for (; v < nvec; v += nthreads) {
            yv[v] = four(av[v], c);
            c = advance(c);
        }
    } else {
        for (size_t i = tid; i < total; i += nthreads) {
            RescaleParams p = uni;
            if (PER_CHANNEL) {
                uint32_t c = (uint32_t)(i % channels);
                p = make_rescale(mult[c], shift[c]);
            }
            y[i] = (uint8_t)(clamp_i32(act_min - z_out, act_max - z_out, rescale_general(acc[i], p)) + z_out);
        }
    }
}

// ---------------------------------------------------------------------- qadd

struct QaddArgs {
    int32_t z_a, mult_a, shift_a, z_b, mult_b, shift_b, left_shift, mult_o, shift_o, z_out, act_min, act_max;
};

// The rescaled value of an input depends only on its 8-bit code, so each block first
// tabulates RESCALE((v - z) * 2^L) for the 256 codes of a and of b in LDS; the streaming
// loop is then two table reads, an add and one rescale per element.
// FUSED: the output rescale may use the 32-bit fused form (1 <= shift_o <= 20 and both tables
// bounded by 2^28, which shift_a, shift_b >= 0 and left_shift <= 20 guarantee).
template <int VEC, bool FUSED>
__global__ void __launch_bounds__(kThreads) qadd_kernel(const uint8_t *__restrict__ a, const uint8_t *__restrict__ b,
                                                        uint8_t *__restrict__ y, size_t n, QaddArgs g)
{
    __shared__ int32_t tab_a[256];
    __shared__ int32_t tab_b[256];
    {
        const int v = threadIdx.x; // kThreads == 256
        tab_a[v] = rescale_general((v - g.z_a) * (1 << g.left_shift), make_rescale(g.mult_a, g.shift_a));
        tab_b[v] = rescale_general((v - g.z_b) * (1 << g.left_shift), make_rescale(g.mult_b, g.shift_b));
    }
    __syncthreads();
    const RescaleParams po = make_rescale(g.mult_o, g.shift_o);
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    const FusedRescale fo = make_fused(g.mult_o, g.shift_o, 0, g.z_out, g.act_min, g.act_max);
    auto one = [&](uint32_t ca, uint32_t cb) -> uint32_t {
        if (FUSED) return (uint32_t)rescale_fused(tab_a[ca] + tab_b[cb], fo);
        int64_t u = (int64_t)tab_a[ca] + (int64_t)tab_b[cb];
        u = u > INT32_MAX ? INT32_MAX : (u < INT32_MIN ? INT32_MIN : u);
        return (uint32_t)(clamp_i32(g.act_min - g.z_out, g.act_max - g.z_out, rescale_general((int32_t)u, po)) + g.z_out);
    };
    if (VEC == 16) {
        const size_t nvec = n / 16;
        const u32x4 *av = reinterpret_cast<const u32x4 *>(a);
        const u32x4 *bv = reinterpret_cast<const u32x4 *>(b);
        u32x4 *yv = reinterpret_cast<u32x4 *>(y);
        for (size_t v = tid; v < nvec; v += nthreads) {
            u32x4 pa = __builtin_nontemporal_load(&av[v]);
            u32x4 pb = __builtin_nontemporal_load(&bv[v]);
            const uint32_t wa[4] = {pa.x, pa.y, pa.z, pa.w};
            const uint32_t wb[4] = {pb.x, pb.y, pb.z, pb.w};
            uint32_t wo[4];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                uint32_t o = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) o |= one((wa[d] >> (8 * j)) & 0xffu, (wb[d] >> (8 * j)) & 0xffu) << (8 * j);
                wo[d] = o;
            }
            u32x4 out = {wo[0], wo[1], wo[2], wo[3]};
            __builtin_nontemporal_store(out, &yv[v]);
        }
        for (size_t i = nvec * 16 + tid; i < n; i += nthreads) y[i] = (uint8_t)one(a[i], b[i]);
    } else {
        for (size_t i = tid; i < n; i += nthreads) y[i] = (uint8_t)one(a[i], b[i]);
    }
}


// ------------------------------------------------------ rescale of uint8 codes (concat)

// Sec. 3.2.1: the inputs of a concatenation carry different quantizers and must be brought to the
// output's before they are laid side by side.  y[m][c] = clamp(z_out + RESCALE(x[m][c] - z_in)) is a
// function of one 8-bit code: a 256-entry byte table per workgroup, one gather per element.  Rows
// have their own pitches, so the destination can be a channel slice of the concatenated tensor.
__global__ void __launch_bounds__(kThreads) rescale_u8_kernel(const uint8_t *__restrict__ x, int64_t ldx, uint8_t *__restrict__ y,
                                                              int64_t ldy, int64_t rows, int64_t cols, int32_t z_in, int32_t mult,
                                                              int32_t shift, int32_t z_out, int32_t act_min, int32_t act_max,
                                                              int vec16)
{
    __shared__ uint8_t lut[256];
    {
        const int v = threadIdx.x; // kThreads == 256
        const int32_t r = rescale_general(v - z_in, make_rescale(mult, shift));
        lut[v] = (uint8_t)(clamp_i32(act_min - z_out, act_max - z_out, r) + z_out);
    }
    __syncthreads();
    const int64_t chunks_per_row = (cols + 15) / 16, total = rows * chunks_per_row;
    for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < total; q += (int64_t)gridDim.x * kThreads) {
        const int64_t m = q / chunks_per_row;
        const int64_t c = (q - m * chunks_per_row) * 16;
        const uint8_t *xp = x + m * ldx + c;
        uint8_t *yp = y + m * ldy + c;
        if (vec16 && c + 16 <= cols) {
            const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(xp));
            u32x4 o;
#pragma unroll
            for (int d = 0; d < 4; ++d)
                o[d] = (uint32_t)lut[a[d] & 0xffu] | ((uint32_t)lut[(a[d] >> 8) & 0xffu] << 8) |
                       ((uint32_t)lut[(a[d] >> 16) & 0xffu] << 16) | ((uint32_t)lut[a[d] >> 24] << 24);
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(yp));
        } else {
            for (int e = 0; e < 16 && c + e < cols; ++e) yp[e] = lut[xp[e]];
        }
    }
}

// ------------------------------------------------ add behind a product, second-pass form

// y = ADD(y, r) row by row, in place (each 16-byte chunk is read, combined and written by one lane)
template <bool FUSED>
__global__ void __launch_bounds__(kThreads) add_inplace_kernel(uint8_t *y, int64_t ldy, const uint8_t *r, int64_t ldr,
                                                               int64_t M, int64_t N, AddParams p, int vec16)
{
    __shared__ int32_t tab[512];
    add_fill_tables(tab, p, threadIdx.x, kThreads);
    __syncthreads();
    const AddOut ao = make_add_out(p);
    const int64_t chunks_per_row = (N + 15) / 16, total = M * chunks_per_row;
    for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < total; q += (int64_t)gridDim.x * kThreads) {
        const int64_t m = q / chunks_per_row;
        const int64_t n = (q - m * chunks_per_row) * 16;
        uint8_t *yp = y + m * ldy + n;
        const uint8_t *rp = r + m * ldr + n;
        if (vec16 && n + 16 <= N) {
            const u32x4 a = *reinterpret_cast<const u32x4 *>(yp), b = *reinterpret_cast<const u32x4 *>(rp);
            u32x4 o;
#pragma unroll
            for (int d = 0; d < 4; ++d) o[d] = add_codes4<FUSED>(a[d], b[d], tab, ao);
            *reinterpret_cast<u32x4 *>(yp) = o;
        } else {
            for (int e = 0; e < 16 && n + e < N; ++e) yp[e] = (uint8_t)add_code1<FUSED>(yp[e], rp[e], tab, ao);
        }
    }
}

// ------------------------------------------------------------------- pack_b

// dst[n][k] = src[k][n], 64x64 byte tiles through LDS so both sides are coalesced
__global__ void __launch_bounds__(kThreads) pack_b_kernel(const int8_t *__restrict__ src, int64_t ld_src, int64_t K,
                                                          int64_t N, int8_t *__restrict__ dst, int64_t ld_dst)
{
    __shared__ int8_t tile[64][65];
    const int64_t k0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
        const int64_t k = k0 + r, n = n0 + tx;
        tile[r][tx] = (k < K && n < N) ? src[k * ld_src + n] : (int8_t)0;
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        const int64_t n = n0 + r, k = k0 + tx;
        if (n < N && k < K) dst[n * ld_dst + k] = tile[tx][r];
    }
}

static bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

qnn_status launch_add_inplace(uint8_t *y, int64_t ldy, const uint8_t *r, int64_t ldr, int64_t M, int32_t N,
                              const AddParams &p, hipStream_t s)
{
    int64_t rows = M, cols = N;
    if (ldy == N && ldr == N) rows = 1, cols = M * (int64_t)N, ldy = ldr = cols; // dense: one long row, whole chunks throughout
    const int vec16 = aligned(y, 16) && aligned(r, 16) && (rows == 1 || ((ldy % 16) == 0 && (ldr % 16) == 0));
    const size_t chunks = (size_t)rows * (size_t)((cols + 15) / 16);
    const int grid = grid_for(chunks, kThreads * 2);
    const bool fused = p.shift_o >= 1 && p.shift_o <= 20 && p.shift_m >= 0 && p.shift_r >= 0 && p.left_shift <= 20;
    if (fused) hipLaunchKernelGGL((add_inplace_kernel<true>), dim3(grid), dim3(kThreads), 0, s, y, ldy, r, ldr, rows, cols, p, vec16);
    else hipLaunchKernelGGL((add_inplace_kernel<false>), dim3(grid), dim3(kThreads), 0, s, y, ldy, r, ldr, rows, cols, p, vec16);
    return launch_status(hipGetLastError());
}

} // namespace qnn

using namespace qnn;

extern "C" {

qnn_status qnn_quantize(const float *x, uint8_t *q, size_t n, float scale, int32_t zero_point, int32_t qmin,
                        int32_t qmax, void *stream)
{
    if (!(scale > 0.0f) || __builtin_isinf(scale)) return QNN_EINVAL;
    if (qmin < 0 || qmax > 255 || qmin > qmax || zero_point < qmin || zero_point > qmax) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (!x || !q) return QNN_EINVAL;
    const float lo = (float)(qmin - zero_point), hi = (float)(qmax - zero_point);
    if (aligned(x, 16) && aligned(q, 4)) {
        const int grid = grid_for(n / 4 + 1, kThreads * 4);
        hipLaunchKernelGGL(quantize_kernel<4>, dim3(grid), dim3(kThreads), 0, as_stream(stream), x, q, n, scale,
                           zero_point, lo, hi);
    } else {
        hipLaunchKernelGGL(quantize_kernel<1>, dim3(grid_for(n, kThreads * 4)), dim3(kThreads), 0, as_stream(stream),
                           x, q, n, scale, zero_point, lo, hi);
    }
    return launch_status(hipGetLastError());
}

qnn_status qnn_dequantize(const uint8_t *q, float *x, size_t n, float scale, int32_t zero_point, void *stream)
{
    if (!(scale > 0.0f) || __builtin_isinf(scale) || zero_point < 0 || zero_point > 255) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (!x || !q) return QNN_EINVAL;
    if (aligned(x, 16) && aligned(q, 4)) {
        hipLaunchKernelGGL(dequantize_kernel<4>, dim3(grid_for(n / 4 + 1, kThreads * 4)), dim3(kThreads), 0,
                           as_stream(stream), q, x, n, scale, zero_point);
    } else {
        hipLaunchKernelGGL(dequantize_kernel<1>, dim3(grid_for(n, kThreads * 4)), dim3(kThreads), 0,
                           as_stream(stream), q, x, n, scale, zero_point);
    }
    return launch_status(hipGetLastError());
}

qnn_status qnn_quantize_u16(const float *x, uint16_t *q, size_t n, float scale, int32_t zero_point, int32_t qmin,
                            int32_t qmax, void *stream)
{
    if (!(scale > 0.0f) || __builtin_isinf(scale)) return QNN_EINVAL;
    if (qmin < 0 || qmax > 65535 || qmin > qmax || zero_point < qmin || zero_point > qmax) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (!x || !q) return QNN_EINVAL;
    const float lo = (float)(qmin - zero_point), hi = (float)(qmax - zero_point);
    if (aligned(x, 16) && aligned(q, 8))
        hipLaunchKernelGGL(quantize_u16_kernel<4>, dim3(grid_for(n / 4 + 1, kThreads * 4)), dim3(kThreads), 0,
                           as_stream(stream), x, q, n, scale, zero_point, lo, hi);
    else
        hipLaunchKernelGGL(quantize_u16_kernel<1>, dim3(grid_for(n, kThreads * 4)), dim3(kThreads), 0, as_stream(stream),
                           x, q, n, scale, zero_point, lo, hi);
    return launch_status(hipGetLastError());
}

qnn_status qnn_dequantize_u16(const uint16_t *q, float *x, size_t n, float scale, int32_t zero_point, void *stream)
{
    if (!(scale > 0.0f) || __builtin_isinf(scale) || zero_point < 0 || zero_point > 65535) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (!x || !q) return QNN_EINVAL;
    if (aligned(x, 16) && aligned(q, 8))
        hipLaunchKernelGGL(dequantize_u16_kernel<4>, dim3(grid_for(n / 4 + 1, kThreads * 4)), dim3(kThreads), 0,
                           as_stream(stream), q, x, n, scale, zero_point);
    else
        hipLaunchKernelGGL(dequantize_u16_kernel<1>, dim3(grid_for(n, kThreads * 4)), dim3(kThreads), 0,
                           as_stream(stream), q, x, n, scale, zero_point);
    return launch_status(hipGetLastError());
}

qnn_status qnn_requantize(const int32_t *acc, uint8_t *y, size_t rows, size_t channels, const int32_t *mult,
                          const int32_t *shift, int per_channel, int32_t z_out, int32_t act_min, int32_t act_max,
                          void *stream)
{
    if (!acc || !y || !mult || !shift || rows == 0 || channels == 0 || channels > 0x7fffffffu) return QNN_EINVAL;
    if (bad_out_range(z_out, act_min, act_max)) return QNN_EINVAL;
    const size_t total = rows * channels;
    const bool vec = aligned(acc, 16) && aligned(y, 4) && (channels % 4 == 0) && aligned(mult, 16) && aligned(shift, 16);
    const hipStream_t s = as_stream(stream);
    const uint32_t ch = (uint32_t)channels;
    if (vec) {
        const int grid = grid_for(total / 4, kThreads * 2);
        if (per_channel)
            hipLaunchKernelGGL((requantize_kernel<4, true>), dim3(grid), dim3(kThreads), 0, s, acc, y, total, ch, mult,
                               shift, z_out, act_min, act_max);
        else
            hipLaunchKernelGGL((requantize_kernel<4, false>), dim3(grid), dim3(kThreads), 0, s, acc, y, total, ch,
                               mult, shift, z_out, act_min, act_max);
    } else {
        const int grid = grid_for(total, kThreads * 4);
        if (per_channel)
            hipLaunchKernelGGL((requantize_kernel<1, true>), dim3(grid), dim3(kThreads), 0, s, acc, y, total, ch, mult,
                               shift, z_out, act_min, act_max);
        else
            hipLaunchKernelGGL((requantize_kernel<1, false>), dim3(grid), dim3(kThreads), 0, s, acc, y, total, ch,
                               mult, shift, z_out, act_min, act_max);
    }
    return launch_status(hipGetLastError());
}

qnn_status qnn_minmax(const float *x, size_t n, float momentum, int bits, qnn_dyn_qparams *state, void *stream)
{
    if (!state || (n && !x) || bits < 2 || bits > 16 || !(momentum >= 0.0f) || !(momentum < 1.0f)) return QNN_EINVAL;
    const hipStream_t s = as_stream(stream);
    hipLaunchKernelGGL(minmax_init_kernel, dim3(1), dim3(1), 0, s, state);
    if (n) hipLaunchKernelGGL(minmax_kernel, dim3(grid_for(n / 4 + 1, kThreads * 4, 256 * 8)), dim3(kThreads), 0, s, x, n, state);
    hipLaunchKernelGGL(range_finalize_kernel, dim3(1), dim3(1), 0, s, state, momentum, bits);
    return launch_status(hipGetLastError());
}

qnn_status qnn_quantize_with(const float *x, uint8_t *q, size_t n, const qnn_dyn_qparams *state, void *stream)
{
    if (!state) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (!x || !q) return QNN_EINVAL;
    hipLaunchKernelGGL(quantize_with_kernel, dim3(grid_for(n / 4 + 1, kThreads * 4)), dim3(kThreads), 0, as_stream(stream), x, q,
                       n, state);
    return launch_status(hipGetLastError());
}

qnn_status qnn_quantize_dynamic(const float *x, uint8_t *q, size_t n, qnn_dyn_qparams *state, void *stream)
{
    if (n && (!x || !q)) return QNN_EINVAL;
    const qnn_status st = qnn_minmax(x, n, 0.0f, 8, state, stream);
    return st != QNN_OK ? st : qnn_quantize_with(x, q, n, state, stream);
}

qnn_status qnn_simquant(const float *x, float *y, size_t n, float scale, int32_t zero_point, int32_t qmin, int32_t qmax,
                        void *stream)
{
    if (!(scale > 0.0f) || __builtin_isinf(scale) || qmin < 0 || qmax > 65535 || qmin > qmax) return QNN_EINVAL;
    if (zero_point < qmin || zero_point > qmax) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (!x || !y) return QNN_EINVAL;
    hipLaunchKernelGGL(simquant_kernel, dim3(grid_for(n, kThreads * 4)), dim3(kThreads), 0, as_stream(stream), x, y, n, scale,
                       zero_point, (float)(qmin - zero_point), (float)(qmax - zero_point));
    return launch_status(hipGetLastError());
}

qnn_status qnn_simquant_backward(const float *x, const float *grad_y, float *grad_x, size_t n, float scale,
                                 int32_t zero_point, int32_t qmin, int32_t qmax, void *stream)
{
    if (!(scale > 0.0f) || __builtin_isinf(scale) || qmin < 0 || qmax > 65535 || qmin > qmax) return QNN_EINVAL;
    if (zero_point < qmin || zero_point > qmax) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (!x || !grad_y || !grad_x) return QNN_EINVAL;
    // the ends of the representable range are the de-quantized extreme codes (one binary32 product each)
    const float xmin = (float)(qmin - zero_point) * scale, xmax = (float)(qmax - zero_point) * scale;
    hipLaunchKernelGGL(simquant_backward_kernel, dim3(grid_for(n, kThreads * 4)), dim3(kThreads), 0, as_stream(stream), x, grad_y,
                       grad_x, n, xmin, xmax);
    return launch_status(hipGetLastError());
}

qnn_status qnn_rescale_u8(const uint8_t *x, int64_t ldx, int32_t z_in, int32_t mult, int32_t shift, int32_t z_out,
                          int32_t act_min, int32_t act_max, uint8_t *y, int64_t ldy, int64_t rows, int64_t cols, void *stream)
{
    if (rows < 0 || cols < 0 || z_in < 0 || z_in > 255 || shift < -31 || shift > 31) return QNN_EINVAL;
    if (bad_out_range(z_out, act_min, act_max)) return QNN_EINVAL;
    if (rows == 0 || cols == 0) return QNN_OK;
    if (!x || !y || ldx < cols || ldy < cols) return QNN_EINVAL;
    int64_t r = rows, c = cols;
    if (ldx == cols && ldy == cols) r = 1, c = rows * cols, ldx = ldy = c; // dense: one long row, whole chunks throughout
    const int vec16 = aligned(x, 16) && aligned(y, 16) && (r == 1 || ((ldx % 16) == 0 && (ldy % 16) == 0));
    const size_t chunks = (size_t)r * (size_t)((c + 15) / 16);
    hipLaunchKernelGGL(rescale_u8_kernel, dim3(grid_for(chunks, kThreads * 2)), dim3(kThreads), 0, as_stream(stream), x, ldx, y, ldy,
                       r, c, z_in, mult, shift, z_out, act_min, act_max, vec16);
    return launch_status(hipGetLastError());
}

qnn_status qnn_qadd(const uint8_t *a, int32_t z_a, int32_t mult_a, int32_t shift_a, const uint8_t *b, int32_t z_b,
                    int32_t mult_b, int32_t shift_b, int32_t left_shift, int32_t mult_o, int32_t shift_o,
                    int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *y, size_t n, void *stream)
{
    if (left_shift < 0 || left_shift > 22 || z_a < 0 || z_a > 255 || z_b < 0 || z_b > 255) return QNN_EINVAL;
    if (bad_out_range(z_out, act_min, act_max)) return QNN_EINVAL;
    auto bad_shift = [](int32_t s) { return s < -31 || s > 31; };
    if (bad_shift(shift_a) || bad_shift(shift_b) || bad_shift(shift_o)) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (!a || !b || !y) return QNN_EINVAL;
    QaddArgs g = {z_a, mult_a, shift_a, z_b, mult_b, shift_b, left_shift, mult_o, shift_o, z_out, act_min, act_max};
    const bool fused = shift_o >= 1 && shift_o <= 20 && shift_a >= 0 && shift_b >= 0 && left_shift <= 20;
    const hipStream_t s = as_stream(stream);
    if (aligned(a, 16) && aligned(b, 16) && aligned(y, 16)) {
        const int grid = grid_for(n / 16 + 1, kThreads * 2);
        if (fused) hipLaunchKernelGGL((qadd_kernel<16, true>), dim3(grid), dim3(kThreads), 0, s, a, b, y, n, g);
        else hipLaunchKernelGGL((qadd_kernel<16, false>), dim3(grid), dim3(kThreads), 0, s, a, b, y, n, g);
    } else {
        const int grid = grid_for(n, kThreads * 4);
        if (fused) hipLaunchKernelGGL((qadd_kernel<1, true>), dim3(grid), dim3(kThreads), 0, s, a, b, y, n, g);
        else hipLaunchKernelGGL((qadd_kernel<1, false>), dim3(grid), dim3(kThreads), 0, s, a, b, y, n, g);
    }
    return launch_status(hipGetLastError());
}

qnn_status qnn_pack_b(const int8_t *src, int64_t ld_src, int64_t K, int64_t N, int8_t *dst, int64_t ld_dst,
                      void *stream)
{
    if (!src || !dst || K <= 0 || N <= 0 || ld_src < N || ld_dst < K) return QNN_EINVAL;
    if ((N + 63) / 64 > 0x7fffffff || (K + 63) / 64 > 65535) return QNN_EINVAL;
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)((K + 63) / 64));
    hipLaunchKernelGGL(pack_b_kernel, grid, dim3(kThreads), 0, as_stream(stream), src, ld_src, K, N, dst, ld_dst);
    return launch_status(hipGetLastError());
}

} // extern "C"
