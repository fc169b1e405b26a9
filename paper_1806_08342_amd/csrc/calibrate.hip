// Calibration kernels for the benchmark: what this very machine sustains on the two resources
// the hot path is bounded by, measured in the same process as the kernels they are compared with.
//   qnn_calibrate_mfma: a register-only loop of v_mfma_i32_32x32x32_i8 (no memory traffic at all);
//   qnn_calibrate_copy: a plain copy with 16 bytes per lane per access;
//   qnn_calibrate_rescale: the exact rescale of the epilogues (its cheapest form) on registers only:
//     how many accumulators per second the vector ALU of the chip can turn into output bytes.
// None is part of the inference path.
#include "igemm.h"

namespace qnn {

// Every wave keeps 4 independent 32x32 accumulators busy for `iters` rounds (2 waves per SIMD when
// launched with 512 threads per CU).  random_operands != 0: the operand registers hold a different
// pseudo-random byte pattern per lane (what real activations and weights look like to the
// datapath); 0: all operand bytes are equal.  One value per lane is stored so that the loop has
// an observable result.
__global__ void __launch_bounds__(512) calibrate_mfma_kernel(int iters, int random_operands, int32_t *sink)
{
    const uint32_t id = blockIdx.x * 512u + threadIdx.x;
    i32x4 a[2], b[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t h = (id * 8u + i * 4u + d + 1u) * 2654435761u;
            h ^= h >> 15, h *= 2246822519u, h ^= h >> 13;
            a[i][d] = random_operands ? (int32_t)h : 0x01010101;
            b[i][d] = random_operands ? (int32_t)(h * 3266489917u) : 0x02020202;
        }
    i32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    int32_t t = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) t += acc[i][j][r];
    sink[id] = t;
}

__global__ void __launch_bounds__(256) calibrate_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t chunks)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < chunks; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Every lane rescales 16 independent accumulators per round with the instruction sequence the
// epilogues use when act_min >= z_out (add + shift, high multiply, add, 3-way median, shift into a
// byte of the packed dword) and feeds the packed dwords back into the accumulators, so that nothing
// can be hoisted out of the loop.  No memory traffic inside the loop.
__global__ void __launch_bounds__(256) calibrate_rescale_kernel(int iters, int32_t mult, int32_t shift, int32_t *sink)
{
    const uint32_t id = blockIdx.x * 256u + threadIdx.x;
    int32_t acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        uint32_t h = (id * 16u + i + 1u) * 2654435761u;
        h ^= h >> 15, h *= 2246822519u, h ^= h >> 13;
        acc[i] = (int32_t)(h >> 10) - (1 << 21); // |acc| < 2^21, as after a K <= 256 reduction
    }
    const FusedRescale p = make_fused(mult, shift, (int32_t)(id & 1023u), 3, 3, 255);
    for (int it = 0; it < iters; ++it) {
        uint32_t packed[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t x = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x = shift_into_byte(x, rescale_fused_w<false>(acc[4 * q + e], p), p.n1, e);
            }
            packed[q] = x;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = (acc[i] ^ (int32_t)(packed[i & 3] >> (i & 12))) & 0x3fffff; // next round's inputs
    }
    int32_t t = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += acc[i];
    sink[id] = t;
}

} // namespace qnn

using namespace qnn;

extern "C" {

qnn_status qnn_calibrate_mfma(int workgroups, int iters, int random_operands, int32_t *sink, double *ops, void *stream)
{
    if (workgroups <= 0 || workgroups > 65536 || iters <= 0 || !sink || !ops) return QNN_EINVAL;
    hipLaunchKernelGGL(calibrate_mfma_kernel, dim3((unsigned)workgroups), dim3(512), 0, as_stream(stream), iters,
                       random_operands, sink);
    *ops = (double)workgroups * 8.0 * (double)iters * 4.0 * 2.0 * 32.0 * 32.0 * 32.0;
    return launch_status(hipGetLastError());
}

qnn_status qnn_calibrate_rescale(int workgroups, int iters, int32_t *sink, double *outputs, void *stream)
{
    if (workgroups <= 0 || workgroups > 65536 || iters <= 0 || !sink || !outputs) return QNN_EINVAL;
    hipLaunchKernelGGL(calibrate_rescale_kernel, dim3((unsigned)workgroups), dim3(256), 0, as_stream(stream), iters,
                       1518500250, 9, sink);
    *outputs = (double)workgroups * 256.0 * (double)iters * 16.0;
    return launch_status(hipGetLastError());
}

qnn_status qnn_calibrate_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst || bytes == 0 || (bytes % 16) != 0 || (reinterpret_cast<uintptr_t>(src) % 16) != 0 ||
        (reinterpret_cast<uintptr_t>(dst) % 16) != 0)
        return QNN_EINVAL;
    const size_t chunks = bytes / 16;
    const size_t want = (chunks + 255) / 256;
    const unsigned blocks = (unsigned)(want < 256 * 32 ? want : 256 * 32);
    hipLaunchKernelGGL(calibrate_copy_kernel, dim3(blocks), dim3(256), 0, as_stream(stream),
                       static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst), chunks);
    return launch_status(hipGetLastError());
}

} // extern "C"
