// Activation sums for per-channel weight zero-points (eq. 5-6: the term z_w * sum_k x_Q is shared
// by all output channels of a pixel, so it is formed once per output row, ahead of the product):
//   rowsum[m] = sum_k (A[m][k] - z_a)            matrices
//   rowsum[m] = sum over the taps inside the image, all channels, of (x - z_x)    convolutions
// (a padding tap holds the code z_x and contributes 0).  16 lanes cooperate on one output row.
#include "igemm_launch.h"

namespace qnn {

__device__ __forceinline__ int32_t reduce16(int32_t v)
{
    v += __shfl_xor(v, 8);
    v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 1);
    return v;
}

// sum of the n bytes at p; vec16: p and n are multiples of 16 (16-byte loads), else byte loads
__device__ __forceinline__ int32_t byte_run_sum(const uint8_t *p, int n, int part, bool vec16)
{
    int32_t s = 0;
    if (vec16) {
        for (int k = part * 16; k < n; k += 256) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(p + k);
#pragma unroll
            for (int d = 0; d < 4; ++d) s = (int32_t)__builtin_amdgcn_udot4(v[d], 0x01010101u, (uint32_t)s, false);
        }
    } else {
        for (int k = part; k < n; k += 16) s += p[k];
    }
    return s;
}

__global__ void __launch_bounds__(256) rowsum_matrix_kernel(const uint8_t *__restrict__ A, int64_t lda, int64_t M, int K,
                                                            int z_a, int vec16, int32_t *__restrict__ out)
{
    const int part = threadIdx.x & 15;
    for (int64_t m = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4); m < M; m += (int64_t)gridDim.x * 16) {
        const int32_t s = reduce16(byte_run_sum(A + m * lda, K, part, vec16 != 0));
        if (part == 0) out[m] = s - K * z_a;
    }
}

__global__ void __launch_bounds__(256) rowsum_conv_kernel(const IgemmArgs g, int kh, int vec16, int32_t *__restrict__ out)
{
    const int part = threadIdx.x & 15;
    const int64_t per_image = (int64_t)g.Ho * g.Wo;
    for (int64_t m = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4); m < g.M; m += (int64_t)gridDim.x * 16) {
        const int64_t img = m / per_image;
        const int rem = (int)(m - img * per_image);
        const int ho = rem / g.Wo, wo = rem - ho * g.Wo;
        const uint8_t *base = g.A + img * ((int64_t)g.H * g.W * g.Cin);
        int32_t s = 0;
        int taps = 0;
        for (int a = 0; a < kh; ++a) {
            const int hi = ho * g.sh - g.ph + a;
            if (hi < 0 || hi >= g.H) continue;
            // the taps of one kernel row that lie inside the image are one contiguous byte run
            int b_lo = g.pw - wo * g.sw;
            b_lo = b_lo < 0 ? 0 : b_lo;
            int b_hi = g.W + g.pw - wo * g.sw;
            b_hi = b_hi > g.kw ? g.kw : b_hi;
            if (b_hi <= b_lo) continue;
            const int wi = wo * g.sw - g.pw + b_lo;
            s += byte_run_sum(base + ((int64_t)hi * g.W + wi) * g.Cin, (b_hi - b_lo) * g.Cin, part, vec16 != 0);
            taps += b_hi - b_lo;
        }
        s = reduce16(s);
        if (part == 0) out[m] = s - taps * g.Cin * g.z_a;
    }
}

qnn_status launch_rowsum(const IgemmArgs &g, int a_mode, int kh, int32_t *out, hipStream_t s)
{
    const int64_t groups = (g.M + 15) / 16;
    const unsigned blocks = (unsigned)(groups < 256 * 32 ? groups : 256 * 32);
    if (a_mode == A_MATRIX) {
        const int vec16 = aligned_to(g.A, 16) && (g.lda % 16) == 0 && (g.K % 16) == 0;
        hipLaunchKernelGGL(rowsum_matrix_kernel, dim3(blocks), dim3(256), 0, s, g.A, g.lda, g.M, g.K, g.z_a, vec16, out);
    } else {
        const int vec16 = aligned_to(g.A, 16) && (g.Cin % 16) == 0;
        hipLaunchKernelGGL(rowsum_conv_kernel, dim3(blocks), dim3(256), 0, s, g, kh, vec16, out);
    }
    return launch_status(hipGetLastError());
}

} // namespace qnn
