// Host-side launch routines of the dense quantized layers; each kernel family is compiled in a
// translation unit of its own (igemm_*.hip) and called from the dispatcher in igemm.hip.
#pragma once

#include <atomic>
#include <cstdint>
#include <cstdlib>

#include "igemm.h"

namespace qnn {

// magic number for dividing by d with a multiply-high (see the kernels that take it)
inline uint32_t magic_for(uint32_t d) { return d <= 1 ? 0u : (uint32_t)(((1ull << 32) + d - 1) / d); }

// Kernels that use more than 64 KB of dynamic LDS must opt in once per device.  One object per kernel
// instantiation (a function-local static); safe to call from several threads (setting the attribute
// twice is harmless).
struct LdsOptIn {
    std::atomic<int> enabled[64] = {}; // bytes enabled so far, per device
    hipError_t ensure(const void *kernel, int bytes)
    {
        int dev = 0;
        if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
        if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        if (enabled[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
        if (hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); e != hipSuccess) return e;
        enabled[dev].store(bytes, std::memory_order_release);
        return hipSuccess;
    }
};

inline bool aligned_to(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Short reduction (K <= 256): weight-stationary kernel of shortk.h.  `strided`: rows are the pixels
// of a strided 1x1 convolution.  Not eligible when the operands miss its alignment rules.
bool shortk_eligible(const IgemmArgs &g, int b_mode, bool strided);
qnn_status launch_shortk(IgemmArgs &g, int b_mode, bool strided, hipStream_t s);

// Few rows (M <= 64): weight-streaming kernel of skinny.h.  Returns false if the shape does not fit.
bool try_skinny(const IgemmArgs &g, int a_mode, int b_mode, int vec, hipStream_t s, qnn_status *status);

// Medium reduction, few output channels: weight-resident kernel of bres.h.  Returns false when the
// shape or the alignment does not fit (the caller then takes the tiled route).
bool try_bres(IgemmArgs &g, int a_mode, int b_mode, hipStream_t s, qnn_status *status);

// Network stems (very few input channels): kernels of stemwave.h / stemconv.h.  `g` carries the
// convolution geometry; returns false if the layer is not a stem these kernels cover.
bool try_stem(IgemmArgs &g, int batch, int kh, int stride_h, int stride_w, int weight_bits, hipStream_t s, qnn_status *status);

// Row sums of the activations for per-channel weight zero-points: out[m], M int32 (igemm_rowsum.hip)
qnn_status launch_rowsum(const IgemmArgs &g, int a_mode, int kh, int32_t *out, hipStream_t s);

// Register-staged tiles of igemm.h (any alignment, any weight layout): 64x64 or 128x128.
void launch_plain_tile(bool big, const IgemmArgs &g, int a_mode, int b_mode, int vec, hipStream_t s);
// the 64x64 tile with per-column weight zero-points (g.zw, g.rowsum set)
void launch_plain_tile_zw(const IgemmArgs &g, int a_mode, int b_mode, int vec, hipStream_t s);

} // namespace qnn
