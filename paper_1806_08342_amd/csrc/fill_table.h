// Constant table of padding codes: kernels that gather convolution taps point an out-of-image tap
// at the chunk holding the activation zero-point, so that it contributes (z_x - z_x) * w = 0
// without a branch or a select behind the load (section 2.1: zero must be exactly representable).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace qnn {

// 256 constant 16-byte chunks: entry v is the byte v repeated (fill codes for padding taps)
struct FillTable {
    uint8_t v[256][16];
    constexpr FillTable() : v{}
    {
        for (int i = 0; i < 256; ++i)
            for (int j = 0; j < 16; ++j) v[i][j] = (uint8_t)i;
    }
};
__device__ const FillTable g_fill_table{};

} // namespace qnn
