// Launch routine of the register-staged tile kernel.
#include "igemm_launch.h"

namespace qnn {

template <int BM, int BN, int WM, int WN, int A_MODE, int B_MODE, int VEC, bool ZW>
static void launch_one(const IgemmArgs &g, hipStream_t s)
{
    const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
    hipLaunchKernelGGL((igemm_kernel<BM, BN, WM, WN, A_MODE, B_MODE, VEC, ZW>), dim3((unsigned)tiles), dim3(WM * WN * 64), 0,
                       s, g);
}

template <int BM, int BN, int WM, int WN, int A_MODE, bool ZW = false>
static void launch_tile(const IgemmArgs &g, int b_mode, int vec, hipStream_t s)
{
    if (b_mode == B_INT8) {
        if (vec == 16) launch_one<BM, BN, WM, WN, A_MODE, B_INT8, 16, ZW>(g, s);
        else if (vec == 8) launch_one<BM, BN, WM, WN, A_MODE, B_INT8, 8, ZW>(g, s);
        else launch_one<BM, BN, WM, WN, A_MODE, B_INT8, 1, ZW>(g, s);
    } else if (b_mode == B_INT4) {
        if (vec == 16) launch_one<BM, BN, WM, WN, A_MODE, B_INT4, 16, ZW>(g, s);
        else if (vec == 8) launch_one<BM, BN, WM, WN, A_MODE, B_INT4, 8, ZW>(g, s);
        else launch_one<BM, BN, WM, WN, A_MODE, B_INT4, 1, ZW>(g, s);
    } else {
        if constexpr (A_MODE == A_MATRIX) launch_one<BM, BN, WM, WN, A_MATRIX, B_INT8_ROWS, 1, ZW>(g, s);
    }
}

void launch_plain_tile_zw(const IgemmArgs &g, int a_mode, int b_mode, int vec, hipStream_t s)
{
    if (a_mode == A_MATRIX) launch_tile<64, 64, 2, 2, A_MATRIX, true>(g, b_mode, vec, s);
    else launch_tile<64, 64, 2, 2, A_CONV, true>(g, b_mode, vec, s);
}

void launch_plain_tile(bool big, const IgemmArgs &g, int a_mode, int b_mode, int vec, hipStream_t s)
{
    const bool mat = a_mode == A_MATRIX;
    if (big) {
        if (mat) launch_tile<128, 128, 2, 2, A_MATRIX>(g, b_mode, vec, s);
        else launch_tile<128, 128, 2, 2, A_CONV>(g, b_mode, vec, s);
    } else {
        if (mat) launch_tile<64, 64, 2, 2, A_MATRIX>(g, b_mode, vec, s);
        else launch_tile<64, 64, 2, 2, A_CONV>(g, b_mode, vec, s);
    }
}

} // namespace qnn
