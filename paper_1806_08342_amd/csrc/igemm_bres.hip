// Launch routine of the weight-resident kernel.
#include "igemm_launch.h"
#include "tuning.h"
#include "bres.h"

namespace qnn {

// Medium reduction, few output channels: weight-resident kernel of bres.h.  Returns false when the
// shape or the alignment does not fit (the caller then takes the tiled route).
template <int NB, int KC, bool INT4, bool CONV, bool PAD = false>
static hipError_t launch_bres_one(const BResArgs &a, unsigned blocks, int lds, hipStream_t s)
{
    auto kernel = bres_kernel<NB, KC, INT4, CONV, PAD>;
    static LdsOptIn opt_in; // per instantiation
    if (hipError_t e = opt_in.ensure(reinterpret_cast<const void *>(kernel), lds); e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(512), lds, s, a);
    return hipGetLastError();
}

template <int NB, bool INT4, bool CONV>
static hipError_t launch_bres_kc(const BResArgs &a, unsigned blocks, int lds, hipStream_t s)
{
    // A fragments travel in chunks of KC K sub-steps; a chunk size that divides K / 32 wastes no MFMA
    const int ks = a.g.K / 32;
    if (ks % 8 == 0) return launch_bres_one<NB, 8, INT4, CONV>(a, blocks, lds, s);
    if (ks % 6 == 0) return launch_bres_one<NB, 6, INT4, CONV>(a, blocks, lds, s);
    if (ks % 4 == 0) return launch_bres_one<NB, 4, INT4, CONV>(a, blocks, lds, s);
    return launch_bres_one<NB, 6, INT4, CONV, true>(a, blocks, lds, s); // last chunk padded with zero operands
}

template <int NB> static hipError_t launch_bres_nb(const BResArgs &a, bool i4, bool conv, unsigned blocks, int lds, hipStream_t s)
{
    if (conv) return i4 ? launch_bres_kc<NB, true, true>(a, blocks, lds, s) : launch_bres_kc<NB, false, true>(a, blocks, lds, s);
    return i4 ? launch_bres_kc<NB, true, false>(a, blocks, lds, s) : launch_bres_kc<NB, false, false>(a, blocks, lds, s);
}

bool try_bres(IgemmArgs &g, int a_mode, int b_mode, hipStream_t s, qnn_status *status)
{
    const int mode = tuning().bres; // tuning aid: 0 = never, 1 = whenever the shape fits
    if (mode == 0 || tuning().forced()) return false;
    if (b_mode == B_INT8_ROWS || (g.K % 32) != 0 || g.K <= 256 || g.M < 4096 || g.M >= 0x7fffffe0) return false;
    const bool conv = a_mode == A_CONV;
    if (conv) {
        if ((g.Cin % 32) != 0 || !aligned_to(g.A, 16) || (int64_t)g.H * g.W * g.Cin >= (1ll << 31)) return false;
    } else if (!aligned_to(g.A, 16) || (g.lda % 16) != 0) {
        return false;
    }
    if (b_mode == B_INT4 ? (!aligned_to(g.B, 8) || (g.ldb % 16) != 0) : (!aligned_to(g.B, 16) || (g.ldb % 16) != 0)) return false;
    int nb = g.N <= 32 ? 1 : (g.N <= 64 ? 2 : 4);
    auto lds_for = [&](int n) { return (g.K / 32) * n * 1024 + 8 * 32 * (32 * n + 32); };
    while (nb > 1 && lds_for(nb) > 160 * 1024) nb /= 2;
    if (lds_for(nb) > 160 * 1024) return false;
    const int col_groups = (g.N + 32 * nb - 1) / (32 * nb);
    // worth it while the layer is far from MFMA-bound and A is not re-read by many column groups
    // ... and there are enough row blocks for every wave of the chip (small layers stay with tiles)
    if (mode != 1 && (col_groups > 2 || g.K > 1024 || g.M < 32768)) return false;
    g.small_acc = 2;
    g.c_vec16 = aligned_to(g.C, 16) && (g.ldc % 16 == 0);
    BResArgs a = {};
    a.g = g, a.col_groups = col_groups;
    const int64_t row_blocks = (g.M + 31) / 32;
    int64_t walkers = 256 / col_groups < 1 ? 1 : 256 / col_groups; // one workgroup (8 waves) per CU
    if (walkers * 8 > row_blocks) walkers = (row_blocks + 7) / 8;
    a.groups_walkers = (int)walkers;
    const unsigned blocks = (unsigned)(walkers * col_groups);
    const int lds = lds_for(nb);
    const bool i4 = b_mode == B_INT4;
    hipError_t e;
    if (nb == 4) e = launch_bres_nb<4>(a, i4, conv, blocks, lds, s);
    else if (nb == 2) e = launch_bres_nb<2>(a, i4, conv, blocks, lds, s);
    else e = launch_bres_nb<1>(a, i4, conv, blocks, lds, s);
    *status = launch_status(e);
    return true;
}

} // namespace qnn
