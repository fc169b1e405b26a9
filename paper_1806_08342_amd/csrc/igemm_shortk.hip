// Launch routines of the weight-stationary short-K kernel and of the few-row kernel.
#include "igemm_launch.h"
#include "tuning.h"
#include "shortk.h"
#include "skinny.h"

namespace qnn {

// Short reduction (K <= 256): weight-stationary kernel of shortk.h.  Returns false when the
// operands do not meet its alignment rules (the caller then takes the general route).
template <int NB, int KS, bool INT4, int VEC, int BVEC, int ADD>
static void launch_shortk_add(const ShortKArgs &a, int64_t waves, hipStream_t s)
{
    // the waves of a workgroup (8 with the 64 KB table of code pairs, else 4) share the table(s); their tiles behind
    constexpr int kWaves = ADD == 2 ? 8 : 4;
    constexpr int kLds = (ADD == 2 ? 65536 : 2048) + kWaves * 32 * (32 * NB + 32);
    auto kernel = shortk_kernel<NB, KS, INT4, VEC, BVEC, ADD>;
    static LdsOptIn opt_in; // per instantiation
    if (opt_in.ensure(reinterpret_cast<const void *>(kernel), kLds) != hipSuccess) return; // the error stays pending for the caller
    hipLaunchKernelGGL(kernel, dim3((unsigned)((waves + kWaves - 1) / kWaves)), dim3(kWaves * 64), kLds, s, a);
}

template <int KS, bool INT4, int VEC> static void launch_shortk_one(const ShortKArgs &a, int64_t waves, hipStream_t s, bool alds)
{
    constexpr int NB = KS <= 4 ? 4 : 2;
    // weights: 16-byte loads when every 16-element piece of a column is 16-byte aligned, else dwords
    const bool b16 = !INT4 && aligned_to(a.g.B, 16) && (a.g.ldb % 16) == 0 && (a.g.K % 16) == 0;
    if constexpr (VEC == 16 && (KS == 4 || KS == 8)) {
        if (alds) { // A rows through LDS, shared by the waves of a workgroup (the caller sized `waves` in workgroups)
            if (b16) hipLaunchKernelGGL((shortk_kernel<NB, KS, INT4, VEC, 16, 0, true>), dim3((unsigned)waves), dim3(256), 0, s, a);
            else hipLaunchKernelGGL((shortk_kernel<NB, KS, INT4, VEC, 4, 0, true>), dim3((unsigned)waves), dim3(256), 0, s, a);
            return;
        }
    }
    if constexpr (VEC == 16) {
        if (a.g.R) { // residual add in the store phase (the launcher only leaves R set for VEC == 16)
            // from 2^24 outputs on the 65536-entry pair table pays for itself; below, two 256-entry tables
            const bool pairs = a.g.M * (int64_t)a.g.N >= ((int64_t)1 << 24);
            if (b16) pairs ? launch_shortk_add<NB, KS, INT4, VEC, 16, 2>(a, waves, s) : launch_shortk_add<NB, KS, INT4, VEC, 16, 1>(a, waves, s);
            else pairs ? launch_shortk_add<NB, KS, INT4, VEC, 4, 2>(a, waves, s) : launch_shortk_add<NB, KS, INT4, VEC, 4, 1>(a, waves, s);
            return;
        }
    }
    const unsigned blocks = (unsigned)((waves + 3) / 4);
    if (b16) hipLaunchKernelGGL((shortk_kernel<NB, KS, INT4, VEC, 16>), dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((shortk_kernel<NB, KS, INT4, VEC, 4>), dim3(blocks), dim3(256), 0, s, a);
}

template <bool INT4, int VEC> static void launch_shortk_ks(const ShortKArgs &a, int ks, int64_t waves, hipStream_t s, bool alds)
{
    if (ks <= 1) launch_shortk_one<1, INT4, VEC>(a, waves, s, false);
    else if (ks <= 2) launch_shortk_one<2, INT4, VEC>(a, waves, s, false);
    else if (ks <= 4) launch_shortk_one<4, INT4, VEC>(a, waves, s, alds);
    else launch_shortk_one<8, INT4, VEC>(a, waves, s, alds);
}

bool shortk_eligible(const IgemmArgs &g, int b_mode, bool strided)
{
    if (g.K > 256 || (g.K % 8) != 0 || g.M <= 64 || g.M >= 0x7fffffe0 || b_mode == B_INT8_ROWS) return false;
    if (tuning().forced() || tuning().no_shortk) return false;
    const int64_t row_pitch = strided ? g.Cin : g.lda;
    if (!aligned_to(g.A, 8) || (row_pitch % 8) != 0) return false;
    if (!aligned_to(g.B, 4) || (g.ldb % 8) != 0) return false;
    return true;
}

qnn_status launch_shortk(IgemmArgs &g, int b_mode, bool strided, hipStream_t s)
{
    g.small_acc = 2; // K <= 256: |acc| <= 2^22
    g.c_vec16 = aligned_to(g.C, 16) && (g.ldc % 16 == 0);
    const int ks = (g.K + 31) / 32;
    const int nb = ks <= 4 ? 4 : 2;
    ShortKArgs a = {};
    a.g = g;
    a.strided = strided ? 1 : 0;
    a.col_groups = (g.N + 32 * nb - 1) / (32 * nb);
    const int64_t row_blocks = (g.M + 31) / 32;
    // as many waves as stay resident together (3 per SIMD for K <= 32, else 2, on 256 CUs), spread
    // over the column groups, then trimmed so that every wave walks the same number of row blocks
    const int64_t row_pitch0 = strided ? g.Cin : g.lda;
    const bool add_fused = g.R != nullptr && aligned_to(g.A, 16) && (row_pitch0 % 16) == 0 && (g.K % 16) == 0 && g.c_vec16 &&
                           g.r_vec16 && (g.N % 16) == 0; // the variant with the add built in: 8-wave workgroups, one per CU
    const int64_t resident = 256 * 4 * ((ks <= 1 && !add_fused) ? 3 : 2);
    int64_t walkers = resident / a.col_groups;
    walkers = walkers < 1 ? 1 : (walkers > row_blocks ? row_blocks : walkers);
    const int64_t per_walker = (row_blocks + walkers - 1) / walkers;
    walkers = (row_blocks + per_walker - 1) / per_walker;
    a.walkers = (int)walkers;
    int64_t waves = walkers * a.col_groups;
    if (waves > 0x7fffffff) return QNN_EINVAL;
    const int64_t row_pitch = strided ? g.Cin : g.lda;
    const bool v16 = aligned_to(g.A, 16) && (row_pitch % 16) == 0 && (g.K % 16) == 0;
    // the add is built into the 16-byte variants only, for outputs and residuals made of whole aligned chunks
    const bool add_pass = g.R != nullptr && !add_fused;
    if (add_pass) a.g.R = nullptr;
    // K = 128 / 256 with enough column groups to fill a workgroup: the A rows go through LDS once per workgroup.
    // Not with the add built in: its 8-wave workgroups (one per CU, sharing the table of code pairs) lose more at
    // the barrier of every row block than the shared rows save (measured 65 against 58 us on 50176 x 1024 x 256).
    const int wg_waves = 4;
    const bool alds = tuning().shortk_alds != 0 && !strided && v16 && !a.g.R && (g.K == 128 || g.K == 256) && a.col_groups >= wg_waves;
    if (alds) {
        const int64_t groups = (a.col_groups + wg_waves - 1) / wg_waves;
        const int64_t resident_wgs = 256 * 2;
        int64_t wk = resident_wgs / groups;
        wk = wk < 1 ? 1 : (wk > row_blocks ? row_blocks : wk);
        const int64_t per = (row_blocks + wk - 1) / wk;
        wk = (row_blocks + per - 1) / per;
        a.walkers = (int)wk;
        waves = groups * wk; // workgroups
    }
    if (b_mode == B_INT4) {
        if (v16) launch_shortk_ks<true, 16>(a, ks, waves, s, alds);
        else launch_shortk_ks<true, 8>(a, ks, waves, s, false);
    } else {
        if (v16) launch_shortk_ks<false, 16>(a, ks, waves, s, alds);
        else launch_shortk_ks<false, 8>(a, ks, waves, s, false);
    }
    const qnn_status st = launch_status(hipGetLastError());
    if (st != QNN_OK || !add_pass) return st;
    return launch_add_inplace(g.C, g.ldc, g.R, g.ldr, g.M, g.N, g.add, s);
}

bool try_skinny(const IgemmArgs &g, int a_mode, int b_mode, int vec, hipStream_t s, qnn_status *status)
{
    // few rows: weight-streaming kernel (one workgroup per 16 output columns, K split over 8 waves)
    if (a_mode == A_MATRIX && g.M <= 64 && vec == 16 && (g.K % 64) == 0 && b_mode != B_INT8_ROWS &&
        !tuning().forced()) {
        const unsigned blocks = (unsigned)((g.N + 15) / 16);
        const int mt = g.M <= 16 ? 1 : (g.M <= 32 ? 2 : 4);
        const bool i4 = b_mode == B_INT4;
        if (mt == 1) {
            if (i4) hipLaunchKernelGGL((skinny_gemm_kernel<1, true>), dim3(blocks), dim3(512), 0, s, g);
            else hipLaunchKernelGGL((skinny_gemm_kernel<1, false>), dim3(blocks), dim3(512), 0, s, g);
        } else if (mt == 2) {
            if (i4) hipLaunchKernelGGL((skinny_gemm_kernel<2, true>), dim3(blocks), dim3(512), 0, s, g);
            else hipLaunchKernelGGL((skinny_gemm_kernel<2, false>), dim3(blocks), dim3(512), 0, s, g);
        } else {
            if (i4) hipLaunchKernelGGL((skinny_gemm_kernel<4, true>), dim3(blocks), dim3(512), 0, s, g);
            else hipLaunchKernelGGL((skinny_gemm_kernel<4, false>), dim3(blocks), dim3(512), 0, s, g);
        }
        *status = launch_status(hipGetLastError());
        return true;
    }
    return false;
}

} // namespace qnn
