// Launch routine of the stem convolution kernels.
#include "igemm_launch.h"
#include "tuning.h"
#include "stemconv.h"
#include "stemwave.h"

namespace qnn {

bool try_stem(IgemmArgs &g, int batch, int kh, int stride_h, int stride_w, int weight_bits, hipStream_t s, qnn_status *status)
{
    const int Cin = g.Cin, kw = g.kw, Cout = g.N, Ho = g.Ho, Wo = g.Wo;
    // a handful of input channels, one kernel row = one short contiguous byte run
    if (!(weight_bits == 8 && Cin < 16 && kw * Cin <= 32 && stride_w * Cin <= 7 && (kh == 3 || kh == 7) && Cout <= 64 &&
          ((int64_t)g.W * Cin) % 4 == 0 && aligned_to(g.A, 4)))
        return false;
    g.small_acc = 2;
    g.c_vec16 = aligned_to(g.C, 16) && (g.ldc % 16 == 0);
    // default: the barrier-free kernel (one wave per 32-pixel strip), built for row strides 1 and 2
    if (!tuning().stem_block && (stride_h == 1 || stride_h == 2)) {
        StemWaveArgs sw = {};
        sw.g = g, sw.kh = kh, sw.run = kw * Cin;
        sw.strips = (Wo + 31) / 32;
        // enough waves for the chip (about 8 per SIMD), but at least 4 output rows per segment:
        // the first row of a segment fetches all kh image rows, the others only stride_h
        const int64_t columns = (int64_t)batch * sw.strips;
        int64_t segments = (8192 + columns - 1) / columns;
        const int64_t most = (Ho + 3) / 4;
        segments = segments < 1 ? 1 : (segments > most ? most : segments);
        sw.rows_per_seg = (int)((Ho + segments - 1) / segments);
        sw.segments = (Ho + sw.rows_per_seg - 1) / sw.rows_per_seg;
        sw.waves = columns * sw.segments;
        const int64_t wblocks = (sw.waves + 3) / 4;
        if (wblocks <= 0x7fffffff) {
            const dim3 grid((unsigned)wblocks);
            const int nb = Cout <= 32 ? 1 : 2;
#define QNN_STEMWAVE(KH_, NB_, SH_) \
    if (kh == KH_ && nb == NB_ && stride_h == SH_) hipLaunchKernelGGL((stemwave_kernel<KH_, NB_, SH_>), grid, dim3(256), 0, s, sw)
            QNN_STEMWAVE(3, 1, 1); QNN_STEMWAVE(3, 1, 2); QNN_STEMWAVE(3, 2, 1); QNN_STEMWAVE(3, 2, 2);
            QNN_STEMWAVE(7, 1, 1); QNN_STEMWAVE(7, 1, 2); QNN_STEMWAVE(7, 2, 1); QNN_STEMWAVE(7, 2, 2);
#undef QNN_STEMWAVE
            *status = launch_status(hipGetLastError());
            return true;
        }
    }
    StemArgs st = {};
    st.g = g, st.kh = kh, st.run = kw * Cin;
    st.strips = (Wo + 127) / 128;
    // a workgroup walks up to 8 output rows (weights are staged once per workgroup), fewer
    // when that would leave the chip with too few workgroups
    const int64_t row_strips = (int64_t)batch * Ho * st.strips;
    st.rows_per_wg = (int)(row_strips / 2048 < 1 ? 1 : (row_strips / 2048 > 8 ? 8 : row_strips / 2048));
    const int64_t blocks = (int64_t)batch * ((Ho + st.rows_per_wg - 1) / st.rows_per_wg) * st.strips;
    if (blocks > 0x7fffffff) return false;
    if (kh == 3 && Cout <= 32) hipLaunchKernelGGL((stemconv_kernel<3, 1>), dim3((unsigned)blocks), dim3(256), 0, s, st);
    else if (kh == 3) hipLaunchKernelGGL((stemconv_kernel<3, 2>), dim3((unsigned)blocks), dim3(256), 0, s, st);
    else if (Cout <= 32) hipLaunchKernelGGL((stemconv_kernel<7, 1>), dim3((unsigned)blocks), dim3(256), 0, s, st);
    else hipLaunchKernelGGL((stemconv_kernel<7, 2>), dim3((unsigned)blocks), dim3(256), 0, s, st);
    *status = launch_status(hipGetLastError());
    return true;
}

} // namespace qnn
