// Tuning switches of the dispatchers.  They are read from the environment ONCE, when the library
// is first used, and can be changed afterwards with qnn_tuning_set (the parity tests use it to
// force every kernel variant on small shapes).  No call reads the environment on its own.
#pragma once

namespace qnn {

struct Tuning {
    char force_tile[24] = ""; // QNN_FORCE_TILE: name of one tile configuration of the tiled kernels ("" = choose)
    int force_split = 0;      // QNN_FORCE_SPLIT: split-K factor used with a forced tile (0 = none)
    int no_shortk = 0;        // QNN_NO_SHORTK: switch the short-K kernel off
    int bres = -1;            // QNN_BRES: weight-resident kernel 0 = never, 1 = whenever the shape fits, -1 = by shape
    int stem_block = 0;       // QNN_STEM_BLOCK: workgroup-per-strip stem kernel
    int xcd_rows = -1;        // QNN_XCD_ROWS: rows of the XCD cut of the tile grid (-1 = choose)
    int dw_rh = 0;            // QNN_DW_RH: patch height of the depthwise kernel (0 = choose)
    int dw_mad = 0;           // QNN_DW_MAD: multiply-add form of the depthwise kernel
    int gemm_prio = -1;       // QNN_GEMM_PRIO: issue-priority scheme of the pipelined tile kernel (-1 = per tile)
    int persist = -1;         // QNN_PERSIST: 0 = one workgroup per tile, 1 = persistent workgroups, -1 = per tile
    int dw_variant = -1;      // QNN_DW_VARIANT: depthwise kernel family (-1 = choose)
    int shortk_alds = 1;      // QNN_SHORTK_ALDS: short-K kernel with the A rows staged in LDS per workgroup (K = 128, 256)
    int dw_xcd = 1;           // QNN_DW_XCD: depthwise workgroups renumbered so that an XCD gets neighbouring patches
    bool forced() const { return force_tile[0] != 0; }
};

Tuning &tuning();

} // namespace qnn
