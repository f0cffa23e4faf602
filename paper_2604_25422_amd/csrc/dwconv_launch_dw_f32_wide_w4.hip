// Weight-gradient stage-1 kernels, fp32, seven to sixteen block offsets, four-wave workgroups on ordinary rows.
#include "dwconv_launch_dw_wide.hip.h"

namespace dwhost {

int launch_dw_wide_w4_f32(int nd, const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                          int dmin, hipStream_t st, int seg0, int nseg, int slices, int own_only)
{
    switch (nd) {
    case 7: return launch_dw_partial_wide_ndw<7, 4>(x, dy, part, dw_out, s, p, dmin, st, seg0, nseg, slices, own_only);
    case 8: return launch_dw_partial_wide_ndw<8, 4>(x, dy, part, dw_out, s, p, dmin, st, seg0, nseg, slices, own_only);
    case 9: return launch_dw_partial_wide_ndw<9, 4>(x, dy, part, dw_out, s, p, dmin, st, seg0, nseg, slices, own_only);
    case 10: return launch_dw_partial_wide_ndw<10, 4>(x, dy, part, dw_out, s, p, dmin, st, seg0, nseg, slices, own_only);
    case 11: return launch_dw_partial_wide_ndw<11, 4>(x, dy, part, dw_out, s, p, dmin, st, seg0, nseg, slices, own_only);
    case 12: return launch_dw_partial_wide_ndw<12, 4>(x, dy, part, dw_out, s, p, dmin, st, seg0, nseg, slices, own_only);
    case 13: return launch_dw_partial_wide_ndw<13, 4>(x, dy, part, dw_out, s, p, dmin, st, seg0, nseg, slices, own_only);
    case 14: return launch_dw_partial_wide_ndw<14, 4>(x, dy, part, dw_out, s, p, dmin, st, seg0, nseg, slices, own_only);
    case 15: return launch_dw_partial_wide_ndw<15, 4>(x, dy, part, dw_out, s, p, dmin, st, seg0, nseg, slices, own_only);
    case 16: return launch_dw_partial_wide_ndw<16, 4>(x, dy, part, dw_out, s, p, dmin, st, seg0, nseg, slices, own_only);
    default: return -1;
    }
}

}  // namespace dwhost
