// Weight-gradient stage-1 kernels, fp32, seven to ten block offsets, whole-channel workgroups of five, eight and sixteen waves.
#include "dwconv_launch_dw_wide.hip.h"

namespace dwhost {

template <int ND>
static int launch_multi_nd(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p, int dmin,
                           hipStream_t st)
{
    switch (p.wpb) {
    case 5: return launch_dw_partial_wide_ndw<ND, 5>(x, dy, part, dw_out, s, p, dmin, st);
    case 8: return launch_dw_partial_wide_ndw<ND, 8>(x, dy, part, dw_out, s, p, dmin, st);
    case 16: return launch_dw_partial_wide_ndw<ND, 16>(x, dy, part, dw_out, s, p, dmin, st);
    default: return -1;
    }
}

int launch_dw_wide_multi_f32(int nd, const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                             int dmin, hipStream_t st)
{
    switch (nd) {
    case 7: return launch_multi_nd<7>(x, dy, part, dw_out, s, p, dmin, st);
    case 8: return launch_multi_nd<8>(x, dy, part, dw_out, s, p, dmin, st);
    case 9: return launch_multi_nd<9>(x, dy, part, dw_out, s, p, dmin, st);
    case 10: return launch_multi_nd<10>(x, dy, part, dw_out, s, p, dmin, st);
    default: return -1;        // (eleven to sixteen offsets: four-wave workgroups only, the plan never asks for more)
    }
}

}  // namespace dwhost
