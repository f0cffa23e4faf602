// Fused backward kernels, f32 storage.
#include "dwconv_launch_bwd.hip.h"

namespace dwhost {

int launch_bwd_fused_f32(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out, bool *wrote_dw,
                          const Shape &s, const DwPlan &p, hipStream_t st)
{
    return launch_bwd_fused<float>(dy, x, w, dx, part, dw_out, wrote_dw, s, p, st);
}

}  // namespace dwhost
