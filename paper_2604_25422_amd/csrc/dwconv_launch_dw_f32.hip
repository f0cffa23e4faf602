// Weight-gradient stage-1 kernels, f32 storage.
#include "dwconv_launch_dw.hip.h"

namespace dwhost {

int launch_dw_partial_f32(const void *x, const void *dy, float *part, void *dw_out, bool *wrote_dw, const Shape &s,
                          const DwPlan &p, hipStream_t st)
{
    return launch_dw_partial<float>(x, dy, part, dw_out, wrote_dw, s, p, st);
}

}  // namespace dwhost
