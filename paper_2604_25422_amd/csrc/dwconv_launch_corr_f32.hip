// Forward / input-gradient kernels, f32 storage.
#include "dwconv_launch_corr.hip.h"

namespace dwhost {

int launch_corr_f32(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st)
{
    return launch_corr<float>(in, f, out, s, pad_eff, reverse, st);
}

}  // namespace dwhost
