// Forward / input-gradient kernels, bf16 storage.
#include "dwconv_launch_corr.hip.h"

namespace dwhost {

int launch_corr_bf16(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st)
{
    return launch_corr<bf16_t>(in, f, out, s, pad_eff, reverse, st);
}

}  // namespace dwhost
