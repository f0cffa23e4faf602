// Forward / input gradient, rows of at most 128 positions with seven to fifteen block offsets, bf16 storage.
#include "dwconv_launch_corr.hip.h"

namespace dwhost {

int launch_corr_rowbatch_wide_bf16(dwconv::RowBatchGeom &rg, int nd, const void *in, const void *f, void *out, const Shape &s,
                                   hipStream_t st)
{
    return launch_corr_rowbatch_wide_t<dwconv::bf16_t>(rg, nd, in, f, out, s, st);
}

}  // namespace dwhost
