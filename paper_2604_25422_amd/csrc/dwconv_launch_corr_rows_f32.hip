// Forward / input gradient on short rows with seven and more block offsets, f32 storage: rows of at most 128 positions
// (sixteen-row kernels, up to fifteen offsets) and virtual rows (up to sixteen).
#include "dwconv_launch_corr.hip.h"

namespace dwhost {

int launch_corr_rowbatch_wide_f32(dwconv::RowBatchGeom &rg, int nd, const void *in, const void *f, void *out, const Shape &s,
                                  hipStream_t st)
{
    return launch_corr_rowbatch_wide_t<float>(rg, nd, in, f, out, s, st);
}

int launch_corr_vrows_wide_f32(const dwconv::CorrGeom &g, const RowsPlan &rp, int nd, const void *in, const void *f, void *out,
                               const Shape &s, hipStream_t st)
{
    auto go = [&](auto kernel) -> int { return launch_corr_vrows_kernel<float>(kernel, g, rp, in, f, out, s, st); };
    switch (nd) {
    case 7: return go(dwconv::corr_mfma_kernel<float, 7, true>);
    case 8: return go(dwconv::corr_mfma_kernel<float, 8, true>);
    case 9: return go(dwconv::corr_mfma_kernel<float, 9, true>);
    case 10: return go(dwconv::corr_mfma_kernel<float, 10, true>);
    case 11: return go(dwconv::corr_mfma_kernel<float, 11, true>);
    case 12: return go(dwconv::corr_mfma_kernel<float, 12, true>);
    case 13: return go(dwconv::corr_mfma_kernel<float, 13, true>);
    case 14: return go(dwconv::corr_mfma_kernel<float, 14, true>);
    default: return -1;        // (fifteen and sixteen offsets: no registers left for the translation of positions)
    }
}

}  // namespace dwhost
