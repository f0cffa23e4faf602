// Weight-gradient stage-1 kernels, fp32, seven to sixteen block offsets on the virtual rows of short rows.
#include "dwconv_launch_dw_wide.hip.h"

namespace dwhost {

// Short rows: the same kernel on the virtual row of a channel (four-wave workgroups, the filter's offsets in one launch).
template <int ND>
int launch_dw_partial_wide_rows(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                                int dmin, hipStream_t st)
{
    constexpr int W = 4;
    constexpr size_t lds = dwconv::dw_direct_lds_bytes(ND, W);
    if constexpr (lds > kMaxLdsBytes) {
        return -1;
    } else {
        if (p.wpb != W || p.passes != 1) return -1;
        auto kernel = dwconv::dw_partial_direct_kernel<ND, W, true>;
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st, static_cast<const float *>(x),
                           static_cast<const float *>(dy), part, static_cast<float *>(dw_out), 1, s.C, s.L, s.K, s.pad, dmin,
                           p.tiles_per_row, p.rows.map, 0, s.K, 0, 0);
        return launch_status();
    }
}


int launch_dw_wide_rows_f32(int nd, const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                            int dmin, hipStream_t st)
{
    switch (nd) {
    case 7: return launch_dw_partial_wide_rows<7>(x, dy, part, dw_out, s, p, dmin, st);
    case 8: return launch_dw_partial_wide_rows<8>(x, dy, part, dw_out, s, p, dmin, st);
    case 9: return launch_dw_partial_wide_rows<9>(x, dy, part, dw_out, s, p, dmin, st);
    case 10: return launch_dw_partial_wide_rows<10>(x, dy, part, dw_out, s, p, dmin, st);
    case 11: return launch_dw_partial_wide_rows<11>(x, dy, part, dw_out, s, p, dmin, st);
    case 12: return launch_dw_partial_wide_rows<12>(x, dy, part, dw_out, s, p, dmin, st);
    case 13: return launch_dw_partial_wide_rows<13>(x, dy, part, dw_out, s, p, dmin, st);
    case 14: return launch_dw_partial_wide_rows<14>(x, dy, part, dw_out, s, p, dmin, st);
    case 15: return launch_dw_partial_wide_rows<15>(x, dy, part, dw_out, s, p, dmin, st);
    case 16: return launch_dw_partial_wide_rows<16>(x, dy, part, dw_out, s, p, dmin, st);
    default: return -1;
    }
}

}  // namespace dwhost
