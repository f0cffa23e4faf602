// Weight-gradient stage-1 kernels, fp32, filters of 67 to 226 taps (a unit of its own: these are the largest
// fully unrolled kernels of the library).
#include "dwconv_host.hip.h"

namespace dwhost {

// fp32, seven to sixteen block offsets (K up to 226): the LDS-direct kernel on ordinary rows.
template <int ND, int W>
int launch_dw_partial_wide_ndw(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                               int dmin, hipStream_t st)
{
    constexpr size_t lds = dwconv::dw_direct_lds_bytes(ND, W);
    if constexpr (lds > kMaxLdsBytes) {
        return -1;
    } else {
        auto kernel = dwconv::dw_partial_direct_kernel<ND, W, false>;
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                           static_cast<const float *>(x), static_cast<const float *>(dy), part,
                           static_cast<float *>(dw_out), s.B, s.C, s.L, s.K, s.pad, dmin, p.tiles_per_row, p.rows.map);
        return launch_status();
    }
}
template <int ND>
int launch_dw_partial_wide_nd(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                              int dmin, hipStream_t st)
{
    if (p.rows.on) return -1;
    if constexpr (ND > kMfmaMaxNDWide) {
        // eleven to sixteen block offsets: four-wave workgroups only (the plan never asks for more)
        return p.wpb == 4 ? launch_dw_partial_wide_ndw<ND, 4>(x, dy, part, dw_out, s, p, dmin, st) : -1;
    } else {
        switch (p.wpb) {
        case 4: return launch_dw_partial_wide_ndw<ND, 4>(x, dy, part, dw_out, s, p, dmin, st);
        case 5: return launch_dw_partial_wide_ndw<ND, 5>(x, dy, part, dw_out, s, p, dmin, st);
        case 8: return launch_dw_partial_wide_ndw<ND, 8>(x, dy, part, dw_out, s, p, dmin, st);
        case 16: return launch_dw_partial_wide_ndw<ND, 16>(x, dy, part, dw_out, s, p, dmin, st);
        default: return -1;
        }
    }
}

int launch_dw_partial_wide_f32(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                               int dmin, int nd, hipStream_t st)
{
    switch (nd) {
    case 7: return launch_dw_partial_wide_nd<7>(x, dy, part, dw_out, s, p, dmin, st);
    case 8: return launch_dw_partial_wide_nd<8>(x, dy, part, dw_out, s, p, dmin, st);
    case 9: return launch_dw_partial_wide_nd<9>(x, dy, part, dw_out, s, p, dmin, st);
    case 10: return launch_dw_partial_wide_nd<10>(x, dy, part, dw_out, s, p, dmin, st);
    case 11: return launch_dw_partial_wide_nd<11>(x, dy, part, dw_out, s, p, dmin, st);
    case 12: return launch_dw_partial_wide_nd<12>(x, dy, part, dw_out, s, p, dmin, st);
    case 13: return launch_dw_partial_wide_nd<13>(x, dy, part, dw_out, s, p, dmin, st);
    case 14: return launch_dw_partial_wide_nd<14>(x, dy, part, dw_out, s, p, dmin, st);
    case 15: return launch_dw_partial_wide_nd<15>(x, dy, part, dw_out, s, p, dmin, st);
    case 16: return launch_dw_partial_wide_nd<16>(x, dy, part, dw_out, s, p, dmin, st);
    default: return -1;
    }
}

}  // namespace dwhost
