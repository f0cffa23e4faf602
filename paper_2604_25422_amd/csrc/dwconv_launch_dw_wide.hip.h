// Shared by the translation units of the fp32 weight-gradient kernels with seven to sixteen block offsets (the largest
// fully unrolled kernels of the library: split over several units so that they compile side by side).
#pragma once
#include "dwconv_host.hip.h"

namespace dwhost {

// fp32, seven to sixteen block offsets (K up to 226): the LDS-direct kernel on ordinary rows.
// seg0 / nseg: the segments of every row the launch walks; slices: workgroups per channel; own_only: write the
// taps the launch owns and nothing else (see dw_partial_direct_kernel).
template <int ND, int W>
int launch_dw_partial_wide_ndw(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                               int dmin, hipStream_t st, int seg0 = 0, int nseg = -1, int slices = -1, int own_only = 0)
{
    constexpr size_t lds = dwconv::dw_direct_lds_bytes(ND, W);
    if constexpr (lds > kMaxLdsBytes) {
        return -1;
    } else {
        auto kernel = dwconv::dw_partial_direct_kernel<ND, W, false>;
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        // the taps this launch owns: those its ND offsets can reach (all K of them when they cover the filter)
        int j0 = 16 * dmin + s.pad - 15, j1 = 16 * (dmin + ND - 1) + s.pad + 16;
        j0 = j0 < 0 ? 0 : (j0 > s.K ? s.K : j0);
        j1 = j1 < j0 ? j0 : (j1 > s.K ? s.K : j1);
        if (j1 - j0 > dwconv::dw_direct_row_floats(ND)) return -1;
        if (nseg < 0) nseg = p.tiles_per_row;
        if (slices < 0) slices = p.S / p.passes;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)slices), dim3(64 * W), lds, st,
                           static_cast<const float *>(x), static_cast<const float *>(dy), part,
                           static_cast<float *>(dw_out), s.B, s.C, s.L, s.K, s.pad, dmin, nseg, p.rows.map, j0, j1, seg0,
                           own_only);
        return launch_status();
    }
}

// The units: four-wave workgroups on ordinary rows (also the launches of the many-launch form), whole-channel workgroups
// of five, eight and sixteen waves (seven to ten offsets), four-wave workgroups on virtual rows.
int launch_dw_wide_w4_f32(int nd, const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                          int dmin, hipStream_t st, int seg0, int nseg, int slices, int own_only);
int launch_dw_wide_multi_f32(int nd, const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                             int dmin, hipStream_t st);
int launch_dw_wide_rows_f32(int nd, const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                            int dmin, hipStream_t st);

}  // namespace dwhost
