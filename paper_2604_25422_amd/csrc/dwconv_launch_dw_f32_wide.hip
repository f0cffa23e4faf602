// Weight-gradient stage-1 kernels, fp32, filters of 67 to 226 taps (a unit of its own: these are the largest
// fully unrolled kernels of the library).
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

template <int ND>
int launch_dw_partial_wide_nd(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                              int dmin, hipStream_t st)
{
    if (p.rows.on) return launch_dw_partial_wide_rows<ND>(x, dy, part, dw_out, s, p, dmin, st);
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

// One launch of the many-pass form: n (nine to sixteen) offsets from d_lo, segments [seg0, seg0 + nseg) of every row.
int launch_dw_manypass_one(const void *x, const void *dy, float *part, const Shape &s, const DwPlan &p, int d_lo, int n,
                           int seg0, int nseg, hipStream_t st)
{
    const int sl = p.S / 2;
    switch (n) {
    case 9: return launch_dw_partial_wide_ndw<9, 4>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 10: return launch_dw_partial_wide_ndw<10, 4>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 11: return launch_dw_partial_wide_ndw<11, 4>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 12: return launch_dw_partial_wide_ndw<12, 4>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 13: return launch_dw_partial_wide_ndw<13, 4>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 14: return launch_dw_partial_wide_ndw<14, 4>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 15: return launch_dw_partial_wide_ndw<15, 4>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 16: return launch_dw_partial_wide_ndw<16, 4>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    default: return -1;
    }
}

int launch_dw_partial_wide_f32(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                               int dmin, int nd, hipStream_t st)
{
    if (p.manypass) {
        if (dw_out || p.wpb != 4 || p.S < 2 || (p.S % 2) != 0 || p.rows.on) return -1;
        const int sl = p.S / 2;
        const size_t set_floats = (size_t)sl * (size_t)s.C * (size_t)s.K;
        {
            // both sets of slices start at zero: a launch stores only the taps it owns
            const size_t n = 2 * set_floats;
            size_t fill_blocks = (n + 256 * 8 - 1) / (256 * 8);
            if (fill_blocks > 65536) fill_blocks = 65536;
            hipLaunchKernelGGL(dwconv::fill_zero_kernel<>, dim3((unsigned)fill_blocks), dim3(256), 0, st, part, n);
        }
        const int segs = (s.L + dwconv::kSegLen - 1) / dwconv::kSegLen;
        for (int i = 0; i < p.passes; ++i) {
            const int d_lo = dmin + kMfmaMaxNDDw * i;
            int n = nd - kMfmaMaxNDDw * i < kMfmaMaxNDDw ? nd - kMfmaMaxNDDw * i : kMfmaMaxNDDw;
            if (n < 9) n = 9;       // (offsets past the last one of the filter reach no tap below K)
            // segments whose x window [1024 seg + 16 d_lo, 1024 (seg + 1) + 16 (d_lo + n)) meets the row
            long long lo = -(1024LL + 16LL * (d_lo + n) - 1);           // 1024 seg >= lo
            long long seg_lo = lo <= 0 ? 0 : (lo + 1023) / 1024;
            long long hi = (long long)s.L - 1 - 16LL * d_lo;            // 1024 seg <= hi
            long long seg_hi = hi < 0 ? -1 : hi / 1024;
            if (seg_hi > segs - 1) seg_hi = segs - 1;
            if (seg_lo > seg_hi) continue;                              // its taps stay zero
            const int rc = launch_dw_manypass_one(x, dy, part + (size_t)(i & 1) * set_floats, s, p, d_lo, n, (int)seg_lo,
                                                  (int)(seg_hi - seg_lo + 1), st);
            if (rc != DWCONV_OK) return rc == -1 ? DWCONV_ERR_LAUNCH : rc;
        }
        return launch_status();
    }
    if (nd > kMfmaMaxNDDw) {
        // p.passes launches over equal parts of the offsets, each into its own share of the slices (nine offsets at
        // least per launch: from there the kernel's tap buffer holds the 16 ND + 15 taps a part of the offsets owns;
        // offsets past the last one of the filter reach no tap below K)
        if (p.passes < 2 || p.passes != (nd + kMfmaMaxNDDw - 1) / kMfmaMaxNDDw || nd > kMfmaMaxNDDw3 || dw_out) return -1;
        const int per = (nd + p.passes - 1) / p.passes;
        const size_t pass_floats = (size_t)(p.S / p.passes) * (size_t)s.C * (size_t)s.K;
        for (int i = 0; i < p.passes; ++i) {
            int n = nd - i * per < per ? nd - i * per : per;
            if (n < 9) n = 9;
            const int rc = launch_dw_partial_wide_f32(x, dy, part + (size_t)i * pass_floats, nullptr, s, p, dmin + i * per, n, st);
            if (rc != DWCONV_OK) return rc;
        }
        return DWCONV_OK;
    }
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
