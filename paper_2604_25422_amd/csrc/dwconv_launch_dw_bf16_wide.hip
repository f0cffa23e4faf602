// Weight-gradient stage-1 kernels, bf16 storage, filters of 67 to 226 taps (a unit of its own, like the fp32 one).
#include "dwconv_host.hip.h"
#include "dwconv_dw_bf16.hip.h"

namespace dwhost {

// bf16, seven to sixteen block offsets: raw rows straight into LDS, bf16 matrix instruction, four-wave workgroups.
// seg0 / nseg / slices / own_only: see launch_dw_partial_wide_ndw of the fp32 unit.
template <int ND>
int launch_dw_partial_wide_bf16_nd(const void *x, const void *dy, float *part, void *dw_out, const Shape &s,
                                   const DwPlan &p, int dmin, hipStream_t st, int seg0 = 0, int nseg = -1, int slices = -1,
                                   int own_only = 0)
{
    constexpr int W = dwconv::kWavesPerBlock;
    constexpr size_t lds = dwconv::dw_bf16_lds_bytes(ND, W);
    static_assert(lds <= kMaxLdsBytes, "LDS budget");
    if (p.rows.on || p.wpb != W) return -1;
    auto kernel = dwconv::dw_partial_bf16_kernel<ND, W>;
    if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
    // the taps this launch owns: those its ND offsets can reach (all K of them when they cover the filter)
    int j0 = 16 * dmin + s.pad - 15, j1 = 16 * (dmin + ND - 1) + s.pad + 16;
    j0 = j0 < 0 ? 0 : (j0 > s.K ? s.K : j0);
    j1 = j1 < j0 ? j0 : (j1 > s.K ? s.K : j1);
    if (j1 - j0 > dwconv::dw_bf16_row_floats(ND)) return -1;
    if (nseg < 0) nseg = p.tiles_per_row;
    if (slices < 0) slices = p.S / p.passes;
    hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)slices), dim3(64 * W), lds, st,
                       static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(dy), part, static_cast<bf16_t *>(dw_out),
                       s.B, s.C, s.L, s.K, s.pad, dmin, nseg, j0, j1, seg0, own_only, dwconv::RowsMap{0, 0, 0, 0, 0u, 0u});
    return launch_status();
}

// One launch of the many-launch form (filters beyond the long-filter kernel's LDS): n (nine to sixteen) offsets from
// d_lo, segments [seg0, seg0 + nseg) of every row, the owned taps only.
static int launch_dw_manypass_one_bf16(const void *x, const void *dy, float *part, const Shape &s, const DwPlan &p, int d_lo,
                                       int n, int seg0, int nseg, hipStream_t st)
{
    const int sl = p.S / 2;
    switch (n) {
    case 9: return launch_dw_partial_wide_bf16_nd<9>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 10: return launch_dw_partial_wide_bf16_nd<10>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 11: return launch_dw_partial_wide_bf16_nd<11>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 12: return launch_dw_partial_wide_bf16_nd<12>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 13: return launch_dw_partial_wide_bf16_nd<13>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 14: return launch_dw_partial_wide_bf16_nd<14>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 15: return launch_dw_partial_wide_bf16_nd<15>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    case 16: return launch_dw_partial_wide_bf16_nd<16>(x, dy, part, nullptr, s, p, d_lo, st, seg0, nseg, sl, 1);
    default: return -1;
    }
}

int launch_dw_partial_wide_bf16(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                                int dmin, int nd, hipStream_t st)
{
    if ((s.L % 8) != 0 || !aligned_to(x, 16) || !aligned_to(dy, 16)) return -1;
    if (p.manypass) {
        // as the fp32 unit: sixteen block offsets per launch into two zero-filled sets of slices
        if (dw_out || p.wpb != dwconv::kWavesPerBlock || p.S < 2 || (p.S % 2) != 0 || p.rows.on) return -1;
        const int sl = p.S / 2;
        const size_t set_floats = (size_t)sl * (size_t)s.C * (size_t)s.K;
        {
            const size_t n = 2 * set_floats;
            size_t fill_blocks = (n + 256 * 8 - 1) / (256 * 8);
            if (fill_blocks > 65536) fill_blocks = 65536;
            hipLaunchKernelGGL(dwconv::fill_zero_kernel<>, dim3((unsigned)fill_blocks), dim3(256), 0, st, part, n);
        }
        const int segs = (s.L + dwconv::kSegLen - 1) / dwconv::kSegLen;
        for (int i = 0; i < p.passes; ++i) {
            const int d_lo = dmin + kMfmaMaxNDDw * i;
            int n = nd - kMfmaMaxNDDw * i < kMfmaMaxNDDw ? nd - kMfmaMaxNDDw * i : kMfmaMaxNDDw;
            if (n < 9) n = 9;
            long long lo = -(1024LL + 16LL * (d_lo + n) - 1);
            long long seg_lo = lo <= 0 ? 0 : (lo + 1023) / 1024;
            long long hi = (long long)s.L - 1 - 16LL * d_lo;
            long long seg_hi = hi < 0 ? -1 : hi / 1024;
            if (seg_hi > segs - 1) seg_hi = segs - 1;
            if (seg_lo > seg_hi) continue;
            const int rc = launch_dw_manypass_one_bf16(x, dy, part + (size_t)(i & 1) * set_floats, s, p, d_lo, n, (int)seg_lo,
                                                       (int)(seg_hi - seg_lo + 1), st);
            if (rc != DWCONV_OK) return rc == -1 ? DWCONV_ERR_LAUNCH : rc;
        }
        return launch_status();
    }
    if (nd > kMfmaMaxNDDw) {
        // p.passes launches over equal parts of the offsets, each into its own share of the slices (nine offsets at
        // least per launch: from there the kernel's tap buffer holds the 16 ND + 15 taps a part of the offsets owns;
        // offsets past the last one of the filter reach no tap below K)
        if (p.passes < 2 || p.passes != (nd + kMfmaMaxNDDw - 1) / kMfmaMaxNDDw || nd > kMfmaMaxNDDw4 || dw_out) return -1;
        const int per = (nd + p.passes - 1) / p.passes;
        const size_t pass_floats = (size_t)(p.S / p.passes) * (size_t)s.C * (size_t)s.K;
        for (int i = 0; i < p.passes; ++i) {
            int n = nd - i * per < per ? nd - i * per : per;
            if (n < 9) n = 9;
            const int rc = launch_dw_partial_wide_bf16(x, dy, part + (size_t)i * pass_floats, nullptr, s, p, dmin + i * per, n, st);
            if (rc != DWCONV_OK) return rc;
        }
        return DWCONV_OK;
    }
    switch (nd) {
    case 7: return launch_dw_partial_wide_bf16_nd<7>(x, dy, part, dw_out, s, p, dmin, st);
    case 8: return launch_dw_partial_wide_bf16_nd<8>(x, dy, part, dw_out, s, p, dmin, st);
    case 9: return launch_dw_partial_wide_bf16_nd<9>(x, dy, part, dw_out, s, p, dmin, st);
    case 10: return launch_dw_partial_wide_bf16_nd<10>(x, dy, part, dw_out, s, p, dmin, st);
    case 11: return launch_dw_partial_wide_bf16_nd<11>(x, dy, part, dw_out, s, p, dmin, st);
    case 12: return launch_dw_partial_wide_bf16_nd<12>(x, dy, part, dw_out, s, p, dmin, st);
    case 13: return launch_dw_partial_wide_bf16_nd<13>(x, dy, part, dw_out, s, p, dmin, st);
    case 14: return launch_dw_partial_wide_bf16_nd<14>(x, dy, part, dw_out, s, p, dmin, st);
    case 15: return launch_dw_partial_wide_bf16_nd<15>(x, dy, part, dw_out, s, p, dmin, st);
    case 16: return launch_dw_partial_wide_bf16_nd<16>(x, dy, part, dw_out, s, p, dmin, st);
    default: return -1;
    }
}

}  // namespace dwhost
