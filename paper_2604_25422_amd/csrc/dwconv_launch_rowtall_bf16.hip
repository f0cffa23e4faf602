// Rows of 132 to 512 positions with filters of the order of the row length, bf16 storage: forward / input gradient
// and stage 1 of the weight gradient on the sixteen-row kernels of dwconv_rowtall.hip.h.
#include "dwconv_host.hip.h"

namespace dwhost {

namespace {

dwconv::RowTallGeom rowtall_geom(const Shape &s, int pad, int reverse)
{
    dwconv::RowTallGeom g;
    int dmin, nd;
    rows_batch_offsets(s.L, s.K, pad, &dmin, &nd);
    g.B = s.B; g.C = s.C; g.L = s.L; g.K = s.K;
    g.pad = pad; g.reverse = reverse;
    g.dmin = dmin; g.dmax = dmin + nd - 1;
    g.m = (s.L + 15) / 16;
    g.n_units = 0; g.J = 0; g.win = 0;
    g.lg_recip = (unsigned)((1ull << 32) / (unsigned long long)((s.L + 3) / 4)) + 1u;
    return g;
}

}  // namespace

int launch_corr_rowtall_bf16(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st)
{
    typedef dwconv::bf16_t T;
    dwconv::RowTallGeom g = rowtall_geom(s, pad_eff, reverse);
    g.n_units = (s.B + dwconv::kRbRows - 1) / dwconv::kRbRows;
    auto kernel = dwconv::corr_rowtall_kernel<T>;
    const size_t lds = dwconv::rt_corr_lds_bytes(g.m);
    if (lds > kMaxLdsBytes) return -1;
    if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
    // one resident round of waves: J per channel, each walking units j, j + J, ...
    const long long resident = corr_wave_slots(kernel, 64 * dwconv::kRtWaves);
    long long J = resident / s.C;
    if (J < 1) J = 1;
    if (J > g.n_units) J = g.n_units;
    const long long upw = (g.n_units + J - 1) / J;
    J = (g.n_units + upw - 1) / upw;
    const long long blocks = ((long long)s.C * J + dwconv::kRtWaves - 1) / dwconv::kRtWaves;
    if (blocks > 0x1fffffffLL) return -1;
    g.J = (int)J;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(64 * dwconv::kRtWaves), lds, st, static_cast<const T *>(in),
                       static_cast<const T *>(f), static_cast<T *>(out), g);
    return launch_status();
}

int launch_dw_rowtall_bf16(const void *x, const void *dy, float *part, const Shape &s, const DwPlan &p, hipStream_t st)
{
    typedef dwconv::bf16_t T;
    dwconv::RowTallGeom g = rowtall_geom(s, s.pad, 0);
    g.n_units = (s.B + 3) / 4;
    const int nwin = (g.dmax - g.dmin + 1 + dwconv::kRtWindow - 1) / dwconv::kRtWindow;
    if (nwin != p.tall_windows || p.S % nwin != 0 || p.S / nwin > 65535) return -1;
    g.win = (g.dmax - g.dmin + 1 + nwin - 1) / nwin;                  // windows of equal size
    auto kernel = dwconv::dw_rowtall_kernel<T>;
    const size_t lds = dwconv::rt_dw_lds_bytes(g.m);
    if (lds > kMaxLdsBytes) return -1;
    if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
    hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)(p.S / nwin), (unsigned)nwin), dim3(64 * dwconv::kRtWaves), lds, st,
                       static_cast<const T *>(x), static_cast<const T *>(dy), part, g);
    return launch_status();
}

}  // namespace dwhost
