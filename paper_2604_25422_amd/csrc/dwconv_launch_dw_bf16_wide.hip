// Weight-gradient stage-1 kernels, bf16 storage, filters of 67 to 226 taps (a unit of its own, like the fp32 one).
#include "dwconv_host.hip.h"
#include "dwconv_dw_bf16.hip.h"

namespace dwhost {

// bf16, seven to sixteen block offsets: raw rows straight into LDS, bf16 matrix instruction, four-wave workgroups.
template <int ND>
int launch_dw_partial_wide_bf16_nd(const void *x, const void *dy, float *part, void *dw_out, const Shape &s,
                                   const DwPlan &p, int dmin, hipStream_t st)
{
    constexpr int W = dwconv::kWavesPerBlock;
    constexpr size_t lds = dwconv::dw_bf16_lds_bytes(ND, W);
    static_assert(lds <= kMaxLdsBytes, "LDS budget");
    if (p.rows.on || p.wpb != W) return -1;
    auto kernel = dwconv::dw_partial_bf16_kernel<ND, W>;
    if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
    hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st, static_cast<const bf16_t *>(x),
                       static_cast<const bf16_t *>(dy), part, static_cast<bf16_t *>(dw_out), s.B, s.C, s.L, s.K, s.pad,
                       dmin, p.tiles_per_row);
    return launch_status();
}

int launch_dw_partial_wide_bf16(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                                int dmin, int nd, hipStream_t st)
{
    if ((s.L % 8) != 0 || !aligned_to(x, 16) || !aligned_to(dy, 16)) return -1;
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
