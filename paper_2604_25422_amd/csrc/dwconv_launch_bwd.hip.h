// Launchers of the fused backward kernels (templates on the storage type; instantiated by
// dwconv_launch_bwd_f32.hip and dwconv_launch_bwd_bf16.hip).
#pragma once
#include "dwconv_host.hip.h"
#include "dwconv_bwd_fused.hip.h"
#include "dwconv_bwd_fused_bf16.hip.h"

namespace dwhost {

// Fused input + weight gradient (matrix-core shape class).  Returns -1 when it does not apply.
template <typename T, int ND, int W>
int launch_bwd_fused_ndw(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out,
                         const Shape &s, const DwPlan &p, int dmin, hipStream_t st)
{
    if constexpr (std::is_same<T, bf16_t>::value) {
        constexpr size_t lds = dwconv::bwd_fused_bf16_lds_bytes(ND, W);
        static_assert(lds <= kMaxLdsBytes, "LDS budget");
        if (p.rows.on) {
            auto kernel = dwconv::bwd_fused_bf16_kernel<ND, W, true>;
            if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
            hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                               static_cast<const bf16_t *>(dy), static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(w),
                               static_cast<bf16_t *>(dx), part, static_cast<bf16_t *>(dw_out), 1, s.C, s.L, s.K, s.pad, dmin,
                               p.tiles_per_row, p.rows.map);
        } else {
            auto kernel = dwconv::bwd_fused_bf16_kernel<ND, W, false>;
            if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
            hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                               static_cast<const bf16_t *>(dy), static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(w),
                               static_cast<bf16_t *>(dx), part, static_cast<bf16_t *>(dw_out), s.B, s.C, s.L, s.K, s.pad, dmin,
                               p.tiles_per_row, p.rows.map);
        }
        return launch_status();
    } else {
    constexpr size_t lds = dwconv::bwd_fused_lds_bytes(ND, W);
    static_assert(lds <= kMaxLdsBytes, "LDS budget");
    if (p.rows.on) {
        auto kernel = dwconv::bwd_fused_kernel<ND, W, true>;
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                           static_cast<const float *>(dy), static_cast<const float *>(x), static_cast<const float *>(w),
                           static_cast<float *>(dx), part, static_cast<float *>(dw_out), 1, s.C, s.L, s.K, s.pad, dmin,
                           p.tiles_per_row, p.rows.map);
    } else {
        auto kernel = dwconv::bwd_fused_kernel<ND, W, false>;
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                           static_cast<const float *>(dy), static_cast<const float *>(x), static_cast<const float *>(w),
                           static_cast<float *>(dx), part, static_cast<float *>(dw_out), s.B, s.C, s.L, s.K, s.pad, dmin,
                           p.tiles_per_row, p.rows.map);
    }
    return launch_status();
    }
}

template <typename T, int ND>
int launch_bwd_fused_nd(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out,
                        const Shape &s, const DwPlan &p, int dmin, hipStream_t st)
{
    switch (p.wpb) {
    case 4: return launch_bwd_fused_ndw<T, ND, 4>(dy, x, w, dx, part, dw_out, s, p, dmin, st);
    case 5: return launch_bwd_fused_ndw<T, ND, 5>(dy, x, w, dx, part, dw_out, s, p, dmin, st);
    case 8: return launch_bwd_fused_ndw<T, ND, 8>(dy, x, w, dx, part, dw_out, s, p, dmin, st);
    case 16: return launch_bwd_fused_ndw<T, ND, 16>(dy, x, w, dx, part, dw_out, s, p, dmin, st);
    default: return -1;
    }
}

// Rows of at most 48 positions: sixteen rows per tile, one wave per (channel, slice).  Returns -1 when it does not apply.
template <typename T>
int launch_bwd_rowbatch(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out, bool *wrote_dw,
                        const Shape &s, const DwPlan &p, hipStream_t st)
{
    int dmin, nd;
    rows_batch_offsets(s.L, s.K, s.pad, &dmin, &nd);        // (rows of at most three blocks: at most five offsets)
    if (s.L > dwconv::kRbBwdMaxL || nd < 2 || nd > kMfmaMaxND || s.C < dwconv::kRbBwdWaves) return -1;
    if (!aligned_to(x, 4) || !aligned_to(dy, 4) || !aligned_to(dx, 4)) return -1;      // (rows that start on a dword)
    void *direct_rb = p.S_fused == 1 ? dw_out : nullptr;
    auto launch_rb = [&](auto kernel, size_t lds_rb) -> int {
        if (lds_rb > kMaxLdsBytes) return -1;
        if (lds_rb > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)((s.C + dwconv::kRbBwdWaves - 1) / dwconv::kRbBwdWaves), (unsigned)p.S_fused),
                           dim3(64 * dwconv::kRbBwdWaves), lds_rb, st, static_cast<const T *>(dy), static_cast<const T *>(x),
                           static_cast<const T *>(w), static_cast<T *>(dx), part, static_cast<T *>(direct_rb), s.B, s.C, s.L,
                           s.K, s.pad, dmin, p.rows.units);
        return launch_status();
    };
    const int m = (s.L + 15) / 16;              // the kernel is compiled per (block offsets, 16-blocks of a row)
    auto launch_m = [&](auto k1, auto k2, auto k3, int ndv) -> int {
        const size_t lds_rb = dwconv::rb_bwd_lds_bytes(s.L, ndv);
        return m == 1 ? launch_rb(k1, lds_rb) : m == 2 ? launch_rb(k2, lds_rb) : launch_rb(k3, lds_rb);
    };
    int rc = -1;
    if ((s.L % 4) != 0) {
        switch (nd) {
        case 2: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 2, 1, true>, dwconv::bwd_rowbatch_kernel<T, 2, 2, true>, dwconv::bwd_rowbatch_kernel<T, 2, 3, true>, 2); break;
        case 3: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 3, 1, true>, dwconv::bwd_rowbatch_kernel<T, 3, 2, true>, dwconv::bwd_rowbatch_kernel<T, 3, 3, true>, 3); break;
        case 4: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 4, 1, true>, dwconv::bwd_rowbatch_kernel<T, 4, 2, true>, dwconv::bwd_rowbatch_kernel<T, 4, 3, true>, 4); break;
        case 5: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 5, 1, true>, dwconv::bwd_rowbatch_kernel<T, 5, 2, true>, dwconv::bwd_rowbatch_kernel<T, 5, 3, true>, 5); break;
        case 6: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 6, 1, true>, dwconv::bwd_rowbatch_kernel<T, 6, 2, true>, dwconv::bwd_rowbatch_kernel<T, 6, 3, true>, 6); break;
        default: break;
        }
    } else {
        switch (nd) {
        case 2: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 2, 1, false>, dwconv::bwd_rowbatch_kernel<T, 2, 2, false>, dwconv::bwd_rowbatch_kernel<T, 2, 3, false>, 2); break;
        case 3: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 3, 1, false>, dwconv::bwd_rowbatch_kernel<T, 3, 2, false>, dwconv::bwd_rowbatch_kernel<T, 3, 3, false>, 3); break;
        case 4: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 4, 1, false>, dwconv::bwd_rowbatch_kernel<T, 4, 2, false>, dwconv::bwd_rowbatch_kernel<T, 4, 3, false>, 4); break;
        case 5: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 5, 1, false>, dwconv::bwd_rowbatch_kernel<T, 5, 2, false>, dwconv::bwd_rowbatch_kernel<T, 5, 3, false>, 5); break;
        case 6: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 6, 1, false>, dwconv::bwd_rowbatch_kernel<T, 6, 2, false>, dwconv::bwd_rowbatch_kernel<T, 6, 3, false>, 6); break;
        default: break;
        }
    }
    if (rc == DWCONV_OK && direct_rb) *wrote_dw = true;
    return rc;
}

template <typename T>
int launch_bwd_fused(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out, bool *wrote_dw,
                     const Shape &s, const DwPlan &p, hipStream_t st)
{
    *wrote_dw = false;
    if (p.longk) return -1;
    if (p.rows.batch) return launch_bwd_rowbatch<T>(dy, x, w, dx, part, dw_out, wrote_dw, s, p, st);
    if (p.rows.tall) return -1;                              // (two launches)
    // bf16 virtual rows: rows of even length (they start on a dword), pitch of whole 16-byte granules (otherwise the two
    // separate kernels)
    if (s.dtype == DWCONV_BF16 && p.rows.on &&
        ((s.L % 2) != 0 || (p.rows.map.P % 8) != 0 || !aligned_to(x, 4) || !aligned_to(dy, 4) || !aligned_to(dx, 4)))
        return -1;
    // bf16: rows that start on a dword
    if (s.dtype == DWCONV_BF16 && (s.L % 2) != 0) return -1;
    const int dmin = toeplitz_dmin(s.pad), dmax = toeplitz_dmax(s.K, s.pad);
    const int nd = dmax - dmin + 1;
    if (s.K < kMfmaMinK || nd < 2 || nd > kMfmaMaxND || s.L > kMfmaMaxL) return -1;
    // whole 16-byte granules; otherwise rows that start on a dword (see ragged_rows_ok), ordinary rows only
    const bool granular = (s.L % (s.dtype == DWCONV_BF16 ? 8 : 4)) == 0 && aligned_to(x, 16) && aligned_to(dy, 16) && aligned_to(dx, 16);
    if (!granular) {
        const bool short_ok = s.dtype == DWCONV_BF16 && (s.L % 4) == 0;      // (bf16 rows in granules of four: any ordinary length)
        const bool rows_ok = p.rows.on;                                      // (virtual rows; bf16: of even length, checked above)
        if ((!short_ok && !rows_ok && !ragged_rows_fused_ok(s, nd)) || (p.rows.on && !rows_ok) || !aligned_to(x, 4) ||
            !aligned_to(dy, 4) || !aligned_to(dx, 4))
            return -1;
    }
    void *direct = (p.single && p.S == 1) ? dw_out : nullptr;
    int rc = -1;
    switch (nd) {
    case 2: rc = launch_bwd_fused_nd<T, 2>(dy, x, w, dx, part, direct, s, p, dmin, st); break;
    case 3: rc = launch_bwd_fused_nd<T, 3>(dy, x, w, dx, part, direct, s, p, dmin, st); break;
    case 4: rc = launch_bwd_fused_nd<T, 4>(dy, x, w, dx, part, direct, s, p, dmin, st); break;
    case 5: rc = launch_bwd_fused_nd<T, 5>(dy, x, w, dx, part, direct, s, p, dmin, st); break;
    case 6: rc = launch_bwd_fused_nd<T, 6>(dy, x, w, dx, part, direct, s, p, dmin, st); break;
    default: break;
    }
    if (rc == DWCONV_OK && direct) *wrote_dw = true;
    return rc;
}

}  // namespace dwhost
