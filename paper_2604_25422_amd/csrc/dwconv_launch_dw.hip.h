// Launchers of the weight-gradient stage-1 kernels (templates on the storage type; instantiated by
// dwconv_launch_dw_f32.hip and dwconv_launch_dw_bf16.hip).
#pragma once
#include "dwconv_host.hip.h"
#include "dwconv_dw_bf16.hip.h"
#include "dwconv_valu.hip.h"

namespace dwhost {

template <typename T, int KCH>
void launch_dw_partial_valu(const void *x, const void *dy, float *part, const Shape &s, const DwPlan &p, hipStream_t st)
{
    if (p.valu_rows.on) {
        hipLaunchKernelGGL((dwconv::dw_partial_valu_kernel<T, kDwThreads, kDwTT, KCH, true>), dim3((unsigned)s.C, (unsigned)p.S),
                           dim3(kDwThreads), 0, st, static_cast<const T *>(x), static_cast<const T *>(dy), part, 1, s.C,
                           s.L, s.K, s.pad, p.valu_tiles_per_row, p.valu_items_per_slice, p.valu_rows.map);
        return;
    }
    hipLaunchKernelGGL((dwconv::dw_partial_valu_kernel<T, kDwThreads, kDwTT, KCH, false>), dim3((unsigned)s.C, (unsigned)p.S),
                       dim3(kDwThreads), 0, st, static_cast<const T *>(x), static_cast<const T *>(dy), part, s.B, s.C,
                       s.L, s.K, s.pad, p.valu_tiles_per_row, p.valu_items_per_slice, dwconv::RowsMap{0, 0, 0, 0, 0u, 0u});
}

// Rows of at most 128 positions, either storage type: sixteen rows per matrix tile.  dmin / nd: the block offsets inside a
// row (rows_batch_offsets); the kernel is compiled per number of 16-blocks of a row, not per number of offsets.
template <typename T, int W>
int launch_dw_rowbatch_w(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p, int dmin,
                         int nd, hipStream_t st)
{
    // rows of at most 128 positions, either storage type: sixteen rows per matrix tile
    auto launch_rb = [&](auto kernel, int nc) -> int {
        const size_t lds_rb = dwconv::rb_dw_lds_bytes(s.L, nd, W, nc);
        if (lds_rb > kMaxLdsBytes) return -1;
        if (lds_rb > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)(s.C / nc), (unsigned)p.S), dim3(64 * W), lds_rb, st,
                           static_cast<const T *>(x), static_cast<const T *>(dy), part, static_cast<T *>(dw_out), s.B,
                           s.C, s.L, s.K, s.pad, dmin, nd, p.tiles_per_row);
        return launch_status();
    };
    // (the kernel is compiled per number of 16-blocks of a row, not per number of block offsets)
    const int m = (s.L + 15) / 16;
    // rows that end inside a granule: the variant with the partial-granule code, four-wave workgroups only (the plan
    // asks for no others there)
    auto rag_rb = [&](auto mc) -> int {
        constexpr int MM = decltype(mc)::value;
        if ((s.L % 4) != 0) {
            if constexpr (W == dwconv::kWavesPerBlock) return launch_rb(dwconv::dw_rowbatch_kernel<T, MM, W, 1, true>, 1);
            else return -1;
        }
        return launch_rb(dwconv::dw_rowbatch_kernel<T, MM, W, 1, false>, 1);
    };
    if constexpr (W == dwconv::kWavesPerBlock) {
        if (p.dw_nc == 2) {
            switch (m) {
            case 1: return launch_rb(dwconv::dw_rowbatch_kernel<T, 1, W, 2, false>, 2);
            case 2: return launch_rb(dwconv::dw_rowbatch_kernel<T, 2, W, 2, false>, 2);
            case 3: return launch_rb(dwconv::dw_rowbatch_kernel<T, 3, W, 2, false>, 2);
            default: return -1;
            }
        }
    }
    switch (m) {
    case 1: return rag_rb(std::integral_constant<int, 1>{});
    case 2: return rag_rb(std::integral_constant<int, 2>{});
    case 3: return rag_rb(std::integral_constant<int, 3>{});
    case 4: return rag_rb(std::integral_constant<int, 4>{});
    case 5: return rag_rb(std::integral_constant<int, 5>{});
    case 6: return rag_rb(std::integral_constant<int, 6>{});
    case 7: return rag_rb(std::integral_constant<int, 7>{});
    case 8: return rag_rb(std::integral_constant<int, 8>{});
    default: return -1;
    }
}

template <typename T>
int launch_dw_rowbatch(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p, hipStream_t st)
{
    int dmin, nd;
    rows_batch_offsets(s.L, s.K, s.pad, &dmin, &nd);
    switch (p.wpb) {
    case 4: return launch_dw_rowbatch_w<T, 4>(x, dy, part, dw_out, s, p, dmin, nd, st);
    case 5: return launch_dw_rowbatch_w<T, 5>(x, dy, part, dw_out, s, p, dmin, nd, st);
    case 8: return launch_dw_rowbatch_w<T, 8>(x, dy, part, dw_out, s, p, dmin, nd, st);
    case 16: return launch_dw_rowbatch_w<T, 16>(x, dy, part, dw_out, s, p, dmin, nd, st);
    default: return -1;
    }
}

// One stage-1 launch on the matrix cores.  dw_out != nullptr only for single-slice plans.
template <typename T, int ND, int W>
int launch_dw_partial_mfma_ndw(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                               int dmin, hipStream_t st)
{
    if constexpr (std::is_same<T, float>::value) {
        // fp32 rows go from memory straight into LDS
        constexpr size_t lds = dwconv::dw_direct_lds_bytes(ND, W);
        static_assert(lds <= kMaxLdsBytes, "LDS budget");
        if (p.rows.on) {
            auto kernel = dwconv::dw_partial_direct_kernel<ND, W, true>;
            if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
            hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                               static_cast<const float *>(x), static_cast<const float *>(dy), part,
                               static_cast<float *>(dw_out), 1, s.C, s.L, s.K, s.pad, dmin, p.tiles_per_row, p.rows.map, 0,
                               s.K, 0, 0);
        } else {
            auto kernel = dwconv::dw_partial_direct_kernel<ND, W, false>;
            if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
            hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                               static_cast<const float *>(x), static_cast<const float *>(dy), part,
                               static_cast<float *>(dw_out), s.B, s.C, s.L, s.K, s.pad, dmin, p.tiles_per_row, p.rows.map,
                               0, s.K, 0, 0);
        }
    } else if (p.rows.on && (s.L % 2) == 0 && (p.rows.map.P % 8) == 0 && aligned_to(x, 4) && aligned_to(dy, 4)) {
        // bf16 short rows of even length (they start on a dword): the virtual row of a channel on the bf16 matrix instruction,
        // raw rows straight into LDS (B4096 C128 L200 K48: 247 -> 88 us against the widening kernel below)
        auto kernel = dwconv::dw_partial_bf16_kernel<ND, W, true>;
        constexpr size_t lds = dwconv::dw_bf16_lds_bytes(ND, W);
        static_assert(lds <= kMaxLdsBytes, "LDS budget");
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                           static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(dy), part,
                           static_cast<bf16_t *>(dw_out), 1, s.C, s.L, s.K, s.pad, dmin, p.tiles_per_row, 0, s.K, 0, 0,
                           p.rows.map);
    } else if (p.rows.on) {
        // bf16 short rows (longer than 64 positions): the virtual row of a channel, widened to fp32 through registers
        auto kernel = dwconv::dw_partial_mfma_kernel<T, ND, W, true>;
        constexpr size_t lds = dwconv::dw_mfma_lds_bytes(ND, W);
        static_assert(lds <= kMaxLdsBytes, "LDS budget");
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st, static_cast<const T *>(x),
                           static_cast<const T *>(dy), part, static_cast<T *>(dw_out), 1, s.C, s.L, s.K, s.pad, dmin,
                           p.tiles_per_row, p.rows.map);
    } else if ((s.L % 2) == 0 && aligned_to(x, 4) && aligned_to(dy, 4)) {
        // bf16 rows that start on a dword: raw rows straight into LDS, bf16 matrix instruction
        auto kernel = dwconv::dw_partial_bf16_kernel<ND, W>;
        constexpr size_t lds = dwconv::dw_bf16_lds_bytes(ND, W);
        static_assert(lds <= kMaxLdsBytes, "LDS budget");
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                           static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(dy), part,
                           static_cast<bf16_t *>(dw_out), s.B, s.C, s.L, s.K, s.pad, dmin, p.tiles_per_row, 0, s.K, 0, 0,
                           dwconv::RowsMap{0, 0, 0, 0, 0u, 0u});
    } else {
        auto kernel = dwconv::dw_partial_mfma_kernel<T, ND, W, false>;
        constexpr size_t lds = dwconv::dw_mfma_lds_bytes(ND, W);
        static_assert(lds <= kMaxLdsBytes, "LDS budget");
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st, static_cast<const T *>(x),
                           static_cast<const T *>(dy), part, static_cast<T *>(dw_out), s.B, s.C, s.L, s.K, s.pad, dmin,
                           p.tiles_per_row, p.rows.map);
    }
    return launch_status();
}

template <typename T, int ND>
int launch_dw_partial_mfma_nd(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                              int dmin, hipStream_t st)
{
    switch (p.wpb) {
    case 4: return launch_dw_partial_mfma_ndw<T, ND, 4>(x, dy, part, dw_out, s, p, dmin, st);
    case 5: return launch_dw_partial_mfma_ndw<T, ND, 5>(x, dy, part, dw_out, s, p, dmin, st);
    case 8: return launch_dw_partial_mfma_ndw<T, ND, 8>(x, dy, part, dw_out, s, p, dmin, st);
    case 16: return launch_dw_partial_mfma_ndw<T, ND, 16>(x, dy, part, dw_out, s, p, dmin, st);
    default: return -1;
    }
}

// Returns -1 when the shape or the pointers do not fit the matrix-core kernel.
template <typename T>
int launch_dw_partial_mfma(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                           hipStream_t st)
{
    const int dmin = toeplitz_dmin(s.pad), dmax = toeplitz_dmax(s.K, s.pad);
    const int nd = dmax - dmin + 1;
    // (rows of at most 128 positions: the sixteen-row kernel needs rows that start on a dword, nothing more)
    if (p.rows.batch) return (aligned_to(x, 4) && aligned_to(dy, 4)) ? launch_dw_rowbatch<T>(x, dy, part, dw_out, s, p, st) : -1;
    if (p.rows.tall) {
        if (!aligned_to(x, 4) || !aligned_to(dy, 4)) return -1;
        if constexpr (std::is_same<T, float>::value) return launch_dw_rowtall_f32(x, dy, part, s, p, st);
        else return launch_dw_rowtall_bf16(x, dy, part, s, p, st);
    }
    if (p.manypass) {
        if constexpr (std::is_same<T, float>::value) {
            if (!aligned_to(x, 16) || !aligned_to(dy, 16)) return -1;
            return launch_dw_partial_wide_f32(x, dy, part, nullptr, s, p, dmin, nd, st);
        } else {
            return launch_dw_partial_wide_bf16(x, dy, part, nullptr, s, p, dmin, nd, st);
        }
    }
    if (s.K < kMfmaMinK || nd < 2 || nd > mfma_max_nd_dw(s) || s.L > kMfmaMaxL) return -1;
    // whole granules of four elements; otherwise only the kernels that load rows straight into LDS apply (see ragged_rows_ok)
    const bool granular = (s.L % 4) == 0 && aligned_to(x, 4 * sizeof(T)) && aligned_to(dy, 4 * sizeof(T));
    // (bf16 virtual rows of even length: launch_dw_partial_mfma_ndw takes them on the kernel that loads raw rows into LDS)
    // (fp32 virtual rows of any length, up to six offsets: the kernel that loads rows straight into LDS)
    const bool rows_direct_bf16 = sizeof(T) == 2 && p.rows.on && (s.L % 2) == 0 && (p.rows.map.P % 8) == 0;
    const bool rows_direct_f32 = sizeof(T) == 4 && p.rows.on && nd <= kMfmaMaxND;
    const bool rows_direct = (rows_direct_bf16 || rows_direct_f32) && aligned_to(x, 4) && aligned_to(dy, 4);
    if (!granular && !rows_direct && (!ragged_rows_ok(s, nd) || p.rows.on || !aligned_to(x, 4) || !aligned_to(dy, 4))) return -1;
    if constexpr (std::is_same<T, float>::value) {
        if (nd > kMfmaMaxND) return launch_dw_partial_wide_f32(x, dy, part, dw_out, s, p, dmin, nd, st);
    } else {
        if (nd > kMfmaMaxND) return launch_dw_partial_wide_bf16(x, dy, part, dw_out, s, p, dmin, nd, st);
    }
    switch (nd) {
    case 2: return launch_dw_partial_mfma_nd<T, 2>(x, dy, part, dw_out, s, p, dmin, st);
    case 3: return launch_dw_partial_mfma_nd<T, 3>(x, dy, part, dw_out, s, p, dmin, st);
    case 4: return launch_dw_partial_mfma_nd<T, 4>(x, dy, part, dw_out, s, p, dmin, st);
    case 5: return launch_dw_partial_mfma_nd<T, 5>(x, dy, part, dw_out, s, p, dmin, st);
    case 6: return launch_dw_partial_mfma_nd<T, 6>(x, dy, part, dw_out, s, p, dmin, st);
    default: return -1;
    }
}

template <typename T, int GD>
int launch_dw_longk_gd(const void *x, const void *dy, float *part, const Shape &s, const DwPlan &p,
                       const dwconv::LongKDwGeom &g, hipStream_t st)
{
    // all slices start at zero: a group stores only the taps it owns
    auto fill = [&]() {
        const size_t n = (size_t)p.S * (size_t)s.C * (size_t)s.K;
        size_t fill_blocks = (n + 256 * 8 - 1) / (256 * 8);
        if (fill_blocks > 65536) fill_blocks = 65536;
        hipLaunchKernelGGL(dwconv::fill_zero_kernel<>, dim3((unsigned)fill_blocks), dim3(256), 0, st, part, n);
    };
    if constexpr (sizeof(T) == 2) {
        // bf16 storage: raw rows in LDS, bf16 matrix instruction
        const size_t lds = dwconv::longk_dw_bf16_lds_bytes(s.L);
        if (lds > kMaxLdsBytes || !allow_large_lds(dwconv::dw_longk_bf16_kernel<GD>)) return -1;
        fill();
        hipLaunchKernelGGL((dwconv::dw_longk_bf16_kernel<GD>), dim3((unsigned)s.C, (unsigned)p.lk_wgs, (unsigned)p.lk_rs),
                           dim3(64 * dwconv::kLkWaves), lds, st, static_cast<const bf16_t *>(x),
                           static_cast<const bf16_t *>(dy), part, g, *p.lk_table);
    } else {
        const size_t lds = dwconv::longk_dw_lds_bytes(s.L, g.NCH);
        if (lds > kMaxLdsBytes || !allow_large_lds(dwconv::dw_longk_kernel<T, GD>)) return -1;
        fill();
        hipLaunchKernelGGL((dwconv::dw_longk_kernel<T, GD>), dim3((unsigned)s.C, (unsigned)p.lk_wgs, (unsigned)p.lk_rs),
                           dim3(64 * dwconv::kLkWaves), lds, st, static_cast<const T *>(x), static_cast<const T *>(dy),
                           part, g, *p.lk_table);
    }
    return launch_status();
}

// Returns -1 when the pointers do not fit the long-filter matrix-core kernel.
template <typename T>
int launch_dw_partial_longk(const void *x, const void *dy, float *part, const Shape &s, const DwPlan &p, hipStream_t st)
{
    if (!aligned_to(x, 4 * sizeof(T)) || !aligned_to(dy, 4 * sizeof(T))) return -1;
    dwconv::LongKDwGeom g;
    g.B = s.B; g.C = s.C; g.L = s.L; g.K = s.K; g.pad = s.pad;
    g.dmin = toeplitz_dmin(s.pad); g.dmax = toeplitz_dmax(s.K, s.pad);
    g.NCH = (s.L + 63) / 64;
    g.bper = p.lk_bper;
    if (p.S != 2 * p.lk_rs) return -1;
    switch (p.lk_gd) {
    case 1: return launch_dw_longk_gd<T, 1>(x, dy, part, s, p, g, st);
    case 2: return launch_dw_longk_gd<T, 2>(x, dy, part, s, p, g, st);
    case 3: return launch_dw_longk_gd<T, 3>(x, dy, part, s, p, g, st);
    case 4: return launch_dw_longk_gd<T, 4>(x, dy, part, s, p, g, st);
    case 6: return launch_dw_longk_gd<T, 6>(x, dy, part, s, p, g, st);
    default: return launch_dw_longk_gd<T, 9>(x, dy, part, s, p, g, st);
    }
}

template <typename T>
int launch_dw_partial(const void *x, const void *dy, float *part, void *dw_out, bool *wrote_dw, const Shape &s,
                      const DwPlan &p, hipStream_t st)
{
    // dw_out: where a single-slice matrix-core launch may put the gradient itself (nullptr: always write part);
    // *wrote_dw tells the caller whether it did.
    if (wrote_dw) *wrote_dw = false;
    if (p.longk) {
        const int rc = launch_dw_partial_longk<T>(x, dy, part, s, p, st);
        if (rc >= 0) return rc;
    }
    void *direct = (p.single && p.S == 1) ? dw_out : nullptr;
    const int rc = launch_dw_partial_mfma<T>(x, dy, part, direct, s, p, st);
    if (rc >= 0) {
        if (wrote_dw && direct && rc == DWCONV_OK) *wrote_dw = true;
        return rc;
    }
    switch (p.kernel) {
    case DW_VALU_K8: launch_dw_partial_valu<T, 8>(x, dy, part, s, p, st); break;
    case DW_VALU_K32: launch_dw_partial_valu<T, 32>(x, dy, part, s, p, st); break;
    case DW_VALU_K64: launch_dw_partial_valu<T, 64>(x, dy, part, s, p, st); break;
    case DW_VALU_K256: launch_dw_partial_valu<T, 256>(x, dy, part, s, p, st); break;
    }
    return launch_status();
}

}  // namespace dwhost
