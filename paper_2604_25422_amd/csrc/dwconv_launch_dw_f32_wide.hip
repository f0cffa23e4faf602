// Weight-gradient stage 1, fp32, filters of 67 taps and more on the register-resident kernel: one launch (seven to sixteen
// block offsets), two or three (up to forty-eight), or the many-launch form (beyond what the long-filter kernel's LDS holds).
// The kernels themselves are compiled in dwconv_launch_dw_f32_wide_{w4,multi,rows}.hip.
#include "dwconv_launch_dw_wide.hip.h"

namespace dwhost {

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
            // (one launch of the many-launch form: n offsets from d_lo, these segments of every row, the owned taps only)
            const int rc = launch_dw_wide_w4_f32(n, x, dy, part + (size_t)(i & 1) * set_floats, nullptr, s, p, d_lo, st, (int)seg_lo,
                                                 (int)(seg_hi - seg_lo + 1), sl, 1);
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
    if (nd < 7 || nd > kMfmaMaxNDDw) return -1;
    if (p.rows.on) return launch_dw_wide_rows_f32(nd, x, dy, part, dw_out, s, p, dmin, st);
    if (p.wpb == 4) return launch_dw_wide_w4_f32(nd, x, dy, part, dw_out, s, p, dmin, st, 0, -1, -1, 0);
    return launch_dw_wide_multi_f32(nd, x, dy, part, dw_out, s, p, dmin, st);
}

}  // namespace dwhost
