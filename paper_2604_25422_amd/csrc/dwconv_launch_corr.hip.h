// Launchers of the forward / input-gradient kernels (templates on the storage type; instantiated by
// dwconv_launch_corr_f32.hip and dwconv_launch_corr_bf16.hip).
//   out = correlate(in, f_eff, pad_eff): the forward is (x, w, pad); the input gradient is (dy, reversed w, K-1-pad).
#pragma once
#include "dwconv_host.hip.h"
#include "dwconv_valu.hip.h"

namespace dwhost {

template <typename T>
int launch_corr_valu(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st)
{
    constexpr int R = 4, THREADS = 256, KCH = 512;
    constexpr int TILE = R * THREADS;
    static_assert(TILE == dwconv::kSegLen, "plan_valu_rows counts tiles of this size");
    const ValuRows vr = plan_valu_rows(s);
    if (vr.on) {
        // short rows: tiles of the virtual row of every channel
        const long long blocks = (long long)s.C * vr.tiles;
        if (blocks > 0x7fffffffLL) return DWCONV_ERR_SHAPE;
        hipLaunchKernelGGL((dwconv::corr_valu_kernel<T, R, THREADS, KCH, true>), dim3((unsigned)blocks), dim3(THREADS), 0, st,
                           static_cast<const T *>(in), static_cast<const T *>(f), static_cast<T *>(out), s.C, s.L, s.K,
                           pad_eff, reverse, (int)vr.tiles, vr.map);
        return launch_status();
    }
    const long long tiles_per_row = ((long long)s.L + TILE - 1) / TILE;
    const long long blocks = (long long)s.B * s.C * tiles_per_row;
    if (blocks > 0x7fffffffLL) return DWCONV_ERR_SHAPE;
    hipLaunchKernelGGL((dwconv::corr_valu_kernel<T, R, THREADS, KCH, false>), dim3((unsigned)blocks), dim3(THREADS), 0, st,
                       static_cast<const T *>(in), static_cast<const T *>(f), static_cast<T *>(out), s.C, s.L, s.K,
                       pad_eff, reverse, (int)tiles_per_row, dwconv::RowsMap{0, 0, 0, 0, 0u, 0u});
    return launch_status();
}

// Rows of at most 128 positions: sixteen rows of a channel (or of two neighbouring channels) per unit.  The block
// offsets are cropped to those that stay inside a row of m 16-blocks (rows_batch_offsets), so a filter as long as the
// row or longer costs the block pairs of the row and nothing else.  Returns -1 when no kernel is compiled for the case.
// (seven to fifteen offsets: translation units of their own, dwconv_launch_corr_rows_*.hip)
int launch_corr_rowbatch_wide_f32(dwconv::RowBatchGeom &rg, int nd, const void *in, const void *f, void *out, const Shape &s,
                                  hipStream_t st);
int launch_corr_rowbatch_wide_bf16(dwconv::RowBatchGeom &rg, int nd, const void *in, const void *f, void *out, const Shape &s,
                                   hipStream_t st);

// The kernels for seven and more block offsets of rows of MB blocks (MB = 4: seven offsets at most).
template <typename T>
int launch_corr_rowbatch_wide_t(dwconv::RowBatchGeom &rg, int nd, const void *in, const void *f, void *out, const Shape &s,
                                hipStream_t st);

template <typename T, typename Kernel>
int launch_corr_rowbatch_kernel(Kernel kernel, dwconv::RowBatchGeom &rg, int nc, const void *in, const void *f, void *out,
                                const Shape &s, hipStream_t st)
{
    // one resident round of waves: J per channel group, each walking units j, j + J, ...
    const long long groups = s.C / nc;
    const long long resident = corr_wave_slots(kernel, 64 * dwconv::kRbCorrWaves);
    long long J = resident / groups;
    if (J < 1) J = 1;
    if (J > rg.n_units) J = rg.n_units;
    const long long upw = (rg.n_units + J - 1) / J;
    J = (rg.n_units + upw - 1) / upw;
    const long long blocks = (groups * J + dwconv::kRbCorrWaves - 1) / dwconv::kRbCorrWaves;
    if (blocks > 0x1fffffffLL) return -1;
    rg.J = (int)J;
    const size_t lds = (size_t)dwconv::kRbCorrWaves * dwconv::rb_corr_wave_floats(s.L, nc) * sizeof(float);
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(64 * dwconv::kRbCorrWaves), lds, st,
                       static_cast<const T *>(in), static_cast<const T *>(f), static_cast<T *>(out), rg);
    return launch_status();
}

template <typename T>
int launch_corr_rowbatch_wide_t(dwconv::RowBatchGeom &rg, int nd, const void *in, const void *f, void *out, const Shape &s,
                                hipStream_t st)
{
    auto go = [&](auto kernel) -> int { return launch_corr_rowbatch_kernel<T>(kernel, rg, 1, in, f, out, s, st); };
    if (rg.m <= 4) return nd == 7 ? go(dwconv::corr_rowbatch_kernel<T, 7, 1, 4, false>) : -1;
    switch (nd) {
    case 7: return go(dwconv::corr_rowbatch_kernel<T, 7, 1, 8, false>);
    case 8: return go(dwconv::corr_rowbatch_kernel<T, 8, 1, 8, false>);
    case 9: return go(dwconv::corr_rowbatch_kernel<T, 9, 1, 8, false>);
    case 10: return go(dwconv::corr_rowbatch_kernel<T, 10, 1, 8, false>);
    case 11: return go(dwconv::corr_rowbatch_kernel<T, 11, 1, 8, false>);
    case 12: return go(dwconv::corr_rowbatch_kernel<T, 12, 1, 8, false>);
    case 13: return go(dwconv::corr_rowbatch_kernel<T, 13, 1, 8, false>);
    case 14: return go(dwconv::corr_rowbatch_kernel<T, 14, 1, 8, false>);
    case 15: return go(dwconv::corr_rowbatch_kernel<T, 15, 1, 8, false>);
    default: return -1;
    }
}

template <typename T>
int launch_corr_rowbatch(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse,
                         const RowsPlan &rp, hipStream_t st)
{
    int dmin, nd;
    rows_batch_offsets(s.L, s.K, pad_eff, &dmin, &nd);
    dwconv::RowBatchGeom rg;
    rg.B = s.B; rg.C = s.C; rg.L = s.L; rg.K = s.K;
    rg.pad = pad_eff; rg.reverse = reverse; rg.dmin = dmin;
    rg.m = (s.L + 15) / 16;
    rg.n_units = rp.units;
    // two channels per wave where that makes whole cache lines of rows that are not, or at least longer pieces;
    // rows of at most 48 positions and at most five block offsets (register budget of the kernel)
    // (two channels are one piece of 2 L elements cut into granules: rows of whole granules)
    const int nc = (s.C % 2 == 0 && (s.L * (int)sizeof(T)) % 128 != 0 && s.L <= 48 && nd <= 5 && (s.L % 4) == 0) ? 2 : 1;
    const bool rag = (s.L % 4) != 0;                   // rows that end inside a granule
    auto launch_batch = [&](auto kernel) -> int { return launch_corr_rowbatch_kernel<T>(kernel, rg, nc, in, f, out, s, st); };
    if (nd > kMfmaMaxND) {
        if (rag) return -1;
        if constexpr (std::is_same<T, float>::value) return launch_corr_rowbatch_wide_f32(rg, nd, in, f, out, s, st);
        else return launch_corr_rowbatch_wide_bf16(rg, nd, in, f, out, s, st);
    }
    if (nc == 2) {
        switch (nd) {
        case 2: return launch_batch(dwconv::corr_rowbatch_kernel<T, 2, 2, 3, false>);
        case 3: return launch_batch(dwconv::corr_rowbatch_kernel<T, 3, 2, 3, false>);
        case 4: return launch_batch(dwconv::corr_rowbatch_kernel<T, 4, 2, 3, false>);
        case 5: return launch_batch(dwconv::corr_rowbatch_kernel<T, 5, 2, 3, false>);
        default: return -1;
        }
    }
    if (rg.m <= 4) {
        switch (nd) {
        case 2: return rag ? launch_batch(dwconv::corr_rowbatch_kernel<T, 2, 1, 4, true>) : launch_batch(dwconv::corr_rowbatch_kernel<T, 2, 1, 4, false>);
        case 3: return rag ? launch_batch(dwconv::corr_rowbatch_kernel<T, 3, 1, 4, true>) : launch_batch(dwconv::corr_rowbatch_kernel<T, 3, 1, 4, false>);
        case 4: return rag ? launch_batch(dwconv::corr_rowbatch_kernel<T, 4, 1, 4, true>) : launch_batch(dwconv::corr_rowbatch_kernel<T, 4, 1, 4, false>);
        case 5: return rag ? launch_batch(dwconv::corr_rowbatch_kernel<T, 5, 1, 4, true>) : launch_batch(dwconv::corr_rowbatch_kernel<T, 5, 1, 4, false>);
        case 6: return rag ? launch_batch(dwconv::corr_rowbatch_kernel<T, 6, 1, 4, true>) : launch_batch(dwconv::corr_rowbatch_kernel<T, 6, 1, 4, false>);
        default: return -1;
        }
    }
    switch (nd) {                              // rows of five to eight blocks
    case 2: return rag ? launch_batch(dwconv::corr_rowbatch_kernel<T, 2, 1, 8, true>) : launch_batch(dwconv::corr_rowbatch_kernel<T, 2, 1, 8, false>);
    case 3: return rag ? launch_batch(dwconv::corr_rowbatch_kernel<T, 3, 1, 8, true>) : launch_batch(dwconv::corr_rowbatch_kernel<T, 3, 1, 8, false>);
    case 4: return rag ? launch_batch(dwconv::corr_rowbatch_kernel<T, 4, 1, 8, true>) : launch_batch(dwconv::corr_rowbatch_kernel<T, 4, 1, 8, false>);
    case 5: return rag ? launch_batch(dwconv::corr_rowbatch_kernel<T, 5, 1, 8, true>) : launch_batch(dwconv::corr_rowbatch_kernel<T, 5, 1, 8, false>);
    case 6: return rag ? launch_batch(dwconv::corr_rowbatch_kernel<T, 6, 1, 8, true>) : launch_batch(dwconv::corr_rowbatch_kernel<T, 6, 1, 8, false>);
    default: return -1;
    }
}

// One launch of a forward / input-gradient kernel on the virtual rows of the channels (short rows, see RowsMap): slots
// ordered (virtual segment, channel).
template <typename T, typename Kernel>
int launch_corr_vrows_kernel(Kernel kernel, dwconv::CorrGeom g, const RowsPlan &rp, const void *in, const void *f, void *out,
                             const Shape &s, hipStream_t st)
{
    constexpr int kThreads = 64 * dwconv::kCorrWavesPerBlock;
    const long long total = (long long)rp.nvs * s.C;
    if (total > 0x3fffffffLL) return -1;
    g.rows = rp.nvs;
    g.segs_per_row = s.C;
    const long long resident = corr_wave_slots(kernel, kThreads);
    long long spw = (total + resident - 1) / resident;
    if (spw < 1) spw = 1;
    long long waves = (total + spw - 1) / spw;
    if (s.C <= resident) {                                // whole virtual segments per round: channel fixed
        long long J = resident / s.C;
        if (J > rp.nvs) J = rp.nvs;
        const long long rounds = (rp.nvs + J - 1) / J;
        J = (rp.nvs + rounds - 1) / rounds;
        waves = J * s.C;
    }
    const long long blocks = (waves + dwconv::kCorrWavesPerBlock - 1) / dwconv::kCorrWavesPerBlock;
    g.n_waves = (int)waves;
    g.step_rows = g.n_waves / g.segs_per_row;
    g.step_seg = g.n_waves % g.segs_per_row;
    g.step_c = 0;
    g.walk_segs = g.segs_per_row; g.n_main = g.n_waves; g.n_light = 0; g.step_c_light = 0;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, static_cast<const T *>(in),
                       static_cast<const T *>(f), static_cast<T *>(out), g, rp.map);
    return launch_status();
}
// (fp32, seven to sixteen block offsets on virtual rows: a translation unit of its own, dwconv_launch_corr_rows_f32.hip)
int launch_corr_vrows_wide_f32(const dwconv::CorrGeom &g, const RowsPlan &rp, int nd, const void *in, const void *f, void *out,
                               const Shape &s, hipStream_t st);

// Returns -1 when the shape or the pointers do not fit the matrix-core kernel.
template <typename T>
int launch_corr_mfma(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st)
{
    const int dmin = toeplitz_dmin(pad_eff), dmax = toeplitz_dmax(s.K, pad_eff);
    const int nd = dmax - dmin + 1;
    const RowsPlan rp = plan_rows(s);
    // (the sixteen-row kernels of short rows move granules with buffer loads and stores that need dword alignment only)
    if (rp.batch) return (aligned_to(in, 4) && aligned_to(out, 4)) ? launch_corr_rowbatch<T>(in, f, out, s, pad_eff, reverse, rp, st) : -1;
    if (rp.tall) {
        if (!aligned_to(in, 4) || !aligned_to(out, 4)) return -1;
        if constexpr (std::is_same<T, float>::value) return launch_corr_rowtall_f32(in, f, out, s, pad_eff, reverse, st);
        else return launch_corr_rowtall_bf16(in, f, out, s, pad_eff, reverse, st);
    }
    if (s.K < kMfmaMinK || nd < 2 || nd > mfma_max_nd(s.dtype) || s.L > kMfmaMaxL) return -1;
    // whole granules of four elements; otherwise only the kernels that load rows straight into LDS apply (see ragged_rows_ok)
    const bool granular = (s.L % 4) == 0 && aligned_to(in, 4 * sizeof(T)) && aligned_to(out, 4 * sizeof(T));
    // bf16 virtual rows on the kernels that load raw rows straight into LDS: rows of even length (they start on a dword),
    // pitch a multiple of 8; fp32 virtual rows of any length on any fp32 tensor: the kernel that loads rows straight into
    // LDS (up to six offsets)
    const bool rows_direct_bf16 = sizeof(T) == 2 && rp.on && (s.L % 2) == 0 && (rp.map.P % 8) == 0 && aligned_to(in, 4) && aligned_to(out, 4);
    const bool rows_direct_f32 = sizeof(T) == 4 && rp.on && nd <= kMfmaMaxND;
    if (!granular && !rows_direct_bf16 && !rows_direct_f32 && (!ragged_rows_ok(s, nd) || !aligned_to(in, 4) || !aligned_to(out, 4))) return -1;
    // block offsets the long-filter kernel takes too (fp32 eleven to sixteen, bf16 seven to sixteen): only where rows
    // fill their 1024-position segments to three quarters (shorter rows do less work on the long-filter kernel,
    // which contracts in-row block pairs only)
    if (!rp.on && nd >= longk_corr_min_nd(s.dtype) &&
        4ll * s.L < 3ll * (((long long)s.L + dwconv::kSegLen - 1) / dwconv::kSegLen * dwconv::kSegLen))
        return -1;
    const long long rows = (long long)s.B * s.C;
    const long long segs_per_row = (s.L + dwconv::kSegLen - 1) / dwconv::kSegLen;
    const long long total_segs = rows * segs_per_row;
    if (total_segs > 0x3fffffffLL) return -1;           // the kernel's segment walk is 32-bit
    dwconv::CorrGeom g;
    g.C = s.C; g.L = s.L; g.K = s.K; g.rows = (int)rows;
    g.pad = pad_eff; g.reverse = reverse; g.dmin = dmin;
    g.segs_per_row = (int)segs_per_row;
    g.walk_segs = (int)segs_per_row; g.n_main = 0; g.n_light = 0; g.step_c_light = 0;
    constexpr int kThreads = 64 * dwconv::kCorrWavesPerBlock;
    const dwconv::RowsMap no_rows{0, 0, 0, 0, 0u, 0u};
    // One resident round of waves, each walking segments wave, wave + n_waves, ...
    // slot_cap: the most wave slots to use.  balance_target > 0 (the kernels that load rows straight into LDS): the
    // number of waves is chosen among whole numbers J of batch entries per round (J * C * segments per row waves, which
    // keeps a wave on one channel) for even loading, the one nearest balance_target among the best: every SIMD gets
    // the same number of waves (a multiple of 1024 waves: with 2560 waves two SIMDs of a compute unit carry three
    // waves and two carry two, and the launch takes as long as the three) and the rounds divide the batch
    // (B32 C256 L4100 K64: 70.3 us with 2560 waves, 65.3 with 3840, 62.4 with 5120; L3000: 43.5 us with 3072).
    // own_light_waves (the kernels that have them): a ragged last segment of at most 512 positions (two live quarters)
    // is left out of this walk and gets waves of its own - about four per compute unit, more for short rows, a whole
    // number of times C where C allows (they then stay on one channel), and out of the resident round, so that all waves
    // of the launch start together.  The others then walk whole segments
    // only, in the order and number of a shape without the ragged end (fwd, B32 C256: L4160 K16 54.9 -> 50.5 us against
    // 48.8 us at L4096; L8196 K16 127 -> 104 us; L4100 K64 62.8 -> 58.4 us).  Where that would take more than a third of
    // the resident waves the light segments stay in the walk.
    auto launch = [&](auto kernel, auto *pi, auto *pf, auto *po, long long slot_cap = kTargetWaves,
                      long long balance_target = 0, bool own_light_waves = false) -> int {
        const long long capacity = balance_target > 0 ? resident_waves(kernel, kThreads) : corr_wave_slots(kernel, kThreads);
        const int last = s.L % dwconv::kSegLen;
        long long n_light = 0;
        if (own_light_waves && balance_target > 0 && last != 0 && last <= dwconv::kSegLen / 2 && segs_per_row >= 2) {
            // a light segment costs its wave about a microsecond (a memory round trip), a row of the walk about
            // 2 L sizeof(T) / 5 TB/s spread over all waves: enough light waves to be done in 0.6 of the launch
            const long long need = (long long)(5.0e6 / (0.6 * 2.0 * (double)s.L * (double)sizeof(T))) + 1;
            const long long want = need > 1024 ? need : 1024;
            n_light = s.C >= want ? s.C : (long long)s.C * ((want + s.C - 1) / s.C);
            if (n_light > rows) n_light = rows;
            if (3 * n_light > capacity) n_light = 0;
        }
        const long long walk_segs = segs_per_row - (n_light > 0 ? 1 : 0);
        const long long walk_total = rows * walk_segs;
        long long resident = capacity - n_light < slot_cap ? capacity - n_light : slot_cap;
        long long spw = (walk_total + resident - 1) / resident;      // segments per wave, rounded up
        if (spw < 1) spw = 1;
        long long waves = (walk_total + spw - 1) / spw;
        // A whole number of batch entries per round where one fits: the stride of the walk is then a multiple of
        // C rows, a wave stays on one channel and loads its Toeplitz operands once.
        const long long per_b = (long long)s.C * walk_segs;
        if (per_b <= resident) {
            long long J = resident / per_b;
            if (J > s.B) J = s.B;
            if (balance_target > 0) {
                const long long simds = 4LL * kComputeUnits;
                long long best_j = 1;
                double best = -1.0;
                for (long long j = 1; j <= J; ++j) {
                    const long long w = j * per_b, rounds = (s.B + j - 1) / j;
                    const double even_simd = (double)w / (double)(simds * ((w + simds - 1) / simds));
                    const double even_rounds = (double)s.B / (double)(j * rounds);
                    const double near = 1.0 - 0.02 * (double)(w > balance_target ? w - balance_target : balance_target - w) /
                                                  (double)balance_target;
                    const double score = even_simd * even_rounds * near * (w < simds * 2 ? 0.8 : 1.0);
                    if (score > best) { best = score; best_j = j; }
                }
                J = best_j;
            } else {
                const long long rounds = (s.B + J - 1) / J;
                J = (s.B + rounds - 1) / rounds;                       // same number of rounds, evened out
            }
            waves = J * per_b;
        }
        g.walk_segs = (int)walk_segs;
        g.n_main = (int)waves;
        g.n_light = (int)n_light;
        g.step_c_light = (int)(n_light % s.C);
        g.n_waves = (int)(waves + n_light);
        g.step_rows = g.n_main / g.walk_segs;
        g.step_seg = g.n_main % g.walk_segs;
        g.step_c = g.step_rows % s.C;
        const long long blocks = (g.n_waves + dwconv::kCorrWavesPerBlock - 1) / dwconv::kCorrWavesPerBlock;
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, pi, pf, po, g, no_rows);
        return launch_status();
    };
    if (!granular && rp.on && !rows_direct_bf16 && !rows_direct_f32) return -1;
    {
        // longer short rows: segments of the virtual row of a channel, slots ordered (virtual segment, channel)
        if (rp.on) {
            auto launch_rows = [&](auto kernel) -> int { return launch_corr_vrows_kernel<T>(kernel, g, rp, in, f, out, s, st); };
            if constexpr (sizeof(T) == 2) {
                // bf16 rows of even length: raw rows straight into LDS, bf16 matrix instruction (B4096 C128 L200
                // K48: 186 -> 104 us against the widening kernel below, which needs whole granules of four)
                if (rows_direct_bf16) {
                    switch (nd) {
                    case 2: return launch_rows(dwconv::corr_direct_bf16_kernel<2, true>);
                    case 3: return launch_rows(dwconv::corr_direct_bf16_kernel<3, true>);
                    case 4: return launch_rows(dwconv::corr_direct_bf16_kernel<4, true>);
                    case 5: return launch_rows(dwconv::corr_direct_bf16_kernel<5, true>);
                    case 6: return launch_rows(dwconv::corr_direct_bf16_kernel<6, true>);
                    default: break;
                    }
                }
            }
            if constexpr (std::is_same<T, float>::value) {
                // fp32 rows that are not whole granules of four, or tensors that are only element-aligned (rows of whole
                // aligned granules: the register-staged kernel below, 1 to 4 % faster there)
                if (!granular) {
                    switch (nd) {
                    case 2: return launch_rows(dwconv::corr_direct_kernel<2, true>);
                    case 3: return launch_rows(dwconv::corr_direct_kernel<3, true>);
                    case 4: return launch_rows(dwconv::corr_direct_kernel<4, true>);
                    case 5: return launch_rows(dwconv::corr_direct_kernel<5, true>);
                    case 6: return launch_rows(dwconv::corr_direct_kernel<6, true>);
                    default: return -1;
                    }
                }
            }
            if (!granular) return -1;             // (the kernels below move whole granules of four)
            switch (nd) {
            case 2: return launch_rows(dwconv::corr_mfma_kernel<T, 2, true>);
            case 3: return launch_rows(dwconv::corr_mfma_kernel<T, 3, true>);
            case 4: return launch_rows(dwconv::corr_mfma_kernel<T, 4, true>);
            case 5: return launch_rows(dwconv::corr_mfma_kernel<T, 5, true>);
            case 6: return launch_rows(dwconv::corr_mfma_kernel<T, 6, true>);
            default: break;
            }
            if constexpr (std::is_same<T, float>::value) return launch_corr_vrows_wide_f32(g, rp, nd, in, f, out, s, st);
            return -1;
        }
    }
    if constexpr (sizeof(T) == 2) {
        // bf16 storage: the bf16 matrix instruction when 16-byte granules of 8 elements line up
        const bool whole8 = (s.L % 8) == 0 && aligned_to(in, 16) && aligned_to(out, 16);
        if (whole8 || (nd <= kMfmaMaxND && (s.L % 2) == 0 && aligned_to(in, 4) && aligned_to(out, 4))) {
            const bf16_t *pi = static_cast<const bf16_t *>(in), *pf = static_cast<const bf16_t *>(f);
            bf16_t *po = static_cast<bf16_t *>(out);
            {
                // two to six block offsets: rows straight into LDS, refilled in place (B128 C768 L1024 K32: 72 us
                // against 76 us through staging registers; a wave has half the bytes of an fp32 one in flight, and a
                // full round of sixteen waves per compute unit is the fastest here)
                const bool ragged_last = (s.L % dwconv::kSegLen) != 0;      // (then: balanced wave count, own waves for light segments)
                switch (nd) {
                case 2: return launch(dwconv::corr_direct_bf16_kernel<2>, pi, pf, po, kTargetWaves, ragged_last ? kTargetWaves : 0, true);
                case 3: return launch(dwconv::corr_direct_bf16_kernel<3>, pi, pf, po, kTargetWaves, ragged_last ? kTargetWaves : 0, true);
                case 4: return launch(dwconv::corr_direct_bf16_kernel<4>, pi, pf, po, kTargetWaves, ragged_last ? kTargetWaves : 0, true);
                case 5: return launch(dwconv::corr_direct_bf16_kernel<5>, pi, pf, po, kTargetWaves, ragged_last ? kTargetWaves : 0, true);
                case 6: return launch(dwconv::corr_direct_bf16_kernel<6>, pi, pf, po, kTargetWaves, ragged_last ? kTargetWaves : 0, true);
                // (seven to nine offsets would still fit the window's tail load; measured no faster than the register-staged
                // kernel below: B128 C768 L1024 K128 81.6 against 80.3 us)
                default: break;
                }
            }
            if (!whole8) return -1;
            switch (nd) {
            case 7: return launch(dwconv::corr_mfma_bf16_kernel<7>, pi, pf, po);
            case 8: return launch(dwconv::corr_mfma_bf16_kernel<8>, pi, pf, po);
            case 9: return launch(dwconv::corr_mfma_bf16_kernel<9>, pi, pf, po);
            case 10: return launch(dwconv::corr_mfma_bf16_kernel<10>, pi, pf, po);
            case 11: return launch(dwconv::corr_mfma_bf16_kernel<11>, pi, pf, po);
            case 12: return launch(dwconv::corr_mfma_bf16_kernel<12>, pi, pf, po);
            case 13: return launch(dwconv::corr_mfma_bf16_kernel<13>, pi, pf, po);
            case 14: return launch(dwconv::corr_mfma_bf16_kernel<14>, pi, pf, po);
            case 15: return launch(dwconv::corr_mfma_bf16_kernel<15>, pi, pf, po);
            case 16: return launch(dwconv::corr_mfma_bf16_kernel<16>, pi, pf, po);
            default: return -1;
            }
        }
    }
    const T *pi = static_cast<const T *>(in), *pf = static_cast<const T *>(f);
    T *po = static_cast<T *>(out);
    if constexpr (std::is_same<T, float>::value) {
        // fp32, two to six block offsets: rows straight into LDS, refilled in place.  Wave slots aimed at: fewer than a
        // full resident round, because a launch is the time its bytes take plus a fill and a drain that grow with the
        // bytes in flight (B32 C256 L4096: K = 7 93 us with 8 waves per compute unit, 96 us with 12 or 16; K = 64 51.4 /
        // 50.8 / 50.9 us with 8 / 12 / 16, the matrix pipe wanting more than two waves per SIMD there); up to 20 per
        // compute unit where that is what loads the SIMDs evenly (see `launch`)
        const long long target = (long long)kComputeUnits * (nd <= 3 ? 8 : 14), cap = (long long)kComputeUnits * (nd <= 3 ? 12 : 20);
        switch (nd) {
        case 2: return launch(dwconv::corr_direct_kernel<2>, pi, pf, po, cap, target, true);
        case 3: return launch(dwconv::corr_direct_kernel<3>, pi, pf, po, cap, target, true);
        case 4: return launch(dwconv::corr_direct_kernel<4>, pi, pf, po, cap, target, true);
        case 5: return launch(dwconv::corr_direct_kernel<5>, pi, pf, po, cap, target, true);
        case 6: return launch(dwconv::corr_direct_kernel<6>, pi, pf, po, cap, target, true);
        default: break;
        }
    }
    // (fp32 rows that are not whole granules: the register-staged kernel below takes them too, see ragged_rows_ok)
    if (!granular && !std::is_same<T, float>::value) return -1;
    if constexpr (!std::is_same<T, float>::value) {
        // (bf16 rows of odd length in whole granules of four: widened to fp32 on the way into LDS)
        switch (nd) {
        case 2: return launch(dwconv::corr_mfma_kernel<T, 2, false>, pi, pf, po);
        case 3: return launch(dwconv::corr_mfma_kernel<T, 3, false>, pi, pf, po);
        case 4: return launch(dwconv::corr_mfma_kernel<T, 4, false>, pi, pf, po);
        case 5: return launch(dwconv::corr_mfma_kernel<T, 5, false>, pi, pf, po);
        case 6: return launch(dwconv::corr_mfma_kernel<T, 6, false>, pi, pf, po);
        default: break;
        }
    }
    if constexpr (std::is_same<T, float>::value) {
        if ((s.L % 4) != 0) {
            switch (nd) {
            case 7: return launch(dwconv::corr_mfma_kernel<float, 7, false, true>, pi, pf, po);
            case 8: return launch(dwconv::corr_mfma_kernel<float, 8, false, true>, pi, pf, po);
            case 9: return launch(dwconv::corr_mfma_kernel<float, 9, false, true>, pi, pf, po);
            case 10: return launch(dwconv::corr_mfma_kernel<float, 10, false, true>, pi, pf, po);
            case 11: return launch(dwconv::corr_mfma_kernel<float, 11, false, true>, pi, pf, po);
            case 12: return launch(dwconv::corr_mfma_kernel<float, 12, false, true>, pi, pf, po);
            case 13: return launch(dwconv::corr_mfma_kernel<float, 13, false, true>, pi, pf, po);
            case 14: return launch(dwconv::corr_mfma_kernel<float, 14, false, true>, pi, pf, po);
            default: return -1;                // (fifteen and sixteen offsets: no registers left for the element stores)
            }
        }
        switch (nd) {
        case 7: return launch(dwconv::corr_mfma_kernel<float, 7, false>, pi, pf, po);
        case 8: return launch(dwconv::corr_mfma_kernel<float, 8, false>, pi, pf, po);
        case 9: return launch(dwconv::corr_mfma_kernel<float, 9, false>, pi, pf, po);
        case 10: return launch(dwconv::corr_mfma_kernel<float, 10, false>, pi, pf, po);
        case 11: return launch(dwconv::corr_mfma_kernel<float, 11, false>, pi, pf, po);
        case 12: return launch(dwconv::corr_mfma_kernel<float, 12, false>, pi, pf, po);
        case 13: return launch(dwconv::corr_mfma_kernel<float, 13, false>, pi, pf, po);
        case 14: return launch(dwconv::corr_mfma_kernel<float, 14, false>, pi, pf, po);
        case 15: return launch(dwconv::corr_mfma_kernel<float, 15, false>, pi, pf, po);
        case 16: return launch(dwconv::corr_mfma_kernel<float, 16, false>, pi, pf, po);
        default: break;
        }
    }
    return -1;
}

// Filters too long for the register-resident Toeplitz form: whole rows and the whole filter in LDS.
// Returns -1 when the shape or the pointers do not fit.
template <typename T>
int launch_corr_longk(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st)
{
    const int dmin = toeplitz_dmin(pad_eff), dmax = toeplitz_dmax(s.K, pad_eff);
    if (dmax - dmin + 1 <= longk_corr_min_nd(s.dtype) - 1 || (s.L % 4) != 0) return -1;
    const int NB = (s.L + 15) / 16;
    if (!aligned_to(in, 4 * sizeof(T)) || !aligned_to(out, 4 * sizeof(T))) return -1;
    if (s.K > dwconv::kLkMaxK || NB > dwconv::kLkMaxBlocks) {
        // beyond what LDS holds whole: pieces of 4096 outputs, filter chunks of 4096 taps
        dwconv::LongKTileGeom tg;
        tg.B = s.B; tg.C = s.C; tg.L = s.L; tg.K = s.K; tg.pad = pad_eff; tg.reverse = reverse; tg.NB = NB;
        tg.NP = (s.L + dwconv::kLkTilePiece - 1) / dwconv::kLkTilePiece;
        tg.NCK = (s.K + dwconv::kLkTileChunk - 1) / dwconv::kLkTileChunk;
        const long long gy = (((long long)s.B + 1) / 2) * tg.NP;
        if (gy > 65535 || s.L > kMfmaMaxL) return -1;
        if constexpr (sizeof(T) == 2) {
            // bf16 storage: raw bf16 operands on the bf16 matrix instruction
            const size_t lds = dwconv::longk_tiled_bf16_lds_bytes();
            if (lds > kMaxLdsBytes || !allow_large_lds(dwconv::corr_longk_tiled_bf16_kernel<>)) return -1;
            hipLaunchKernelGGL((dwconv::corr_longk_tiled_bf16_kernel<>), dim3((unsigned)s.C, (unsigned)gy),
                               dim3(64 * dwconv::kLkWaves), lds, st, static_cast<const bf16_t *>(in),
                               static_cast<const bf16_t *>(f), static_cast<bf16_t *>(out), tg);
            return launch_status();
        } else {
            const size_t lds = dwconv::longk_tiled_lds_bytes();
            if (lds > kMaxLdsBytes || !allow_large_lds(dwconv::corr_longk_tiled_kernel<T>)) return -1;
            hipLaunchKernelGGL((dwconv::corr_longk_tiled_kernel<T>), dim3((unsigned)s.C, (unsigned)gy),
                               dim3(64 * dwconv::kLkWaves), lds, st, static_cast<const T *>(in), static_cast<const T *>(f),
                               static_cast<T *>(out), tg);
            return launch_status();
        }
    }
    dwconv::LongKGeom g;
    g.B = s.B; g.C = s.C; g.L = s.L; g.K = s.K;
    g.pad = pad_eff; g.reverse = reverse; g.dmin = dmin; g.dmax = dmax;
    g.NB = NB; g.NT = (NB + 15) / 16;
    // rows per workgroup: about 32 (row pair, tile) items for its 16 waves, no more than the batch, and within half of
    // the LDS of a compute unit, so that two workgroups share it and one stages its rows while the other computes
    // (sixteen rows of 1024 positions in one resident workgroup measured slower than two rows in each of two)
    auto lds_for = [&](int R) -> size_t {
        return sizeof(T) == 2 ? dwconv::longk_corr_bf16_lds_bytes(s.K, NB, R) : dwconv::longk_corr_lds_bytes(s.K, NB, R);
    };
    int R = 2 * ((2 * dwconv::kLkWaves + g.NT - 1) / g.NT);
    if (R > 2 * ((s.B + 1) / 2)) R = 2 * ((s.B + 1) / 2);
    while (R > 2 && lds_for(R) > kMaxLdsBytes / 2) R -= 2;
    g.R = R;
    const long long row_groups = ((long long)s.B + R - 1) / R;
    if (row_groups > 65535) return -1;
    if constexpr (sizeof(T) == 2) {
        // bf16 storage: raw rows and four shifted copies of the filter in LDS, bf16 matrix instruction
        const size_t lds = lds_for(R);
        if (lds > kMaxLdsBytes) return -1;
        if (!allow_large_lds(dwconv::corr_longk_bf16_kernel<>)) return -1;
        hipLaunchKernelGGL(dwconv::corr_longk_bf16_kernel<>, dim3((unsigned)s.C, (unsigned)row_groups),
                           dim3(64 * dwconv::kLkWaves), lds, st, static_cast<const bf16_t *>(in),
                           static_cast<const bf16_t *>(f), static_cast<bf16_t *>(out), g);
    } else {
        const size_t lds = lds_for(R);
        if (lds > kMaxLdsBytes) return -1;
        if (!allow_large_lds(dwconv::corr_longk_kernel<T>)) return -1;
        hipLaunchKernelGGL((dwconv::corr_longk_kernel<T>), dim3((unsigned)s.C, (unsigned)row_groups),
                           dim3(64 * dwconv::kLkWaves), lds, st, static_cast<const T *>(in), static_cast<const T *>(f),
                           static_cast<T *>(out), g);
    }
    return launch_status();
}

template <typename T>
int launch_corr(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st)
{
    int rc = launch_corr_mfma<T>(in, f, out, s, pad_eff, reverse, st);
    if (rc >= 0) return rc;
    rc = launch_corr_longk<T>(in, f, out, s, pad_eff, reverse, st);
    if (rc >= 0) return rc;
    return launch_corr_valu<T>(in, f, out, s, pad_eff, reverse, st);
}

}  // namespace dwhost
