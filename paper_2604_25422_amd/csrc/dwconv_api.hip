// C ABI of the gfx950 depthwise 1-D convolution library: argument validation,
// kernel selection and launch.  Declarations and argument contracts are in
// include/dwconv.h; the operator is the one of the paper's Sec. IV-A.
#include "../../include/dwconv.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <array>
#include <map>
#include <memory>
#include <mutex>
#include <vector>
#include <type_traits>

#include "dwconv_bwd_fused.hip.h"
#include "dwconv_bwd_fused_bf16.hip.h"
#include "dwconv_common.hip.h"
#include "dwconv_dw_bf16.hip.h"
#include "dwconv_dw_direct.hip.h"
#include "dwconv_longk.hip.h"
#include "dwconv_mfma.hip.h"
#include "dwconv_rowbatch.hip.h"
#include "dwconv_valu.hip.h"

namespace {

using dwconv::bf16_t;

constexpr int kVersion = 100;   // 0.1.0

struct Shape {
    int B, C, L, K, pad, dtype;
};

int check_shape(int B, int C, int L, int K, int pad, int dtype)
{
    if (B < 1 || C < 1 || L < 1 || K < 1) return DWCONV_ERR_SHAPE;
    const unsigned long long n = (unsigned long long)B * (unsigned long long)C;
    if (n > (1ull << 40) || n * (unsigned long long)L > (1ull << 40)) return DWCONV_ERR_SHAPE;
    if ((unsigned long long)C * (unsigned long long)K > (1ull << 40)) return DWCONV_ERR_SHAPE;
    if (pad < 0 || pad > K - 1) return DWCONV_ERR_PAD;
    if (dtype != DWCONV_F32 && dtype != DWCONV_BF16) return DWCONV_ERR_DTYPE;
    return DWCONV_OK;
}

bool aligned_to(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
size_t elem_size(int dtype) { return dtype == DWCONV_F32 ? 4 : 2; }

int launch_status()
{
    return hipGetLastError() == hipSuccess ? DWCONV_OK : DWCONV_ERR_LAUNCH;
}

// ------------------------------------------------------------------ forward / input gradient
// out = correlate(in, f_eff, pad_eff): the forward is (x, w, pad); the input gradient is
// (dy, reversed w, K-1-pad).

// Block offsets d of the 16-blocked Toeplitz form that can hold a tap: d in [dmin, dmax].
int toeplitz_dmin(int pad) { return -((pad + 15) / 16); }
int toeplitz_dmax(int K, int pad) { return (K - pad + 14) / 16; }

constexpr int kMfmaMinK = 3;      // shorter filters stay on the vector ALU
constexpr int kMfmaMaxND = 6;          // fused backward, bf16, short rows
constexpr int kMfmaMaxNDWide = 10;     // fp32 forward / input gradient / weight gradient on long rows (K up to 130)
int mfma_max_nd(int dtype) { return dtype == DWCONV_F32 ? kMfmaMaxNDWide : kMfmaMaxND; }
constexpr int kComputeUnits = 256;     // MI355X
constexpr int kMfmaMaxL = 1 << 27;      // byte offsets inside a row stay below the out-of-row marker of the buffer loads

// Short rows (see dwconv::RowsMap): whether the matrix-core kernels should walk the virtual row of a channel, and
// its geometry.  Depends on the shape only; the gap is the same for the forward and the input-gradient pads.
struct RowsPlan {
    bool on;
    bool batch;             // rows of at most 128 positions: sixteen rows of a channel per matrix tile instead
    int units;              // batch: groups of sixteen rows per channel
    int nvs;                // 1024-position segments of the virtual row
    dwconv::RowsMap map;
};
RowsPlan plan_rows(const Shape &s)
{
    RowsPlan r;
    r.on = false; r.batch = false; r.units = 0; r.nvs = 0;
    r.map = dwconv::RowsMap{0, 0, 0, 0, 0u, 0u};
    const int nd = toeplitz_dmax(s.K, s.pad) - toeplitz_dmin(s.pad) + 1;
    if (s.K < kMfmaMinK || nd < 2 || nd > kMfmaMaxND || (s.L % 4) != 0) return r;
    const long long es = (long long)elem_size(s.dtype);
    const long long halo = s.pad > s.K - 1 - s.pad ? s.pad : s.K - 1 - s.pad;
    const long long P = s.L + (halo + 3) / 4 * 4;
    const long long padded = ((long long)s.L + dwconv::kSegLen - 1) / dwconv::kSegLen * dwconv::kSegLen;
    if (4 * padded <= 5 * P) return r;                       // ordinary segments waste less than a quarter
    // sixteen rows per tile (either storage type): byte offsets inside a unit stay below the out-of-row marker
    const bool batch = s.L <= dwconv::kRbMaxL && (long long)dwconv::kRbRows * s.C * s.L * es < (1ll << 30);
    const long long elems = (long long)s.B * s.C * s.L;
    if (elems * es > (1ll << 30) || (long long)s.B * P * P >= (1ll << 32) || (long long)s.B * P >= (1ll << 31)) {
        // too large for virtual rows (32-bit positions); the sixteen-row kernels have no such limit
        if (batch) {
            r.on = true; r.batch = true;
            r.units = (s.B + dwconv::kRbRows - 1) / dwconv::kRbRows;
        }
        return r;
    }
    r.on = true;
    r.nvs = (int)(((long long)s.B * P + dwconv::kSegLen - 1) / dwconv::kSegLen);
    r.map.P = (int)P; r.map.L = s.L; r.map.CL = s.C * s.L; r.map.Lv = (int)(s.B * P);
    r.map.M = (unsigned)((1ull << 32) / (unsigned long long)P) + 1u;
    r.map.bytes = (unsigned)(elems * es);
    if (batch) {
        r.batch = true;
        r.units = (s.B + dwconv::kRbRows - 1) / dwconv::kRbRows;
    }
    return r;
}

template <typename T>
int launch_corr_valu(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st)
{
    constexpr int R = 4, THREADS = 256, KCH = 512;
    constexpr int TILE = R * THREADS;
    const long long tiles_per_row = ((long long)s.L + TILE - 1) / TILE;
    const long long blocks = (long long)s.B * s.C * tiles_per_row;
    if (blocks > 0x7fffffffLL) return DWCONV_ERR_SHAPE;
    hipLaunchKernelGGL((dwconv::corr_valu_kernel<T, R, THREADS, KCH>), dim3((unsigned)blocks), dim3(THREADS), 0, st,
                       static_cast<const T *>(in), static_cast<const T *>(f), static_cast<T *>(out), s.C, s.L, s.K,
                       pad_eff, reverse, (int)tiles_per_row);
    return launch_status();
}

constexpr long long kTargetWaves = 4096;   // 256 CUs x 16 resident waves (weight-gradient plan; shape-only)

// Waves of `kernel` that are resident on the current device at once (one full round), from the
// occupancy the runtime reports; falls back to kTargetWaves if the query fails.
template <typename Kernel>
long long resident_waves(Kernel kernel, int block_threads)
{
    static std::mutex mu;
    static std::map<std::pair<int, const void *>, long long> cache;      // (device, kernel) -> waves
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return kTargetWaves;
    }
    const std::pair<int, const void *> key(dev, reinterpret_cast<const void *>(kernel));
    std::lock_guard<std::mutex> lock(mu);
    auto it = cache.find(key);
    if (it != cache.end()) return it->second;
    int cus = 0, blocks_per_cu = 0;
    long long waves = kTargetWaves;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks_per_cu, kernel, block_threads, 0) == hipSuccess &&
        cus >= 1 && blocks_per_cu >= 1)
        waves = (long long)cus * blocks_per_cu * (block_threads / 64);
    else
        (void)hipGetLastError();
    cache[key] = waves;
    return waves;
}

// Wave slots of a correlate launch: one resident round, but no more than 16 waves per compute unit.  Kernels
// light enough for five or six waves per SIMD measured slower with the larger round (short filter, K = 7:
// 105 us with 5120 slots, 97.6 us with 4096).
template <typename Kernel>
long long corr_wave_slots(Kernel kernel, int block_threads)
{
    const long long r = resident_waves(kernel, block_threads);
    return r < kTargetWaves ? r : kTargetWaves;
}

// Returns -1 when the shape or the pointers do not fit the matrix-core kernel.
template <typename T>
int launch_corr_mfma(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st)
{
    const int dmin = toeplitz_dmin(pad_eff), dmax = toeplitz_dmax(s.K, pad_eff);
    const int nd = dmax - dmin + 1;
    if (s.K < kMfmaMinK || nd < 2 || nd > mfma_max_nd(s.dtype) || (s.L % 4) != 0 || s.L > kMfmaMaxL) return -1;
    if (!aligned_to(in, 4 * sizeof(T)) || !aligned_to(out, 4 * sizeof(T))) return -1;
    const long long rows = (long long)s.B * s.C;
    const long long segs_per_row = (s.L + dwconv::kSegLen - 1) / dwconv::kSegLen;
    const long long total_segs = rows * segs_per_row;
    if (total_segs > 0x3fffffffLL) return -1;           // the kernel's segment walk is 32-bit
    dwconv::CorrGeom g;
    g.C = s.C; g.L = s.L; g.K = s.K; g.rows = (int)rows;
    g.pad = pad_eff; g.reverse = reverse; g.dmin = dmin;
    g.segs_per_row = (int)segs_per_row;
    constexpr int kThreads = 64 * dwconv::kCorrWavesPerBlock;
    const dwconv::RowsMap no_rows{0, 0, 0, 0, 0u, 0u};
    // One resident round of waves, each walking segments wave, wave + n_waves, ...
    auto launch = [&](auto kernel, auto *pi, auto *pf, auto *po) -> int {
        const long long resident = corr_wave_slots(kernel, kThreads);
        long long spw = (total_segs + resident - 1) / resident;      // segments per wave, rounded up
        if (spw < 1) spw = 1;
        long long waves = (total_segs + spw - 1) / spw;
        // A whole number of batch entries per round where one fits: the stride of the walk is then a multiple of
        // C rows, a wave stays on one channel and loads its Toeplitz operands once.
        const long long per_b = (long long)s.C * segs_per_row;
        if (per_b <= resident) {
            long long J = resident / per_b;
            if (J > s.B) J = s.B;
            const long long rounds = (s.B + J - 1) / J;
            J = (s.B + rounds - 1) / rounds;                           // same number of rounds, evened out
            waves = J * per_b;
        }
        const long long blocks = (waves + dwconv::kCorrWavesPerBlock - 1) / dwconv::kCorrWavesPerBlock;
        g.n_waves = (int)waves;
        g.step_rows = g.n_waves / g.segs_per_row;
        g.step_seg = g.n_waves % g.segs_per_row;
        g.step_c = g.step_rows % s.C;
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, pi, pf, po, g, no_rows);
        return launch_status();
    };
    const RowsPlan rp = plan_rows(s);
    if (rp.batch) {
        // rows of at most 128 positions: sixteen rows of a channel (or of two neighbouring channels) per unit
        dwconv::RowBatchGeom rg;
        rg.B = s.B; rg.C = s.C; rg.L = s.L; rg.K = s.K;
        rg.pad = pad_eff; rg.reverse = reverse; rg.dmin = dmin;
        rg.m = (s.L + 15) / 16;
        rg.n_units = rp.units;
        // two channels per wave where that makes whole cache lines of rows that are not, or at least longer pieces;
        // rows of at most 48 positions and at most five block offsets (register budget of the kernel)
        const int nc = (s.C % 2 == 0 && (s.L * (int)sizeof(T)) % 128 != 0 && s.L <= 48 && nd <= 5) ? 2 : 1;
        auto launch_batch = [&](auto kernel) -> int {
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
        };
        if (nc == 2) {
            switch (nd) {
            case 2: return launch_batch(dwconv::corr_rowbatch_kernel<T, 2, 2, 3>);
            case 3: return launch_batch(dwconv::corr_rowbatch_kernel<T, 3, 2, 3>);
            case 4: return launch_batch(dwconv::corr_rowbatch_kernel<T, 4, 2, 3>);
            case 5: return launch_batch(dwconv::corr_rowbatch_kernel<T, 5, 2, 3>);
            default: return -1;
            }
        }
        if (rg.m <= 4) {
            switch (nd) {
            case 2: return launch_batch(dwconv::corr_rowbatch_kernel<T, 2, 1, 4>);
            case 3: return launch_batch(dwconv::corr_rowbatch_kernel<T, 3, 1, 4>);
            case 4: return launch_batch(dwconv::corr_rowbatch_kernel<T, 4, 1, 4>);
            case 5: return launch_batch(dwconv::corr_rowbatch_kernel<T, 5, 1, 4>);
            case 6: return launch_batch(dwconv::corr_rowbatch_kernel<T, 6, 1, 4>);
            default: return -1;
            }
        }
        switch (nd) {                              // rows of five to eight blocks
        case 2: return launch_batch(dwconv::corr_rowbatch_kernel<T, 2, 1, 8>);
        case 3: return launch_batch(dwconv::corr_rowbatch_kernel<T, 3, 1, 8>);
        case 4: return launch_batch(dwconv::corr_rowbatch_kernel<T, 4, 1, 8>);
        case 5: return launch_batch(dwconv::corr_rowbatch_kernel<T, 5, 1, 8>);
        case 6: return launch_batch(dwconv::corr_rowbatch_kernel<T, 6, 1, 8>);
        default: return -1;
        }
    }
    {
        // longer short rows: segments of the virtual row of a channel, slots ordered (virtual segment, channel)
        if (rp.on) {
            const long long total = (long long)rp.nvs * s.C;
            if (total > 0x3fffffffLL) return -1;
            g.rows = rp.nvs;
            g.segs_per_row = s.C;
            auto launch_rows = [&](auto kernel) -> int {
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
                hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, static_cast<const T *>(in),
                                   static_cast<const T *>(f), static_cast<T *>(out), g, rp.map);
                return launch_status();
            };
            switch (nd) {
            case 2: return launch_rows(dwconv::corr_mfma_kernel<T, 2, true>);
            case 3: return launch_rows(dwconv::corr_mfma_kernel<T, 3, true>);
            case 4: return launch_rows(dwconv::corr_mfma_kernel<T, 4, true>);
            case 5: return launch_rows(dwconv::corr_mfma_kernel<T, 5, true>);
            case 6: return launch_rows(dwconv::corr_mfma_kernel<T, 6, true>);
            default: return -1;
            }
        }
    }
    if constexpr (sizeof(T) == 2) {
        // bf16 storage: the bf16 matrix instruction when 16-byte granules of 8 elements line up
        if ((s.L % 8) == 0 && aligned_to(in, 16) && aligned_to(out, 16)) {
            const bf16_t *pi = static_cast<const bf16_t *>(in), *pf = static_cast<const bf16_t *>(f);
            bf16_t *po = static_cast<bf16_t *>(out);
            switch (nd) {
            case 2: return launch(dwconv::corr_mfma_bf16_kernel<2>, pi, pf, po);
            case 3: return launch(dwconv::corr_mfma_bf16_kernel<3>, pi, pf, po);
            case 4: return launch(dwconv::corr_mfma_bf16_kernel<4>, pi, pf, po);
            case 5: return launch(dwconv::corr_mfma_bf16_kernel<5>, pi, pf, po);
            case 6: return launch(dwconv::corr_mfma_bf16_kernel<6>, pi, pf, po);
            default: return -1;
            }
        }
    }
    const T *pi = static_cast<const T *>(in), *pf = static_cast<const T *>(f);
    T *po = static_cast<T *>(out);
    switch (nd) {
    case 2: return launch(dwconv::corr_mfma_kernel<T, 2, false>, pi, pf, po);
    case 3: return launch(dwconv::corr_mfma_kernel<T, 3, false>, pi, pf, po);
    case 4: return launch(dwconv::corr_mfma_kernel<T, 4, false>, pi, pf, po);
    case 5: return launch(dwconv::corr_mfma_kernel<T, 5, false>, pi, pf, po);
    case 6: return launch(dwconv::corr_mfma_kernel<T, 6, false>, pi, pf, po);
    default: break;
    }
    if constexpr (std::is_same<T, float>::value) {
        switch (nd) {
        case 7: return launch(dwconv::corr_mfma_kernel<float, 7, false>, pi, pf, po);
        case 8: return launch(dwconv::corr_mfma_kernel<float, 8, false>, pi, pf, po);
        case 9: return launch(dwconv::corr_mfma_kernel<float, 9, false>, pi, pf, po);
        case 10: return launch(dwconv::corr_mfma_kernel<float, 10, false>, pi, pf, po);
        default: break;
        }
    }
    return -1;
}

constexpr size_t kMaxLdsBytes = 160 * 1024;

// Lets `kernel` use more than the default 64 KiB of dynamic LDS (once per kernel and process).
template <typename Kernel>
bool allow_large_lds(Kernel kernel)
{
    static std::mutex mu;
    static std::map<const void *, bool> done;
    std::lock_guard<std::mutex> lock(mu);
    const void *key = reinterpret_cast<const void *>(kernel);
    auto it = done.find(key);
    if (it != done.end()) return it->second;
    const bool ok = hipFuncSetAttribute(key, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxLdsBytes) == hipSuccess;
    if (!ok) (void)hipGetLastError();
    done[key] = ok;
    return ok;
}

// Filters too long for the register-resident Toeplitz form: whole rows and the whole filter in LDS.
// Returns -1 when the shape or the pointers do not fit.
template <typename T>
int launch_corr_longk(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st)
{
    const int dmin = toeplitz_dmin(pad_eff), dmax = toeplitz_dmax(s.K, pad_eff);
    if (dmax - dmin + 1 <= mfma_max_nd(s.dtype) || s.K > dwconv::kLkMaxK || (s.L % 4) != 0) return -1;
    const int NB = (s.L + 15) / 16;
    if (NB > dwconv::kLkMaxBlocks) return -1;
    if (!aligned_to(in, 4 * sizeof(T)) || !aligned_to(out, 4 * sizeof(T))) return -1;
    const size_t lds = dwconv::longk_corr_lds_bytes(s.K, NB);
    const long long row_groups = ((long long)s.B + dwconv::kLkRows - 1) / dwconv::kLkRows;
    if (lds > kMaxLdsBytes || row_groups > 65535) return -1;
    if (!allow_large_lds(dwconv::corr_longk_kernel<T>)) return -1;
    dwconv::LongKGeom g;
    g.B = s.B; g.C = s.C; g.L = s.L; g.K = s.K;
    g.pad = pad_eff; g.reverse = reverse; g.dmin = dmin; g.dmax = dmax;
    g.NB = NB; g.NT = (NB + 15) / 16;
    hipLaunchKernelGGL((dwconv::corr_longk_kernel<T>), dim3((unsigned)s.C, (unsigned)row_groups),
                       dim3(64 * dwconv::kLkWaves), lds, st, static_cast<const T *>(in), static_cast<const T *>(f),
                       static_cast<T *>(out), g);
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

int corr_entry(const void *in, const void *f, void *out, int B, int C, int L, int K, int pad, int dtype, void *stream,
               bool is_dx)
{
    if (!in || !f || !out) return DWCONV_ERR_NULL;
    const int rc = check_shape(B, C, L, K, pad, dtype);
    if (rc != DWCONV_OK) return rc;
    const size_t es = elem_size(dtype);
    if (!aligned_to(in, es) || !aligned_to(f, es) || !aligned_to(out, es)) return DWCONV_ERR_ALIGN;
    const Shape s{B, C, L, K, pad, dtype};
    const int pad_eff = is_dx ? (K - 1 - pad) : pad;
    const int reverse = is_dx ? 1 : 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == DWCONV_F32) return launch_corr<float>(in, f, out, s, pad_eff, reverse, st);
    return launch_corr<bf16_t>(in, f, out, s, pad_eff, reverse, st);
}

// ------------------------------------------------------------------ weight gradient
enum DwKernel { DW_VALU_K8, DW_VALU_K32, DW_VALU_K64, DW_VALU_K256 };

struct DwPlan {
    DwKernel kernel;
    bool longk;            // shape fits the long-filter matrix-core kernel (two zero-filled slices)
    int lk_wgs, lk_gd;     // its workgroups per channel, largest group of offsets (accumulators per group)
    std::shared_ptr<const dwconv::LongKDwTable> lk_table;   // which offsets every wave slot owns
    int S;                 // partial slices per coefficient
    RowsPlan rows;         // short rows: stage 1 walks the virtual row of a channel
    int wpb;               // waves per block of the matrix-core stage-1 kernels
    int dw_nc;             // short rows, sixteen-row units: channels per block of the stage-1 kernel (1 or 2)
    int S_fused;           // slices the fused backward call writes (differs from S for rows of at most 48 positions)
    bool single;           // S == 1 with one block per channel: stage 1 may write the gradient itself
    int tiles_per_row;     // segments the matrix-core kernels walk per row (per virtual row for short rows)
    int valu_tiles_per_row, valu_items_per_slice;   // the same bookkeeping for the generic kernel (always real rows)
    int segs_per_wave;     // (b, segment) items a wave of the matrix-core kernels walks
    int items_per_slice;   // (b, segment) items each slice owns = wpb * segs_per_wave
};

constexpr int kDwTT = dwconv::kSegLen;   // positions per staged tile (every stage-1 kernel)
constexpr int kDwThreads = 256;

// Long filters: the assignment of block offsets to wave slots (dwconv::LongKDwTable), balanced by work.
// Work of an offset d = the 64-position chunks in which it reaches the row; a group of n offsets runs n matrix
// instructions over the union of its offsets' chunks.  Groups are cut greedily under a cap on size (9) and on
// work; the cap is searched so that at most two groups per slot suffice and the busiest slot is as light as
// possible; groups go to slots heaviest first, each to the least loaded slot that still has room.  The result
// depends on (L, K, pad, slots) only and is cached.
std::shared_ptr<const dwconv::LongKDwTable> longk_dw_table(const Shape &s, int wgs, int *max_group)
{
    struct Entry { std::shared_ptr<const dwconv::LongKDwTable> table; int max_group; };
    static std::mutex mu;
    static std::map<std::array<int, 4>, Entry> cache;
    const std::array<int, 4> key = {s.L, s.K, s.pad, wgs};
    std::lock_guard<std::mutex> lock(mu);
    auto it = cache.find(key);
    if (it != cache.end()) { *max_group = it->second.max_group; return it->second.table; }

    const int dmin = toeplitz_dmin(s.pad), dmax = toeplitz_dmax(s.K, s.pad);
    const int NCH = (s.L + 63) / 64;
    const int nslots = wgs * dwconv::kLkWaves;
    auto fdiv = [](int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); };
    auto ch_lo = [&](int d) { const int v = -fdiv(63 + 16 * d, 64); return v > 0 ? v : 0; };      // ceil((-63 - 16 d) / 64)
    auto ch_hi = [&](int d) { const int v = fdiv(s.L - 1 - 16 * d, 64); return v < NCH - 1 ? v : NCH - 1; };
    auto group_work = [&](int a, int n) {           // n offsets a .. a + n - 1
        const int c = ch_hi(a) - ch_lo(a + n - 1) + 1;
        return (long long)n * (c > 0 ? c : 0);
    };
    long long exact = 0;
    for (int d = dmin; d <= dmax; ++d) exact += group_work(d, 1);
    struct Group { int a, n; long long w; };
    std::vector<Group> best_groups;
    std::vector<int> best_slot;
    long long best_max = -1;
    for (int pct = 40; pct <= 400; pct += 4) {
        const long long cap = exact * pct / (100LL * nslots) + 1;
        std::vector<Group> groups;
        for (int d = dmin; d <= dmax;) {
            int n = 1;
            while (d + n <= dmax && n < dwconv::kLkDwMaxGD && group_work(d, n + 1) <= cap) ++n;
            groups.push_back({d, n, group_work(d, n)});
            d += n;
        }
        if ((int)groups.size() > 2 * nslots || (int)groups.size() > dwconv::kLkDwMaxGroups) continue;
        std::vector<int> order(groups.size());
        for (size_t i = 0; i < order.size(); ++i) order[i] = (int)i;
        std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return groups[x].w > groups[y].w; });
        std::vector<long long> load(nslots, 0);
        std::vector<int> count(nslots, 0), slot_of(groups.size(), 0);
        for (int gi : order) {
            int pick = -1;
            for (int j = 0; j < nslots; ++j)
                if (count[j] < 2 && (pick < 0 || load[j] < load[pick])) pick = j;
            load[pick] += groups[gi].w;
            ++count[pick];
            slot_of[gi] = pick;
        }
        const long long mx = *std::max_element(load.begin(), load.end());
        if (best_max < 0 || mx < best_max) { best_max = mx; best_groups = groups; best_slot = slot_of; }
    }
    if (best_max < 0 || nslots > dwconv::kLkDwMaxSlots) {        // no assignment with two groups per slot
        cache[key] = Entry{nullptr, 0};
        *max_group = 0;
        return nullptr;
    }
    auto table = std::make_shared<dwconv::LongKDwTable>();
    for (int i = 0; i < dwconv::kLkDwMaxGroups; ++i) { table->da[i] = 0; table->n[i] = 0; }
    for (int j = 0; j < dwconv::kLkDwMaxSlots; ++j) table->g0[j] = table->g1[j] = dwconv::kLkDwNoGroup;
    int mg = 1;
    for (size_t i = 0; i < best_groups.size(); ++i) {
        table->da[i] = (short)best_groups[i].a;
        table->n[i] = (unsigned char)best_groups[i].n;
        if (best_groups[i].n > mg) mg = best_groups[i].n;
        const int j = best_slot[i];
        if (table->g0[j] == dwconv::kLkDwNoGroup) table->g0[j] = (unsigned char)i;
        else table->g1[j] = (unsigned char)i;
    }
    static const int kGd[] = {1, 2, 3, 4, 6, 9};
    int gd = 9;
    for (int v : kGd)
        if (v >= mg) { gd = v; break; }
    cache[key] = Entry{table, gd};
    *max_group = gd;
    return table;
}

// Depends on the shape only, so stage 1, stage 2 and the workspace query always agree.
DwPlan plan_dw(const Shape &s)
{
    DwPlan p;
    p.kernel = s.K <= 8 ? DW_VALU_K8 : s.K <= 32 ? DW_VALU_K32 : s.K <= 64 ? DW_VALU_K64 : DW_VALU_K256;
    p.rows = plan_rows(s);
    long long tiles = p.rows.on ? p.rows.nvs : ((long long)s.L + kDwTT - 1) / kDwTT;
    if (p.rows.batch) {                                          // units of the weight-gradient kernel, one channel per block
        const int ru = dwconv::rb_dw_unit_rows(s.L, 1);
        tiles = (s.B + ru - 1) / ru;
    }
    long long items = p.rows.on ? tiles : (long long)s.B * tiles;                        // per channel
    const int nd = toeplitz_dmax(s.K, s.pad) - toeplitz_dmin(s.pad) + 1;
    const bool mfma_shape = s.K >= kMfmaMinK && nd >= 2 && nd <= mfma_max_nd(s.dtype) && (s.L % 4) == 0 && s.L <= kMfmaMaxL;
    // When the channels alone fill the chip evenly (C = 1, 2 or 3 per compute unit), one block of 16, 8 or 5
    // waves takes a whole channel: no slices, no second stage.
    p.wpb = dwconv::kWavesPerBlock;
    p.single = false;
    p.dw_nc = 1;
    if (mfma_shape && s.C % kComputeUnits == 0 && s.C / kComputeUnits <= 3) {
        const int wpb = 16 / (s.C / kComputeUnits);
        // (sixteen-row units of rows longer than 48 positions need more LDS than sixteen waves have)
        const bool fits = (!p.rows.batch || dwconv::rb_dw_lds_bytes(s.L, nd, wpb, 1) <= kMaxLdsBytes) &&
                          (nd <= kMfmaMaxND || dwconv::dw_direct_lds_bytes(nd, wpb) <= kMaxLdsBytes);
        if (items >= 2 * wpb && fits) { p.wpb = wpb; p.single = true; }
    }
    long long groups = s.C;                                      // blocks along the channel axis
    if (p.rows.batch && !p.single && s.C % 2 == 0 && (s.L * (int)elem_size(s.dtype)) % 128 != 0 && s.L <= 48) {
        // two neighbouring channels per block: rows that are not whole cache lines become pieces that are;
        // a unit is then eight rows of both channels
        p.dw_nc = 2;
        groups = s.C / 2;
        tiles = (s.B + dwconv::kRbRows / 2 - 1) / (dwconv::kRbRows / 2);
        items = tiles;
    }
    long long want = (kTargetWaves / p.wpb + groups - 1) / groups;   // blocks per channel (group)
    if (p.single) want = 1;
    if (want < 1) want = 1;
    if (want > 65535) want = 65535;
    long long spw = (items + want * p.wpb - 1) / (want * p.wpb);
    if (spw < 1) spw = 1;
    const long long per = spw * p.wpb;
    p.segs_per_wave = (int)spw;
    p.items_per_slice = (int)per;
    p.S = (int)((items + per - 1) / per);
    // the fused backward kernel of these shapes works on one channel per block: its own slice count
    p.S_fused = p.S;
    if (p.rows.batch && s.L <= dwconv::kRbBwdMaxL) {
        // one wave per (channel, slice), sixteen-row units: about kTargetWaves waves
        long long wantf = kTargetWaves / s.C;
        if (wantf < 1) wantf = 1;
        if (wantf > p.rows.units) wantf = p.rows.units;
        if (wantf > 65535) wantf = 65535;
        const long long upw = (p.rows.units + wantf - 1) / wantf;
        p.S_fused = (int)((p.rows.units + upw - 1) / upw);
    }
    p.tiles_per_row = (int)tiles;
    {
        const long long real_tiles = ((long long)s.L + kDwTT - 1) / kDwTT;
        const long long real_items = (long long)s.B * real_tiles;
        p.valu_tiles_per_row = (int)real_tiles;
        p.valu_items_per_slice = (int)((real_items + p.S - 1) / p.S);
    }
    // long filters: offsets are split over waves instead, partials land in exactly two slices
    p.longk = false;
    p.lk_wgs = p.lk_gd = 0;
    const int NCH = (s.L + 63) / 64;
    if (nd > mfma_max_nd(s.dtype) && s.K <= dwconv::kLkMaxK && (s.L % 4) == 0 && (s.L + 15) / 16 <= dwconv::kLkMaxBlocks &&
        dwconv::longk_dw_lds_bytes(s.L, NCH) <= kMaxLdsBytes) {
        const int per_wg = 2 * dwconv::kLkWaves * dwconv::kLkDwMaxGD;
        p.lk_wgs = (nd + per_wg - 1) / per_wg;
        p.lk_table = longk_dw_table(s, p.lk_wgs, &p.lk_gd);
    }
    if (p.lk_table) {
        p.longk = true;
        p.S = 2;
        p.items_per_slice = (int)((items + 1) / 2);        // the generic kernel, if it has to run, uses two slices too
        p.valu_items_per_slice = p.items_per_slice;
    }
    return p;
}

size_t dw_workspace_bytes(const Shape &s, const DwPlan &p)
{
    const size_t bytes = (size_t)(p.S > p.S_fused ? p.S : p.S_fused) * (size_t)s.C * (size_t)s.K * sizeof(float);
    return (bytes + 255) & ~(size_t)255;
}

int check_dw_shape(int B, int C, int L, int K, int pad, int dtype)
{
    const int rc = check_shape(B, C, L, K, pad, dtype);
    if (rc != DWCONV_OK) return rc;
    // the slice bookkeeping of stage 1 is 32-bit
    const long long tiles = ((long long)L + kDwTT - 1) / kDwTT;
    if ((long long)B * tiles > 0x3fffffffLL || C > 0x7fffffff / 2) return DWCONV_ERR_SHAPE;
    return DWCONV_OK;
}

template <typename T, int KCH>
void launch_dw_partial_valu(const void *x, const void *dy, float *part, const Shape &s, const DwPlan &p, hipStream_t st)
{
    hipLaunchKernelGGL((dwconv::dw_partial_valu_kernel<T, kDwThreads, kDwTT, KCH>), dim3((unsigned)s.C, (unsigned)p.S),
                       dim3(kDwThreads), 0, st, static_cast<const T *>(x), static_cast<const T *>(dy), part, s.B, s.C,
                       s.L, s.K, s.pad, p.valu_tiles_per_row, p.valu_items_per_slice);
}

// One stage-1 launch on the matrix cores.  dw_out != nullptr only for single-slice plans.
template <typename T, int ND, int W>
int launch_dw_partial_mfma_ndw(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                               int dmin, hipStream_t st)
{
    if (p.rows.batch) {
        // rows of at most 128 positions, either storage type: sixteen rows per matrix tile
        auto launch_rb = [&](auto kernel, int nc) -> int {
            const size_t lds_rb = dwconv::rb_dw_lds_bytes(s.L, ND, W, nc);
            if (lds_rb > kMaxLdsBytes) return -1;
            if (lds_rb > 64 * 1024 && !allow_large_lds(kernel)) return -1;
            hipLaunchKernelGGL(kernel, dim3((unsigned)(s.C / nc), (unsigned)p.S), dim3(64 * W), lds_rb, st,
                               static_cast<const T *>(x), static_cast<const T *>(dy), part, static_cast<T *>(dw_out), s.B,
                               s.C, s.L, s.K, s.pad, dmin, ND, p.tiles_per_row);
            return launch_status();
        };
        // (the kernel is compiled per number of 16-blocks of a row, not per number of block offsets)
        const int m = (s.L + 15) / 16;
        if constexpr (W == dwconv::kWavesPerBlock) {
            if (p.dw_nc == 2) {
                switch (m) {
                case 1: return launch_rb(dwconv::dw_rowbatch_kernel<T, 1, W, 2>, 2);
                case 2: return launch_rb(dwconv::dw_rowbatch_kernel<T, 2, W, 2>, 2);
                case 3: return launch_rb(dwconv::dw_rowbatch_kernel<T, 3, W, 2>, 2);
                default: return -1;
                }
            }
        }
        switch (m) {
        case 1: return launch_rb(dwconv::dw_rowbatch_kernel<T, 1, W, 1>, 1);
        case 2: return launch_rb(dwconv::dw_rowbatch_kernel<T, 2, W, 1>, 1);
        case 3: return launch_rb(dwconv::dw_rowbatch_kernel<T, 3, W, 1>, 1);
        case 4: return launch_rb(dwconv::dw_rowbatch_kernel<T, 4, W, 1>, 1);
        case 5: return launch_rb(dwconv::dw_rowbatch_kernel<T, 5, W, 1>, 1);
        case 6: return launch_rb(dwconv::dw_rowbatch_kernel<T, 6, W, 1>, 1);
        case 7: return launch_rb(dwconv::dw_rowbatch_kernel<T, 7, W, 1>, 1);
        case 8: return launch_rb(dwconv::dw_rowbatch_kernel<T, 8, W, 1>, 1);
        default: return -1;
        }
    }
    if constexpr (std::is_same<T, float>::value) {
        // fp32 rows go from memory straight into LDS
        constexpr size_t lds = dwconv::dw_direct_lds_bytes(ND, W);
        static_assert(lds <= kMaxLdsBytes, "LDS budget");
        if (p.rows.on) {
            auto kernel = dwconv::dw_partial_direct_kernel<ND, W, true>;
            if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
            hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                               static_cast<const float *>(x), static_cast<const float *>(dy), part,
                               static_cast<float *>(dw_out), 1, s.C, s.L, s.K, s.pad, dmin, p.tiles_per_row, p.rows.map);
        } else {
            auto kernel = dwconv::dw_partial_direct_kernel<ND, W, false>;
            if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
            hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                               static_cast<const float *>(x), static_cast<const float *>(dy), part,
                               static_cast<float *>(dw_out), s.B, s.C, s.L, s.K, s.pad, dmin, p.tiles_per_row, p.rows.map);
        }
    } else if (p.rows.on) {
        // bf16 short rows (longer than 64 positions): the virtual row of a channel, widened to fp32 through registers
        auto kernel = dwconv::dw_partial_mfma_kernel<T, ND, W, true>;
        constexpr size_t lds = dwconv::dw_mfma_lds_bytes(ND, W);
        static_assert(lds <= kMaxLdsBytes, "LDS budget");
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st, static_cast<const T *>(x),
                           static_cast<const T *>(dy), part, static_cast<T *>(dw_out), 1, s.C, s.L, s.K, s.pad, dmin,
                           p.tiles_per_row, p.rows.map);
    } else if ((s.L % 8) == 0 && aligned_to(x, 16) && aligned_to(dy, 16)) {
        // bf16 rows of whole 16-byte granules: raw rows straight into LDS, bf16 matrix instruction
        auto kernel = dwconv::dw_partial_bf16_kernel<ND, W>;
        constexpr size_t lds = dwconv::dw_bf16_lds_bytes(ND, W);
        static_assert(lds <= kMaxLdsBytes, "LDS budget");
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                           static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(dy), part,
                           static_cast<bf16_t *>(dw_out), s.B, s.C, s.L, s.K, s.pad, dmin, p.tiles_per_row);
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

// fp32, seven to ten block offsets (K up to 130): the LDS-direct kernel on ordinary rows.
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
    switch (p.wpb) {
    case 4: return launch_dw_partial_wide_ndw<ND, 4>(x, dy, part, dw_out, s, p, dmin, st);
    case 5: return launch_dw_partial_wide_ndw<ND, 5>(x, dy, part, dw_out, s, p, dmin, st);
    case 8: return launch_dw_partial_wide_ndw<ND, 8>(x, dy, part, dw_out, s, p, dmin, st);
    case 16: return launch_dw_partial_wide_ndw<ND, 16>(x, dy, part, dw_out, s, p, dmin, st);
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
    if (s.K < kMfmaMinK || nd < 2 || nd > mfma_max_nd(s.dtype) || (s.L % 4) != 0 || s.L > kMfmaMaxL) return -1;
    if (!aligned_to(x, 4 * sizeof(T)) || !aligned_to(dy, 4 * sizeof(T))) return -1;
    if constexpr (std::is_same<T, float>::value) {
        switch (nd) {
        case 7: return launch_dw_partial_wide_nd<7>(x, dy, part, dw_out, s, p, dmin, st);
        case 8: return launch_dw_partial_wide_nd<8>(x, dy, part, dw_out, s, p, dmin, st);
        case 9: return launch_dw_partial_wide_nd<9>(x, dy, part, dw_out, s, p, dmin, st);
        case 10: return launch_dw_partial_wide_nd<10>(x, dy, part, dw_out, s, p, dmin, st);
        default: break;
        }
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
void launch_dw_longk_gd(const void *x, const void *dy, float *part, const Shape &s, const DwPlan &p,
                        const dwconv::LongKDwGeom &g, size_t lds, hipStream_t st)
{
    hipLaunchKernelGGL((dwconv::dw_longk_kernel<T, GD>), dim3((unsigned)s.C, (unsigned)p.lk_wgs),
                       dim3(64 * dwconv::kLkWaves), lds, st, static_cast<const T *>(x), static_cast<const T *>(dy),
                       part, g, *p.lk_table);
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
    const size_t lds = dwconv::longk_dw_lds_bytes(s.L, g.NCH);
    bool ok = true;
    switch (p.lk_gd) {
    case 1: ok = allow_large_lds(dwconv::dw_longk_kernel<T, 1>); break;
    case 2: ok = allow_large_lds(dwconv::dw_longk_kernel<T, 2>); break;
    case 3: ok = allow_large_lds(dwconv::dw_longk_kernel<T, 3>); break;
    case 4: ok = allow_large_lds(dwconv::dw_longk_kernel<T, 4>); break;
    case 6: ok = allow_large_lds(dwconv::dw_longk_kernel<T, 6>); break;
    default: ok = allow_large_lds(dwconv::dw_longk_kernel<T, 9>); break;
    }
    if (!ok) return -1;
    // both slices start at zero: a group stores only the taps it owns
    const size_t n = (size_t)2 * (size_t)s.C * (size_t)s.K;
    size_t fill_blocks = (n + 256 * 8 - 1) / (256 * 8);
    if (fill_blocks > 65536) fill_blocks = 65536;
    hipLaunchKernelGGL(dwconv::fill_zero_kernel, dim3((unsigned)fill_blocks), dim3(256), 0, st, part, n);
    switch (p.lk_gd) {
    case 1: launch_dw_longk_gd<T, 1>(x, dy, part, s, p, g, lds, st); break;
    case 2: launch_dw_longk_gd<T, 2>(x, dy, part, s, p, g, lds, st); break;
    case 3: launch_dw_longk_gd<T, 3>(x, dy, part, s, p, g, lds, st); break;
    case 4: launch_dw_longk_gd<T, 4>(x, dy, part, s, p, g, lds, st); break;
    case 6: launch_dw_longk_gd<T, 6>(x, dy, part, s, p, g, lds, st); break;
    default: launch_dw_longk_gd<T, 9>(x, dy, part, s, p, g, lds, st); break;
    }
    return launch_status();
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

// Fused input + weight gradient (matrix-core shape class).  Returns -1 when it does not apply.
template <int ND, int W>
int launch_bwd_fused_ndw(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out,
                         const Shape &s, const DwPlan &p, int dmin, hipStream_t st)
{
    if (s.dtype == DWCONV_BF16) {
        auto kernel = dwconv::bwd_fused_bf16_kernel<ND, W>;
        constexpr size_t lds = dwconv::bwd_fused_bf16_lds_bytes(ND, W);
        static_assert(lds <= kMaxLdsBytes, "LDS budget");
        if (lds > 64 * 1024 && !allow_large_lds(kernel)) return -1;
        hipLaunchKernelGGL(kernel, dim3((unsigned)s.C, (unsigned)p.S), dim3(64 * W), lds, st,
                           static_cast<const bf16_t *>(dy), static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(w),
                           static_cast<bf16_t *>(dx), part, static_cast<bf16_t *>(dw_out), s.B, s.C, s.L, s.K, s.pad, dmin,
                           p.tiles_per_row);
        return launch_status();
    }
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

template <int ND>
int launch_bwd_fused_nd(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out,
                        const Shape &s, const DwPlan &p, int dmin, hipStream_t st)
{
    switch (p.wpb) {
    case 4: return launch_bwd_fused_ndw<ND, 4>(dy, x, w, dx, part, dw_out, s, p, dmin, st);
    case 5: return launch_bwd_fused_ndw<ND, 5>(dy, x, w, dx, part, dw_out, s, p, dmin, st);
    case 8: return launch_bwd_fused_ndw<ND, 8>(dy, x, w, dx, part, dw_out, s, p, dmin, st);
    case 16: return launch_bwd_fused_ndw<ND, 16>(dy, x, w, dx, part, dw_out, s, p, dmin, st);
    default: return -1;
    }
}

// Rows of at most 48 positions: sixteen rows per tile, one wave per (channel, slice).  Returns -1 when it does not apply.
template <typename T>
int launch_bwd_rowbatch(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out, bool *wrote_dw,
                        const Shape &s, const DwPlan &p, hipStream_t st)
{
    const int dmin = toeplitz_dmin(s.pad), dmax = toeplitz_dmax(s.K, s.pad);
    const int nd = dmax - dmin + 1;
    if (s.L > dwconv::kRbBwdMaxL || nd < 2 || nd > kMfmaMaxND) return -1;
    if (!aligned_to(x, 4 * sizeof(T)) || !aligned_to(dy, 4 * sizeof(T)) || !aligned_to(dx, 4 * sizeof(T))) return -1;
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
    switch (nd) {
    case 2: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 2, 1>, dwconv::bwd_rowbatch_kernel<T, 2, 2>, dwconv::bwd_rowbatch_kernel<T, 2, 3>, 2); break;
    case 3: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 3, 1>, dwconv::bwd_rowbatch_kernel<T, 3, 2>, dwconv::bwd_rowbatch_kernel<T, 3, 3>, 3); break;
    case 4: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 4, 1>, dwconv::bwd_rowbatch_kernel<T, 4, 2>, dwconv::bwd_rowbatch_kernel<T, 4, 3>, 4); break;
    case 5: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 5, 1>, dwconv::bwd_rowbatch_kernel<T, 5, 2>, dwconv::bwd_rowbatch_kernel<T, 5, 3>, 5); break;
    case 6: rc = launch_m(dwconv::bwd_rowbatch_kernel<T, 6, 1>, dwconv::bwd_rowbatch_kernel<T, 6, 2>, dwconv::bwd_rowbatch_kernel<T, 6, 3>, 6); break;
    default: break;
    }
    if (rc == DWCONV_OK && direct_rb) *wrote_dw = true;
    return rc;
}

int launch_bwd_fused(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out, bool *wrote_dw,
                     const Shape &s, const DwPlan &p, hipStream_t st)
{
    *wrote_dw = false;
    if (p.longk) return -1;
    if (p.rows.batch) {
        if (s.dtype == DWCONV_F32) return launch_bwd_rowbatch<float>(dy, x, w, dx, part, dw_out, wrote_dw, s, p, st);
        return launch_bwd_rowbatch<bf16_t>(dy, x, w, dx, part, dw_out, wrote_dw, s, p, st);
    }
    if (s.dtype == DWCONV_BF16 && p.rows.on) return -1;      // bf16 virtual rows: the two separate kernels
    // bf16: whole 16-byte granules of 8 elements
    if (s.dtype == DWCONV_BF16 && (s.L % 8) != 0) return -1;
    const int dmin = toeplitz_dmin(s.pad), dmax = toeplitz_dmax(s.K, s.pad);
    const int nd = dmax - dmin + 1;
    if (s.K < kMfmaMinK || nd < 2 || nd > kMfmaMaxND || (s.L % 4) != 0 || s.L > kMfmaMaxL) return -1;
    if (!aligned_to(x, 16) || !aligned_to(dy, 16) || !aligned_to(dx, 16)) return -1;
    void *direct = (p.single && p.S == 1) ? dw_out : nullptr;
    int rc = -1;
    switch (nd) {
    case 2: rc = launch_bwd_fused_nd<2>(dy, x, w, dx, part, direct, s, p, dmin, st); break;
    case 3: rc = launch_bwd_fused_nd<3>(dy, x, w, dx, part, direct, s, p, dmin, st); break;
    case 4: rc = launch_bwd_fused_nd<4>(dy, x, w, dx, part, direct, s, p, dmin, st); break;
    case 5: rc = launch_bwd_fused_nd<5>(dy, x, w, dx, part, direct, s, p, dmin, st); break;
    case 6: rc = launch_bwd_fused_nd<6>(dy, x, w, dx, part, direct, s, p, dmin, st); break;
    default: break;
    }
    if (rc == DWCONV_OK && direct) *wrote_dw = true;
    return rc;
}

template <typename T>
int launch_dw_finalize(const float *part, void *dw, const Shape &s, const DwPlan &p, hipStream_t st)
{
    const size_t CK = (size_t)s.C * (size_t)s.K;
    const size_t blocks = (CK + 255) / 256;
    if (blocks > 0x7fffffffull) return DWCONV_ERR_SHAPE;
    hipLaunchKernelGGL((dwconv::dw_finalize_kernel<T>), dim3((unsigned)blocks), dim3(256), 0, st, part,
                       static_cast<T *>(dw), p.S, CK);
    return launch_status();
}

int check_workspace(const void *ws, size_t ws_bytes, const Shape &s, const DwPlan &p)
{
    if (!ws || !aligned_to(ws, 16) || ws_bytes < dw_workspace_bytes(s, p)) return DWCONV_ERR_WORKSPACE;
    return DWCONV_OK;
}

}  // namespace

extern "C" {

int dwconv_fwd(const void *x, const void *w, void *y, int B, int C, int L, int K, int pad_left, int dtype, void *stream)
{
    return corr_entry(x, w, y, B, C, L, K, pad_left, dtype, stream, false);
}

int dwconv_bwd_input(const void *dy, const void *w, void *dx, int B, int C, int L, int K, int pad_left, int dtype,
                     void *stream)
{
    return corr_entry(dy, w, dx, B, C, L, K, pad_left, dtype, stream, true);
}

int dwconv_bwd_weight_partial(const void *x, const void *dy, void *workspace, size_t workspace_bytes, int B, int C,
                              int L, int K, int pad_left, int dtype, void *stream)
{
    if (!x || !dy) return DWCONV_ERR_NULL;
    int rc = check_dw_shape(B, C, L, K, pad_left, dtype);
    if (rc != DWCONV_OK) return rc;
    const size_t es = elem_size(dtype);
    if (!aligned_to(x, es) || !aligned_to(dy, es)) return DWCONV_ERR_ALIGN;
    const Shape s{B, C, L, K, pad_left, dtype};
    const DwPlan p = plan_dw(s);
    rc = check_workspace(workspace, workspace_bytes, s, p);
    if (rc != DWCONV_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *part = static_cast<float *>(workspace);
    if (dtype == DWCONV_F32) return launch_dw_partial<float>(x, dy, part, nullptr, nullptr, s, p, st);
    return launch_dw_partial<bf16_t>(x, dy, part, nullptr, nullptr, s, p, st);
}

int dwconv_bwd_weight_finalize(const void *workspace, size_t workspace_bytes, void *dw, int B, int C, int L, int K,
                               int pad_left, int dtype, void *stream)
{
    if (!dw) return DWCONV_ERR_NULL;
    int rc = check_dw_shape(B, C, L, K, pad_left, dtype);
    if (rc != DWCONV_OK) return rc;
    if (!aligned_to(dw, elem_size(dtype))) return DWCONV_ERR_ALIGN;
    const Shape s{B, C, L, K, pad_left, dtype};
    const DwPlan p = plan_dw(s);
    rc = check_workspace(workspace, workspace_bytes, s, p);
    if (rc != DWCONV_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float *part = static_cast<const float *>(workspace);
    if (dtype == DWCONV_F32) return launch_dw_finalize<float>(part, dw, s, p, st);
    return launch_dw_finalize<bf16_t>(part, dw, s, p, st);
}

int dwconv_bwd_weight(const void *x, const void *dy, void *dw, void *workspace, size_t workspace_bytes, int B, int C,
                      int L, int K, int pad_left, int dtype, void *stream)
{
    if (!x || !dy || !dw) return DWCONV_ERR_NULL;
    int rc = check_dw_shape(B, C, L, K, pad_left, dtype);
    if (rc != DWCONV_OK) return rc;
    const size_t es = elem_size(dtype);
    if (!aligned_to(x, es) || !aligned_to(dy, es) || !aligned_to(dw, es)) return DWCONV_ERR_ALIGN;
    const Shape s{B, C, L, K, pad_left, dtype};
    const DwPlan p = plan_dw(s);
    rc = check_workspace(workspace, workspace_bytes, s, p);
    if (rc != DWCONV_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *part = static_cast<float *>(workspace);
    bool wrote_dw = false;
    rc = (dtype == DWCONV_F32) ? launch_dw_partial<float>(x, dy, part, dw, &wrote_dw, s, p, st)
                               : launch_dw_partial<bf16_t>(x, dy, part, dw, &wrote_dw, s, p, st);
    if (rc != DWCONV_OK || wrote_dw) return rc;
    if (dtype == DWCONV_F32) return launch_dw_finalize<float>(part, dw, s, p, st);
    return launch_dw_finalize<bf16_t>(part, dw, s, p, st);
}

int dwconv_bwd(const void *dy, const void *x, const void *w, void *dx, void *dw, void *workspace,
               size_t workspace_bytes, int B, int C, int L, int K, int pad_left, int dtype, void *stream)
{
    if (!dy || !x || !w || !dx || !dw) return DWCONV_ERR_NULL;
    int rc = check_dw_shape(B, C, L, K, pad_left, dtype);
    if (rc != DWCONV_OK) return rc;
    const size_t es = elem_size(dtype);
    if (!aligned_to(dy, es) || !aligned_to(x, es) || !aligned_to(w, es) || !aligned_to(dx, es) || !aligned_to(dw, es))
        return DWCONV_ERR_ALIGN;
    const Shape s{B, C, L, K, pad_left, dtype};
    const DwPlan p = plan_dw(s);
    rc = check_workspace(workspace, workspace_bytes, s, p);
    if (rc != DWCONV_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *part = static_cast<float *>(workspace);
    bool wrote_dw = false;
    DwPlan pf = p;
    pf.S = p.S_fused;                                             // slices the fused kernel wrote
    rc = launch_bwd_fused(dy, x, w, dx, part, dw, &wrote_dw, s, p, st);
    if (rc >= 0) {
        if (rc != DWCONV_OK || wrote_dw) return rc;
        if (dtype == DWCONV_F32) return launch_dw_finalize<float>(part, dw, s, pf, st);
        return launch_dw_finalize<bf16_t>(part, dw, s, pf, st);
    }
    // shapes and types the fused kernel does not take: the two gradients one after the other
    rc = dwconv_bwd_input(dy, w, dx, B, C, L, K, pad_left, dtype, stream);
    if (rc != DWCONV_OK) return rc;
    return dwconv_bwd_weight(x, dy, dw, workspace, workspace_bytes, B, C, L, K, pad_left, dtype, stream);
}

int dwconv_bwd_is_fused(int B, int C, int L, int K, int pad_left, int dtype)
{
    if (check_dw_shape(B, C, L, K, pad_left, dtype) != DWCONV_OK) return 0;
    const Shape s{B, C, L, K, pad_left, dtype};
    const DwPlan p = plan_dw(s);
    const int nd = toeplitz_dmax(K, pad_left) - toeplitz_dmin(pad_left) + 1;
    if (p.rows.batch) return L <= dwconv::kRbBwdMaxL ? 1 : 0;      // sixteen rows per tile: either storage type, L % 4 == 0
    if (dtype == DWCONV_BF16 && p.rows.on) return 0;
    return (!p.longk && K >= kMfmaMinK && nd >= 2 && nd <= kMfmaMaxND && (L % (dtype == DWCONV_BF16 ? 8 : 4)) == 0 &&
            L <= kMfmaMaxL) ? 1 : 0;
}

int dwconv_bwd_weight_single_pass(int B, int C, int L, int K, int pad_left, int dtype)
{
    if (check_dw_shape(B, C, L, K, pad_left, dtype) != DWCONV_OK) return 0;
    const Shape s{B, C, L, K, pad_left, dtype};
    const DwPlan p = plan_dw(s);
    return (p.single && p.S == 1 && !p.longk) ? 1 : 0;
}

int dwconv_bwd_weight_slices(int B, int C, int L, int K, int pad_left, int dtype)
{
    if (check_dw_shape(B, C, L, K, pad_left, dtype) != DWCONV_OK) return 0;
    const Shape s{B, C, L, K, pad_left, dtype};
    return plan_dw(s).S;
}

size_t dwconv_bwd_weight_workspace_bytes(int B, int C, int L, int K, int pad_left, int dtype)
{
    if (check_dw_shape(B, C, L, K, pad_left, dtype) != DWCONV_OK) return 0;
    const Shape s{B, C, L, K, pad_left, dtype};
    return dw_workspace_bytes(s, plan_dw(s));
}

const char *dwconv_status_string(int status)
{
    switch (status) {
    case DWCONV_OK: return "ok";
    case DWCONV_ERR_NULL: return "a required pointer is NULL";
    case DWCONV_ERR_SHAPE: return "B, C, L and K must be >= 1 and B*C*L must fit 2^40 elements";
    case DWCONV_ERR_PAD: return "pad_left must lie in [0, K-1]";
    case DWCONV_ERR_DTYPE: return "dtype must be DWCONV_F32 or DWCONV_BF16";
    case DWCONV_ERR_WORKSPACE: return "workspace is NULL, smaller than dwconv_bwd_weight_workspace_bytes() or not 16-byte aligned";
    case DWCONV_ERR_ALIGN: return "a tensor pointer is not aligned to its element size";
    case DWCONV_ERR_LAUNCH: return "HIP reported an error at kernel launch";
    default: return "unknown status";
    }
}

int dwconv_version(void) { return kVersion; }

}  // extern "C"
