// Host side shared by the translation units of the library: shapes, limits, the plans that pick kernels, and the
// launch entry points every unit provides.  The kernels are instantiated in the dwconv_launch_*.hip units (one per
// path and storage type, so that they compile side by side); dwconv_api.hip holds validation, the plans and the C ABI.
#pragma once
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

#include "dwconv_common.hip.h"
#include "dwconv_dw_direct.hip.h"
#include "dwconv_longk.hip.h"
#include "dwconv_mfma.hip.h"
#include "dwconv_rowbatch.hip.h"
#include "dwconv_rowtall.hip.h"
#include "dwconv_corr_direct.hip.h"

namespace dwhost {

using dwconv::bf16_t;

struct Shape {
    int B, C, L, K, pad, dtype;
};

inline bool aligned_to(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t elem_size(int dtype) { return dtype == DWCONV_F32 ? 4 : 2; }

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? DWCONV_OK : DWCONV_ERR_LAUNCH;
}

// Block offsets d of the 16-blocked Toeplitz form that can hold a tap: d in [dmin, dmax].
inline int toeplitz_dmin(int pad) { return -((pad + 15) / 16); }
// (a one-tap filter touches a single block offset; the kernels are written for two and more, so it gets a second one
// whose taps all lie outside the filter and count as zeros)
inline int toeplitz_dmax(int K, int pad)
{
    const int d = (K - pad + 14) / 16, dm = toeplitz_dmin(pad);
    return d > dm ? d : dm + 1;
}

// Rows of m = ceil(L / 16) blocks: only the block offsets -(m - 1) .. m - 1 have a block pair inside the row, whatever the
// length of the filter; at least two (the kernels' minimum; a pair outside the row is skipped).
inline void rows_batch_offsets(int L, int K, int pad, int *dmin_out, int *nd_out)
{
    const int m = (L + 15) / 16;
    int dmin = toeplitz_dmin(pad), dmax = toeplitz_dmax(K, pad);
    if (dmin < -(m - 1)) dmin = -(m - 1);
    if (dmax > m - 1) dmax = m - 1;
    if (dmax < dmin + 1) dmax = dmin + 1;
    *dmin_out = dmin;
    *nd_out = dmax - dmin + 1;
}
constexpr int kRbMaxND = 15;      // sixteen-row kernels: offsets of a row of eight blocks

constexpr int kMfmaMinK = 1;      // (one and two taps ran 2.4x slower on the vector-ALU kernels: B32 C256 L4096 314 us per step
                                  // against 133 us at three taps)
constexpr int kMfmaMaxND = 6;          // fused backward, bf16, short rows
constexpr int kMfmaMaxNDWide = 10;     // fp32 on long rows, K up to 130: whole-channel workgroups for dW still possible
constexpr int kMfmaMaxNDDw = 16;       // fp32 on long rows, K up to 226: four-wave dW workgroups, two correlate waves per SIMD
constexpr int kMfmaMaxNDDw2 = 32;      // dW in two passes over the block offsets (K up to 482), each into its own slices
constexpr int kMfmaMaxNDDw3 = 48;      // fp32 dW in up to three passes (K up to 738)
constexpr int kMfmaMaxNDDw4 = 64;      // bf16 dW in up to four passes (K up to 994): a pass is bound by memory there
inline int mfma_max_nd(int /* either storage type */) { return kMfmaMaxNDDw; }                      // fwd, dX
// fewest block offsets the long-filter forward / input-gradient kernel takes (from there to sixteen: whichever of
// the two kernels wastes less on the row length)
inline int longk_corr_min_nd(int dtype) { return (dtype == DWCONV_F32 ? kMfmaMaxNDWide : kMfmaMaxND) + 1; }
// dW stage 1 (bf16 above six offsets: rows of whole 16-byte granules only)
inline int mfma_max_nd_dw(const Shape &s)
{
    if (s.dtype == DWCONV_F32 || (s.L % 8) == 0) {
        // two passes only where rows fill their 1024-position segments to three quarters (else the long-filter kernel)
        const long long padded = ((long long)s.L + dwconv::kSegLen - 1) / dwconv::kSegLen * dwconv::kSegLen;
        return 4ll * s.L >= 3 * padded ? (s.dtype == DWCONV_F32 ? kMfmaMaxNDDw3 : kMfmaMaxNDDw4) : kMfmaMaxNDDw;
    }
    return kMfmaMaxND;
}
// Rows that are not whole 16-byte granules (fp32 lengths that are not multiples of four, tensors whose base is only
// element-aligned; bf16: even lengths that are not multiples of eight).  The kernels that bring rows straight into
// LDS take them when every row starts on a dword: their loads are range-checked per dword, so a granule that
// straddles the end of its row is completed with zeros, and the last outputs of a row are stored by element.  Two to
// six block offsets; fp32 also the register-staged forward / input-gradient kernel of seven to sixteen offsets (row
// resources, the same range check) and the weight-gradient kernel in every number of launches; rows long enough that
// 1024-position segments are not mostly padding (the kernels skip what lies past the end of a row, the fused one does not).
// Short rows of such lengths with up to six block offsets are walked as virtual rows instead (plan_rows): there the granule in
// which a row ends is completed with zeros in LDS by the lane that loaded it.
constexpr int kRaggedMinL = 768;           // the fused backward kernel on such rows (it contracts whole segments), many-launch dW
constexpr int kRaggedRowsMinL = 129;       // forward / input gradient / weight gradient (they skip the quarters or regions past
                                           // the end of a row): B4096 C128 L202 K48 798 us per step against 1343 us on the
                                           // generic kernels; the fused kernel took 1279 us for the backward half alone
constexpr int kRaggedMaxNDF32 = 48;        // (fp32 weight gradient in up to three launches of sixteen offsets)
inline bool ragged_rows_ok(const Shape &s, int nd)
{
    return s.K >= kMfmaMinK && nd >= 2 && nd <= (s.dtype == DWCONV_F32 ? kRaggedMaxNDF32 : kMfmaMaxND) && s.L >= kRaggedRowsMinL &&
           (s.dtype == DWCONV_F32 || (s.L % 2) == 0);
}
inline bool ragged_rows_fused_ok(const Shape &s, int nd) { return ragged_rows_ok(s, nd) && s.L >= kRaggedMinL; }
constexpr int kComputeUnits = 256;     // MI355X
constexpr int kMfmaMaxL = 1 << 27;      // byte offsets inside a row stay below the out-of-row marker of the buffer loads

// Short rows (see dwconv::RowsMap): whether the matrix-core kernels should walk the virtual row of a channel, and
// its geometry.  Depends on the shape only; the gap is the same for the forward and the input-gradient pads.
struct RowsPlan {
    bool on;
    bool batch;             // rows of at most 128 positions: sixteen rows of a channel per matrix tile instead
    bool tall;              // rows of 132 to 512 positions with more block offsets than the virtual-row kernels take: sixteen
                            // rows per tile with filter and unit in LDS (dwconv_rowtall.hip.h); `on` stays false
    int units;              // batch: groups of sixteen rows per channel
    int nvs;                // 1024-position segments of the virtual row
    dwconv::RowsMap map;
};
RowsPlan plan_rows(const Shape &s);

// The same idea for the generic vector-ALU kernels, which take any row length and alignment: short rows are walked as
// the virtual row of their channel (pitch L + max(pad, K-1-pad), no rounding: these kernels load by element) when at
// least two rows fit a 1024-position tile and positions and element offsets stay 32-bit (B16384 C128 L50 K48, which no
// matrix-core kernel takes: 3.1 ms per forward with one tile per 50-position row).
struct ValuRows {
    bool on;
    long long tiles;        // 1024-position tiles of the virtual row
    dwconv::RowsMap map;
};
inline ValuRows plan_valu_rows(const Shape &s)
{
    ValuRows r;
    r.on = false; r.tiles = 0;
    r.map = dwconv::RowsMap{0, 0, 0, 0, 0u, 0u};
    const long long halo = s.pad > s.K - 1 - s.pad ? s.pad : s.K - 1 - s.pad;
    const long long P = (long long)s.L + halo;
    const long long elems = (long long)s.B * s.C * s.L;
    if (s.B < 2 || P < 2 || 2 * P > dwconv::kSegLen || elems >= (1ll << 31)) return r;     // (P = 1: 2^32 / P + 1 is not 32-bit)
    if (((long long)s.B * P + 2 * dwconv::kSegLen + s.K) * P >= (1ll << 32)) return r;      // (exact division by P)
    r.on = true;
    r.tiles = ((long long)s.B * P + dwconv::kSegLen - 1) / dwconv::kSegLen;
    r.map.P = (int)P; r.map.L = s.L; r.map.CL = s.C * s.L; r.map.Lv = (int)(s.B * P);
    r.map.M = (unsigned)((1ull << 32) / (unsigned long long)P) + 1u;
    r.map.bytes = 0u;
    return r;
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

constexpr size_t kMaxLdsBytes = 160 * 1024;

// Lets `kernel` use more than the default 64 KiB of dynamic LDS (once per kernel, device and process).
template <typename Kernel>
bool allow_large_lds(Kernel kernel)
{
    static std::mutex mu;
    static std::map<std::pair<int, const void *>, bool> done;        // (device, kernel)
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    const void *fn = reinterpret_cast<const void *>(kernel);
    const std::pair<int, const void *> key(dev, fn);
    std::lock_guard<std::mutex> lock(mu);
    auto it = done.find(key);
    if (it != done.end()) return it->second;
    const bool ok = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxLdsBytes) == hipSuccess;
    if (!ok) (void)hipGetLastError();
    done[key] = ok;
    return ok;
}

enum DwKernel { DW_VALU_K8, DW_VALU_K32, DW_VALU_K64, DW_VALU_K256 };

struct DwPlan {
    DwKernel kernel;
    bool longk;            // shape fits the long-filter matrix-core kernel (two zero-filled slices)
    int lk_wgs, lk_gd;     // its workgroups per channel, largest group of offsets (accumulators per group)
    int tall_windows;      // rows.tall: windows of fifteen relative block offsets (grid z), S / tall_windows slices each
    int lk_rs, lk_bper;    // its batch slices (each with two slices of partial sums of its own) and batch entries per slice
    std::shared_ptr<const dwconv::LongKDwTable> lk_table;   // which offsets every wave slot owns
    int S;                 // partial slices per coefficient (all passes together)
    int passes;            // launches of the stage-1 kernel, each over part of the block offsets into S / passes slices
    bool manypass;         // filters beyond the long-filter kernel's LDS: `passes` launches of sixteen offsets into TWO
                           // zero-filled sets of S / 2 slices (even launches the first set, odd launches the second)
    RowsPlan rows;         // short rows: stage 1 walks the virtual row of a channel
    int wpb;               // waves per block of the matrix-core stage-1 kernels
    int dw_nc;             // short rows, sixteen-row units: channels per block of the stage-1 kernel (1 or 2)
    int S_fused;           // slices the fused backward call writes (differs from S for rows of at most 48 positions)
    bool single;           // S == 1 with one block per channel: stage 1 may write the gradient itself
    int tiles_per_row;     // segments the matrix-core kernels walk per row (per virtual row for short rows)
    int valu_tiles_per_row, valu_items_per_slice;   // the same bookkeeping for the generic kernel
    ValuRows valu_rows;    // short rows on the generic kernel: tiles of the virtual row of a channel
    int segs_per_wave;     // (b, segment) items a wave of the matrix-core kernels walks
    int items_per_slice;   // (b, segment) items each slice owns = wpb * segs_per_wave
};

constexpr int kDwTT = dwconv::kSegLen;   // positions per staged tile (every stage-1 kernel)
constexpr int kDwThreads = 256;

DwPlan plan_dw(const Shape &s);

// Launch entry points of the per-path units.  A return value of -1 (fused backward only) means "does not apply".
// Rows of 132 to 512 positions with long filters (RowsPlan::tall; units of their own: dwconv_launch_rowtall_*.hip).
int launch_corr_rowtall_f32(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st);
int launch_corr_rowtall_bf16(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st);
int launch_dw_rowtall_f32(const void *x, const void *dy, float *part, const Shape &s, const DwPlan &p, hipStream_t st);
int launch_dw_rowtall_bf16(const void *x, const void *dy, float *part, const Shape &s, const DwPlan &p, hipStream_t st);
int launch_corr_f32(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st);
int launch_corr_bf16(const void *in, const void *f, void *out, const Shape &s, int pad_eff, int reverse, hipStream_t st);
int launch_dw_partial_f32(const void *x, const void *dy, float *part, void *dw_out, bool *wrote_dw, const Shape &s,
                          const DwPlan &p, hipStream_t st);
int launch_dw_partial_bf16(const void *x, const void *dy, float *part, void *dw_out, bool *wrote_dw, const Shape &s,
                           const DwPlan &p, hipStream_t st);
// (fp32, seven to sixteen block offsets; returns -1 when it does not apply)
int launch_dw_partial_wide_f32(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                               int dmin, int nd, hipStream_t st);
// (bf16, seven to sixteen block offsets, rows of whole 16-byte granules; returns -1 when it does not apply)
int launch_dw_partial_wide_bf16(const void *x, const void *dy, float *part, void *dw_out, const Shape &s, const DwPlan &p,
                                int dmin, int nd, hipStream_t st);
int launch_bwd_fused_f32(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out, bool *wrote_dw,
                         const Shape &s, const DwPlan &p, hipStream_t st);
int launch_bwd_fused_bf16(const void *dy, const void *x, const void *w, void *dx, float *part, void *dw_out,
                          bool *wrote_dw, const Shape &s, const DwPlan &p, hipStream_t st);

}  // namespace dwhost
