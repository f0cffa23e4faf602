// C ABI of the gfx950 depthwise 1-D convolution library: argument validation,
// kernel selection and launch.  Declarations and argument contracts are in
// include/dwconv.h; the operator is the one of the paper's Sec. IV-A.
#include "dwconv_host.hip.h"
#include "dwconv_valu.hip.h"

// Partial sums of the weight gradient for callers that cannot hand over a workspace (dwconv_bwd_weight_noalloc):
// one array per GPU, living in the code object's data segment until the process ends.  In host code the name below
// is only a handle for hipGetSymbolAddress; kernels get the device address that call returns.
constexpr size_t kScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace dwhost {

constexpr int kVersion = 101;   // 0.1.1

// Device address of `scratch` on the current device (looked up once per device and kept).
int scratch_pointer(void **out)
{
    static std::mutex mu;
    static std::map<int, void *> per_device;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return DWCONV_ERR_LAUNCH;
    }
    std::lock_guard<std::mutex> lock(mu);
    auto it = per_device.find(dev);
    if (it == per_device.end()) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return DWCONV_ERR_LAUNCH;
        }
        it = per_device.emplace(dev, ptr).first;
    }
    *out = it->second;
    return DWCONV_OK;
}

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

RowsPlan plan_rows(const Shape &s)
{
    RowsPlan r;
    r.on = false; r.batch = false; r.tall = false; r.units = 0; r.nvs = 0;
    r.map = dwconv::RowsMap{0, 0, 0, 0, 0u, 0u};
    const int nd = toeplitz_dmax(s.K, s.pad) - toeplitz_dmin(s.pad) + 1;
    if (s.K < kMfmaMinK || nd < 2) return r;
    const long long es = (long long)elem_size(s.dtype);
    // Sixteen rows per tile (rows of at most 128 positions, either storage type): byte offsets inside a unit stay below
    // the out-of-row marker; the offsets that count are those inside the row (rows_batch_offsets: a filter as long as
    // the row, or longer, is no different from a short one).  Rows that are not whole granules of four must start on a
    // dword (any fp32 row, bf16 rows of even length) and have their kernels for up to six offsets only.
    bool batch = s.L <= dwconv::kRbMaxL && (long long)dwconv::kRbRows * s.C * s.L * es < (1ll << 30);
    if (batch) {
        int bd, bn;
        rows_batch_offsets(s.L, s.K, s.pad, &bd, &bn);
        if ((s.L % 4) != 0) batch = bn <= kMfmaMaxND && (s.dtype == DWCONV_F32 || (s.L % 2) == 0);
        else batch = bn <= kRbMaxND;
    }
    // Virtual rows (whole granules; up to six offsets, fp32 sixteen): where a 1024-position segment of a row would be more than a
    // quarter padding, and positions stay 32-bit.
    const long long halo = s.pad > s.K - 1 - s.pad ? s.pad : s.K - 1 - s.pad;
    // (pitch: whole granules of four; bf16 of eight - rows AND gaps - so that the kernels that load 16 bytes per lane apply;
    // a bf16 row of even length that is not a multiple of eight ends inside its last granule, see rows_granule8_byte_offset)
    const long long gr = s.dtype == DWCONV_F32 ? 4 : 8;
    const long long P = (s.L + gr - 1) / gr * gr + (halo + gr - 1) / gr * gr;
    const long long padded = ((long long)s.L + dwconv::kSegLen - 1) / dwconv::kSegLen * dwconv::kSegLen;
    const long long elems = (long long)s.B * s.C * s.L;
    // (seven to sixteen offsets, fp32: only while the gaps stay below half a row - with a filter as long as the row half of
    // the virtual row is gap, and the tall-row kernels below do better: B3200 C128 L160 K160 fwd 354 us here)
    // (rows that end inside a 16-byte granule - fp32 lengths that are not multiples of four, bf16 even lengths that are not
    // multiples of eight: the kernels that load rows straight into LDS, up to six offsets; bf16 rows of odd length do not
    // start on a dword)
    const bool vrows = (s.dtype == DWCONV_F32 ? ((s.L % 4) == 0 || nd <= kMfmaMaxND) : (s.L % 2) == 0) &&
                       (nd <= kMfmaMaxND || (s.dtype == DWCONV_F32 && (s.L % 4) == 0 && nd <= kMfmaMaxNDDw && 2 * P <= 3 * (long long)s.L)) &&
                       4 * padded > 5 * P && elems * es <= (1ll << 30) &&
                       (long long)s.B * P * P < (1ll << 32) && (long long)s.B * P < (1ll << 31);
    if (vrows) {
        r.on = true;
        r.nvs = (int)(((long long)s.B * P + dwconv::kSegLen - 1) / dwconv::kSegLen);
        r.map.P = (int)P; r.map.L = s.L; r.map.CL = s.C * s.L; r.map.Lv = (int)(s.B * P);
        r.map.M = (unsigned)((1ull << 32) / (unsigned long long)P) + 1u;
        r.map.bytes = (unsigned)(elems * es);
    }
    // bf16 rows of 64 to 128 positions in whole 16-byte granules: the virtual-row kernels bring the raw bf16 rows straight
    // into LDS for the bf16 matrix instruction, while the sixteen-row kernels widen them to fp32 in registers (B8192 C128
    // L128 K48: 542 -> 313 us per step, L96: 528 -> 366, L64: 462 -> 346; at 48 positions and below the sixteen-row kernels
    // win, 416 against 525 us)
    if (batch && vrows && s.dtype == DWCONV_BF16 && s.L >= 64 && (s.L % 2) == 0 && (P % 8) == 0) batch = false;
    if (batch) {
        r.on = true; r.batch = true;
        r.units = (s.B + dwconv::kRbRows - 1) / dwconv::kRbRows;
    }
    // Rows of nine to thirty-two blocks with more block offsets than the virtual-row kernels take (filters of the order
    // of the row length): sixteen rows per tile with the filter window and the unit in LDS.
    const int m = (s.L + 15) / 16;
    // (bf16 up to twenty blocks: beyond, the long-filter kernels on the bf16 matrix instruction are faster - B1016 C128 L516
    // K516 882 us per step there against 1389 us here at L = 512; fp32 2068 against 1373 us)
    // (rows that are not whole granules: they must start on a dword - any fp32 length, bf16 even lengths)
    const bool tall_rag = (s.L % 4) != 0 && nd > kMfmaMaxND && (s.dtype == DWCONV_F32 || (s.L % 2) == 0);      // (up to six offsets:
                                                                     // the kernels that load rows straight into LDS)
    if (!batch && !vrows && ((s.L % 4) == 0 || tall_rag) && s.L > dwconv::kRbMaxL && m >= dwconv::kRtMinBlocks &&
        m <= (s.dtype == DWCONV_F32 ? dwconv::kRtMaxBlocks : 20) &&
        (long long)dwconv::kRbRows * s.C * s.L * es < (1ll << 30)) {
        r.tall = true;
        r.units = (s.B + dwconv::kRbRows - 1) / dwconv::kRbRows;
    }
    return r;
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
    if (dtype == DWCONV_F32) return launch_corr_f32(in, f, out, s, pad_eff, reverse, st);
    return launch_corr_bf16(in, f, out, s, pad_eff, reverse, st);
}

// ------------------------------------------------------------------ weight gradient
// Long filters: the assignment of block offsets to wave slots (dwconv::LongKDwTable), balanced by work.
// Work of an offset d = the 64-position chunks in which it reaches the row; a group of n offsets runs n matrix
// instructions over the union of its offsets' chunks.  Groups are cut greedily under a cap on size (9) and on
// work; the cap is searched so that at most two groups per slot suffice and the busiest slot is as light as
// possible; groups go to slots heaviest first, each to the least loaded slot that still has room.  The result
// depends on (L, K, pad, slots) only and is cached.
// Block offsets of the filter that have a block pair inside a row of ceil(L / 16) blocks (at least one).
static void longk_dw_offsets(const Shape &s, int *dmin_out, int *dmax_out)
{
    const int nb = (s.L + 15) / 16;
    int dmin = toeplitz_dmin(s.pad), dmax = toeplitz_dmax(s.K, s.pad);
    if (dmin < -(nb - 1)) dmin = -(nb - 1);
    if (dmax > nb - 1) dmax = nb - 1;
    if (dmax < dmin) dmax = dmin;
    *dmin_out = dmin;
    *dmax_out = dmax;
}

std::shared_ptr<const dwconv::LongKDwTable> longk_dw_table(const Shape &s, int wgs, int *max_group)
{
    struct Entry { std::shared_ptr<const dwconv::LongKDwTable> table; int max_group; };
    static std::mutex mu;
    static std::map<std::array<int, 4>, Entry> cache;
    const std::array<int, 4> key = {s.L, s.K, s.pad, wgs};
    std::lock_guard<std::mutex> lock(mu);
    auto it = cache.find(key);
    if (it != cache.end()) { *max_group = it->second.max_group; return it->second.table; }

    // (only the block offsets that have a block pair inside a row: a filter longer than the row has offsets that reach nothing)
    int dmin, dmax;
    longk_dw_offsets(s, &dmin, &dmax);
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
    int nd = toeplitz_dmax(s.K, s.pad) - toeplitz_dmin(s.pad) + 1;
    if (p.rows.batch) {                                          // (the offsets inside a row are all that count there)
        int bd;
        rows_batch_offsets(s.L, s.K, s.pad, &bd, &nd);
    }
    const bool mfma_shape = p.rows.batch || (s.K >= kMfmaMinK && nd >= 2 && nd <= mfma_max_nd_dw(s) &&
                                             ((s.L % 4) == 0 || ragged_rows_ok(s, nd)) && s.L <= kMfmaMaxL);
    // When the channels alone fill the chip evenly (C = 1, 2 or 3 per compute unit), one block of 16, 8 or 5
    // waves takes a whole channel: no slices, no second stage.
    p.wpb = dwconv::kWavesPerBlock;
    p.single = false;
    p.dw_nc = 1;
    if (mfma_shape && nd <= (s.dtype == DWCONV_F32 ? kMfmaMaxNDWide : kMfmaMaxND) && s.C % kComputeUnits == 0 &&
        s.C / kComputeUnits <= 3 && !(p.rows.batch && (s.L % 4) != 0) && !(p.rows.on && !p.rows.batch && nd > kMfmaMaxND)) {
        int wpb = 16 / (s.C / kComputeUnits);
        // short filters leave the matrix pipe idle, and what then counts is how many bytes the chip has in flight:
        // two rows of 4 KiB per wave are enough with 8 to 12 waves per compute unit (B64 C512 L2048 K7: 82 us against
        // 87 us with 16 waves; bf16 B128 C768 L1024 K32: 59.6 against 60.8 us)
        if (nd <= 3 && s.C / kComputeUnits >= 2) wpb = 4;
        // (sixteen-row units of rows longer than 48 positions need more LDS than sixteen waves have)
        const bool fits = (!p.rows.batch || dwconv::rb_dw_lds_bytes(s.L, nd, wpb, 1) <= kMaxLdsBytes) &&
                          (nd <= kMfmaMaxND || dwconv::dw_direct_lds_bytes(nd, wpb) <= kMaxLdsBytes);
        if (items >= 2 * wpb && fits) { p.wpb = wpb; p.single = true; }
    }
    // Small problems (at most four segments or units per wave of one four-wave workgroup per channel) are bound by
    // launch latency: one workgroup per channel and no second launch there too.
    if (mfma_shape && !p.single && items <= 4 * dwconv::kWavesPerBlock) p.single = true;
    long long groups = s.C;                                      // blocks along the channel axis
    if (p.rows.batch && !p.single && s.C % 2 == 0 && (s.L * (int)elem_size(s.dtype)) % 128 != 0 && s.L <= 48 && (s.L % 4) == 0) {
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
    // seventeen to thirty-two block offsets: two launches of the register-resident kernel, each over half of
    // the offsets and into its own slices (a launch writes zeros to the taps of the other half); stage 2 adds them
    // (bf16: up to four launches over quarters of up to sixty-four offsets)
    p.passes = (mfma_shape && nd > kMfmaMaxNDDw) ? (nd + kMfmaMaxNDDw - 1) / kMfmaMaxNDDw : 1;
    if (p.passes > 1) {
        p.single = false;
        p.S *= p.passes;
    }
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
    p.lk_rs = 1; p.lk_bper = s.B;
    const int NCH = (s.L + 63) / 64;
    if (!p.rows.batch && nd > mfma_max_nd_dw(s) && s.K <= dwconv::kLkMaxK && (s.L % 4) == 0 && (s.L + 15) / 16 <= dwconv::kLkMaxBlocks &&
        dwconv::longk_dw_lds_bytes(s.L, NCH) <= kMaxLdsBytes) {
        const int per_wg = 2 * dwconv::kLkWaves * dwconv::kLkDwMaxGD;
        int lk_dmin, lk_dmax;
        longk_dw_offsets(s, &lk_dmin, &lk_dmax);
        p.lk_wgs = (lk_dmax - lk_dmin + 1 + per_wg - 1) / per_wg;
        p.lk_table = longk_dw_table(s, p.lk_wgs, &p.lk_gd);
    }
    p.manypass = false;
    if (!p.rows.batch && !p.lk_table && nd > mfma_max_nd_dw(s) && (s.L % (s.dtype == DWCONV_F32 ? 4 : 8)) == 0 && s.L >= kRaggedMinL &&
        s.L <= kMfmaMaxL && !p.rows.on) {
        // filters (or rows) too long for the long-filter kernel's LDS: the register-resident kernel, sixteen block
        // offsets per launch, every launch adding the taps it owns to one of two zero-filled sets of slices
        p.manypass = true;
        p.single = false;
        p.wpb = dwconv::kWavesPerBlock;
        p.passes = (nd + kMfmaMaxNDDw - 1) / kMfmaMaxNDDw;
        long long sp = (kTargetWaves / p.wpb + s.C - 1) / s.C;       // workgroups per channel and launch
        const long long all_items = (long long)s.B * (((long long)s.L + kDwTT - 1) / kDwTT);
        if (sp > (all_items + p.wpb - 1) / p.wpb) sp = (all_items + p.wpb - 1) / p.wpb;
        if (sp < 1) sp = 1;
        p.S = (int)(2 * sp);
        p.S_fused = p.S;
        p.tiles_per_row = (int)(((long long)s.L + kDwTT - 1) / kDwTT);
        p.valu_items_per_slice = (int)((all_items + p.S - 1) / p.S);
        p.items_per_slice = p.valu_items_per_slice;
    }
    if (p.lk_table) {
        p.longk = true;
        // Workgroups: channels x groups of offsets.  Where that is fewer than two per compute unit (few channels, or rows
        // so short that the offsets fit one workgroup) the batch is cut into slices too, each with its own two slices
        // of partial sums (B78125 C1 L256 K700: one workgroup walked the whole batch, 112 ms; B128 C128 L4096 K4096: 128
        // workgroups on 256 compute units).  At most 128, at least one pair of rows each, workspace at most 64 MiB.
        long long rs = (2LL * kComputeUnits + (long long)s.C * p.lk_wgs - 1) / ((long long)s.C * p.lk_wgs);
        if (rs > 128) rs = 128;
        if (rs > (s.B + dwconv::kLkRows - 1) / dwconv::kLkRows) rs = (s.B + dwconv::kLkRows - 1) / dwconv::kLkRows;
        while (rs > 1 && 2 * rs * (long long)s.C * s.K * (long long)sizeof(float) > (64ll << 20)) --rs;
        if (rs < 1) rs = 1;
        long long bper = ((s.B + rs - 1) / rs + dwconv::kLkRows - 1) / dwconv::kLkRows * dwconv::kLkRows;
        rs = (s.B + bper - 1) / bper;
        p.lk_rs = (int)rs;
        p.lk_bper = (int)bper;
        p.S = (int)(2 * rs);
        p.S_fused = p.S;                                   // (no fused kernel for long filters: nothing needs more slices)
        p.items_per_slice = (int)((items + p.S - 1) / p.S);       // the generic kernel, if it has to run, uses the same slices
        p.valu_items_per_slice = (int)(((long long)s.B * p.valu_tiles_per_row + p.S - 1) / p.S);      // (of its own items: real rows)
    }
    p.tall_windows = 0;
    if (p.rows.tall) {
        // windows of fifteen relative block offsets (grid z), each with S / windows slices over units of four rows: about two
        // workgroups per compute unit
        int bd, bn;
        rows_batch_offsets(s.L, s.K, s.pad, &bd, &bn);
        const long long nwin = (bn + dwconv::kRtWindow - 1) / dwconv::kRtWindow;
        const long long units = (s.B + 3) / 4;
        long long su = (2LL * kComputeUnits + (long long)s.C * nwin - 1) / ((long long)s.C * nwin);
        const long long su_max = (units + dwconv::kRtWaves - 1) / dwconv::kRtWaves;
        if (su > su_max) su = su_max;
        if (su > 4096) su = 4096;
        if (su < 1) su = 1;
        p.tall_windows = (int)nwin;
        p.longk = false; p.lk_table = nullptr; p.manypass = false; p.single = false; p.passes = 1;
        p.wpb = dwconv::kRtWaves;
        p.S = (int)(su * nwin);
        p.S_fused = p.S;
        p.tiles_per_row = (int)units;
        p.items_per_slice = (int)((units + su - 1) / su);
        p.valu_items_per_slice = (int)(((long long)s.B * p.valu_tiles_per_row + p.S - 1) / p.S);
    }
    // the generic kernel on short rows: its items are the tiles of the virtual row of the channel
    p.valu_rows = plan_valu_rows(s);
    if (p.valu_rows.on) {
        p.valu_tiles_per_row = (int)p.valu_rows.tiles;
        p.valu_items_per_slice = (int)((p.valu_rows.tiles + p.S - 1) / p.S);
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

template <typename T>
int launch_dw_finalize(const float *part, void *dw, const Shape &s, const DwPlan &p, hipStream_t st)
{
    const size_t CK = (size_t)s.C * (size_t)s.K;
    if (p.S >= 32 && CK <= 16 * 2048) {
        // many slices of few coefficients: the slices in parallel (same order of the sum)
        const size_t nb = (CK + 15) / 16;
        hipLaunchKernelGGL((dwconv::dw_finalize_many_kernel<T>), dim3((unsigned)nb), dim3(256), 0, st, part,
                           static_cast<T *>(dw), p.S, CK);
        return launch_status();
    }
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

}  // namespace dwhost

using namespace dwhost;

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
    if (dtype == DWCONV_F32) return launch_dw_partial_f32(x, dy, part, nullptr, nullptr, s, p, st);
    return launch_dw_partial_bf16(x, dy, part, nullptr, nullptr, s, p, st);
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
    rc = (dtype == DWCONV_F32) ? launch_dw_partial_f32(x, dy, part, dw, &wrote_dw, s, p, st)
                               : launch_dw_partial_bf16(x, dy, part, dw, &wrote_dw, s, p, st);
    if (rc != DWCONV_OK || wrote_dw) return rc;
    if (dtype == DWCONV_F32) return launch_dw_finalize<float>(part, dw, s, p, st);
    return launch_dw_finalize<bf16_t>(part, dw, s, p, st);
}

int dwconv_bwd_weight_noalloc(const void *x, const void *dy, void *dw, int B, int C, int L, int K, int pad_left,
                              int dtype, void *stream)
{
    if (!x || !dy || !dw) return DWCONV_ERR_NULL;
    int rc = check_dw_shape(B, C, L, K, pad_left, dtype);
    if (rc != DWCONV_OK) return rc;
    const size_t es = elem_size(dtype);
    if (!aligned_to(x, es) || !aligned_to(dy, es) || !aligned_to(dw, es)) return DWCONV_ERR_ALIGN;
    const Shape s{B, C, L, K, pad_left, dtype};
    if (dw_workspace_bytes(s, plan_dw(s)) > kScratchBytes) return DWCONV_ERR_SCRATCH;
    void *ptr = nullptr;
    rc = scratch_pointer(&ptr);
    if (rc != DWCONV_OK) return rc;
    return dwconv_bwd_weight(x, dy, dw, ptr, kScratchBytes, B, C, L, K, pad_left, dtype, stream);
}

size_t dwconv_noalloc_scratch_bytes(void) { return kScratchBytes; }

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
    rc = dtype == DWCONV_F32 ? launch_bwd_fused_f32(dy, x, w, dx, part, dw, &wrote_dw, s, p, st)
                             : launch_bwd_fused_bf16(dy, x, w, dx, part, dw, &wrote_dw, s, p, st);
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
    // sixteen rows per tile, either storage type (its workgroups own four neighbouring channels: with fewer, most of
    // their waves would idle and the two separate kernels are faster - B416666 C1 L48 K33: 298 against 120 us)
    if (p.rows.batch) return (L <= dwconv::kRbBwdMaxL && C >= dwconv::kRbBwdWaves) ? 1 : 0;
    if (p.rows.tall) return 0;
    if (dtype == DWCONV_BF16 && p.rows.on && !p.rows.batch && ((L % 2) != 0 || (p.rows.map.P % 8) != 0)) return 0;
    const bool rows_fit = p.rows.on ? true      // (virtual rows; bf16: of even length, checked above)
                          : dtype == DWCONV_BF16 ? ((L % 8) == 0 || ((L % 2) == 0 && ((L % 4) != 0 ? ragged_rows_fused_ok(s, nd) : true)))
                                                 : ((L % 4) == 0 || ragged_rows_fused_ok(s, nd));
    return (!p.longk && K >= kMfmaMinK && nd >= 2 && nd <= kMfmaMaxND && rows_fit && L <= kMfmaMaxL) ? 1 : 0;
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
    case DWCONV_ERR_SCRATCH: return "this shape needs more partial-sum space than the library's built-in scratch holds "
                                    "(dwconv_noalloc_scratch_bytes()): use dwconv_bwd_weight with a workspace";
    default: return "unknown status";
    }
}

int dwconv_version(void) { return kVersion; }

}  // extern "C"

