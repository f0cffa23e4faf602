// Forward / input gradient (Sec. IV-A eq. (dwconv) and its adjoint), fp32 storage, rows brought from memory
// straight into LDS.
//
// The contraction is that of corr_mfma_kernel (Y[n][r] = sum_d Toep_d[r][q] X[n + d][q] on v_mfma_f32_16x16x4_f32,
// Toeplitz operands in registers); what differs is how a segment reaches the matrix cores.  Buffer loads with the
// LDS bit write 16 bytes per lane into consecutive LDS slots: no staging registers, no copy through the vector ALU,
// zeros outside the row from the hardware range check.  The wave's window (1024 + 16 (ND - 1) positions) is refilled
// IN PLACE: a segment is processed in four quarters of 256 outputs; quarter i reads 16-blocks 16 i .. 16 i + 14 + ND,
// so after it the floats [256 i, 256 i + 256) are dead and the loads of the NEXT segment for them are issued at
// once.  The loads of a segment are therefore in flight for three quarters of an iteration on average instead of for
// the matrix phase alone, and a wave needs 4.5 KiB of LDS and no prefetch registers.
// Loads of a segment in issue order: r0 r1 r2 r3 (1 KiB each), then two 4-byte-per-lane tail loads ta tb.  The
// vector-memory counter retires in order, so "everything quarter i reads has landed" is one constant s_waitcnt;
// the stores share the counter and only make a wait stricter.
// The four 16-byte granules of every 16-block are permuted in LDS (granule g of block nb sits at
// g ^ ((nb >> 1) & 3)), which keeps the strided 16-byte operand reads conflict-free without padding; the
// permutation is applied on the memory side, each lane fetching the granule that belongs in its LDS slot.
#pragma once
#include "dwconv_bwd_fused.hip.h"
#include "dwconv_bwd_fused_bf16.hip.h"

namespace dwconv {

constexpr int kCorrDirectWin = kSegLen + 128;      // floats per wave: 1024 + two 64-float tail loads

// ROWS: short rows whose length is not a multiple of four (those that are take the register-staged kernel), the unit of
// work is a segment of the virtual row of a channel (see RowsMap; pitch a multiple of 4): the walk's "row" is the virtual
// segment, its "segment" the channel (walk_segs = segs_per_row = C), every lane translates the position of its granule on
// the memory side of the loads; the granule in which a row ends also brings elements of the next row in memory, which
// the lane clears in LDS once the load has landed (rows_granule4_byte_offset); the outputs of a group of four go to their
// row, as far as it reaches, or nowhere.
template <int ND, bool ROWS = false>
__global__ __launch_bounds__(64 * kCorrWavesPerBlock, kMfmaWavesPerSimd) void corr_direct_kernel(
    const float *__restrict__ in, const float *__restrict__ f, float *__restrict__ out, const CorrGeom g,
    const RowsMap rm)
{
    static_assert(ND >= 2 && 16 * (ND - 1) <= 128, "window tail is two 64-float loads");
    constexpr int XW = kSegLen + 16 * (ND - 1);    // floats of the window that are ever read
    __shared__ __align__(16) float s_in[kCorrWavesPerBlock][kCorrDirectWin];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i16 = lane & 15, k4 = lane >> 4;

    const int wg = (int)blockIdx.x * kCorrWavesPerBlock + __builtin_amdgcn_readfirstlane(wave);
    // Wave n_light + w takes segments w, w + n_main, ... of the memory order (row, segment), over the first walk_segs
    // segments of every row: at any moment the chip then reads one contiguous stretch of memory (waves that walk along
    // rows of their own, 4096 scattered streams, measured 8 to 12 % slower).  walk_segs is all segments of a row, or all
    // but the last when that one holds few positions: a nearly empty segment costs a wave as much as a memory round
    // trip and would tie the number of waves to an awkward number of segments per row, so such segments go to n_light
    // waves of their own (the first of the launch: wave w takes the last segment of rows w, w + n_light, ...).
    const bool light = wg < g.n_light;
    const int wm = wg - g.n_light;
    int row = __builtin_amdgcn_readfirstlane(light ? wg : wm / g.walk_segs);                 // b * C + c
    int seg = __builtin_amdgcn_readfirstlane(light ? g.segs_per_row - 1 : wm % g.walk_segs);
    int c = ROWS ? seg : __builtin_amdgcn_readfirstlane(row % g.C);
    if (wg >= g.n_waves || row >= g.rows) return;      // (the last block may hold spare waves)

    float *sg = s_in[wave];                            // sg[swz_pos(i)] = in~[t0 + 16 dmin + i]
    const unsigned lds_g = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) void *)sg);

    // Toeplitz operands: A[d][v] (lane (r, k)) = f_eff[16 (dmin + d) + 4k + v - r + pad]
    float A[ND][4];
    auto load_filter = [&](int ch) {
        const float *f_c = f + (size_t)ch * (size_t)g.K;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int j = 16 * (g.dmin + d) + 4 * k4 + v - i16 + g.pad;
                const bool ok = j >= 0 && j < g.K;
                const int jc = ok ? (g.reverse ? (g.K - 1 - j) : j) : 0;
                const float a = f_c[jc];
                A[d][v] = ok ? a : 0.f;
            }
    };
    // operand of lane (block i16, group k4) for offset d: granule k4 of window block 16 i + i16 + d (i: the quarter)
    const float *gx[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) gx[d] = sg + 16 * (i16 + d) + 4 * (k4 ^ (((i16 + d) >> 1) & 3));
    // memory-side offsets (floats inside the window) of what belongs in the lane's LDS slot
    const int fo_g = 4 * (4 * (lane >> 2) + ((lane & 3) ^ ((lane >> 3) & 3)));
    int fo_gt[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int slot = kSegLen + 64 * h + lane;
        const int nb = slot >> 4, gp = (slot >> 2) & 3, e = slot & 3;
        const int fg = 16 * nb + 4 * (gp ^ ((nb >> 1) & 3)) + e;
        fo_gt[h] = fg < XW ? fg : -1;
    }

    // resource of the segment the next loads belong to (wave-uniform); empty past the last segment
    uintx4 rg;
    int g_shift;                 // negative when the window starts before the row: added to the lane offsets
    int vg0 = 0;                 // ROWS: virtual position of the first float of the window
    int live_next[4] = {4, 4, 4, 4}, live_cur[4] = {4, 4, 4, 4};    // ROWS: see rows_granule4_byte_offset (loads r0 .. r3)
    auto aim = [&](int prow, int pseg) {
        if constexpr (ROWS) {
            g_shift = 0;
            if (prow < g.rows) {
                vg0 = prow * kSegLen + 16 * g.dmin;
                const unsigned long long a0 = reinterpret_cast<unsigned long long>(in + (size_t)pseg * (size_t)g.L);
                rg = uintx4{(unsigned)a0, (unsigned)(a0 >> 32) & 0xffffu, rm.bytes - (unsigned)(pseg * g.L) * 4u, kBufferFlags};
            } else {
                rg = uintx4{0u, 0u, 0u, kBufferFlags};
            }
        } else if (prow < g.rows) {
            const int v0 = 4 * (pseg * kSegLen + 16 * g.dmin);
            g_shift = v0 < 0 ? v0 : 0;
            rg = row_tail_resource(in + (size_t)prow * (size_t)g.L, g.L, v0 > 0 ? v0 : 0);
        } else {
            g_shift = 0;
            rg = uintx4{0u, 0u, 0u, kBufferFlags};
        }
    };
    auto load_region = [&](auto ic) {       // i = 0..3
        constexpr int i = decltype(ic)::value;
        if constexpr (ROWS)
            buffer_load_x4_to_lds_keep(rg, rows_granule4_byte_offset(rm, vg0 + fo_g + 256 * i, live_next[i]), lds_g + 1024u * (unsigned)i);
        else
            buffer_load_x4_to_lds_keep(rg, 4 * fo_g + (1024 * i + g_shift), lds_g + 1024u * (unsigned)i);
    };
    auto tail_offset = [&](int fo) {
        if constexpr (ROWS) return fo >= 0 ? rows_byte_offset<4>(rm, vg0 + fo) : kOutOfRow;
        else return fo >= 0 ? 4 * fo + g_shift : kOutOfRow;
    };
    auto load_tails = [&]() {
        buffer_load_x1_to_lds_keep(rg, tail_offset(fo_gt[0]), lds_g + 4096u);
        buffer_load_x1_to_lds_keep(rg, tail_offset(fo_gt[1]), lds_g + 4096u + 256u);
    };

    // The loads of the first segment go out first, the filter loads of the first channel right behind them: the wait
    // the compiler places in front of the first use of a filter value then covers both (one memory round trip at the
    // start of a wave instead of two).
    aim(row, seg);
    static_for<0, 4>([&](auto ic) { load_region(ic); });
    load_tails();
    load_filter(c);
    int cur_c = c;

    for (;;) {
        int seg_n, row_n, c_n;
        if (light) {
            seg_n = seg;
            row_n = row + g.n_light;
            c_n = c + g.step_c_light;
            c_n -= c_n >= g.C ? g.C : 0;
        } else {
            seg_n = seg + g.step_seg;
            const int carry = seg_n >= g.walk_segs ? 1 : 0;
            seg_n -= carry ? g.walk_segs : 0;
            row_n = row + g.step_rows + carry;
            c_n = c + g.step_c + carry;
            c_n -= c_n >= g.C ? g.C : 0;
            c_n -= c_n >= g.C ? g.C : 0;
            if constexpr (ROWS) c_n = seg_n;
        }
        float *out_seg = ROWS ? out + (size_t)c * (size_t)g.L                          // (ROWS: the channel's first row)
                              : out + (size_t)row * (size_t)g.L + (size_t)(seg * kSegLen);   // wave-uniform
        const bool whole = ROWS ? false : (seg + 1) * kSegLen <= g.L;
        const int t_seg = ROWS ? row * kSegLen : seg * kSegLen;
        aim(row_n, seg_n);
        if (c != cur_c) {
            load_filter(c);
            cur_c = c;
        }
        if constexpr (ROWS) {
#pragma unroll
            for (int j = 0; j < 4; ++j) live_cur[j] = live_next[j];
        }

        static_for<0, 4>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            // six loads per segment (r0 r1 r2 r3 ta tb); before quarter i everything up to r_{i+1} (i < 3) or all of
            // them has landed; i loads of the next segment have been issued since
            constexpr int need = i < 3 ? i + 1 : 5;
            wait_vmcnt_at_most<(5 - need) + i>();
            if constexpr (ROWS) {
                // what has just landed: r0 and r1 before quarter 0, r2 before quarter 1, r3 before quarter 2
                if constexpr (i == 0) { zero_slot_tail(sg + 4 * lane, live_cur[0]); zero_slot_tail(sg + 256 + 4 * lane, live_cur[1]); }
                if constexpr (i == 1 || i == 2) zero_slot_tail(sg + 256 * (i + 1) + 4 * lane, live_cur[i + 1]);
            }
            // (a quarter that lies wholly past the end of the row - the last segment of a row that is not a multiple of
            // 1024 positions - has no outputs: its matrix work is skipped, its part of the refill is not)
            const bool live = ROWS || whole || t_seg + 256 * i < g.L;
            floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
            if (live) {
                float4 bv[ND];
#pragma unroll
                for (int d = 0; d < ND; ++d) bv[d] = *reinterpret_cast<const float4 *>(gx[d] + 256 * i);
#pragma unroll
                for (int d = 0; d < ND; ++d) {
                    acc = mfma16x16x4(A[d][0], bv[d].x, acc);
                    acc = mfma16x16x4(A[d][1], bv[d].y, acc);
                    acc = mfma16x16x4(A[d][2], bv[d].z, acc);
                    acc = mfma16x16x4(A[d][3], bv[d].w, acc);
                }
            }
            // region i of the window is dead: refill it for the next segment
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            load_region(ic);
            if constexpr (i == 3) load_tails();
            // store tile i: lane (block j = i16, row group k4) owns outputs 16 j + 4 k4 + 0..3
            const int lt = 256 * i + 16 * i16 + 4 * k4;
            if constexpr (ROWS) {
                int n;
                const int e = rows_element_group(rm, t_seg + lt, n);    // four outputs: one row, one gap, or the end of a row
                if (e >= 0) st_rows_group(out_seg + e, make_float4(acc[0], acc[1], acc[2], acc[3]), n);
            } else {
                if (whole) st_elem4_stream(out_seg + lt, make_float4(acc[0], acc[1], acc[2], acc[3]));
                else if (live) st_elem4_stream_upto(out_seg + lt, make_float4(acc[0], acc[1], acc[2], acc[3]), t_seg + lt, g.L);
            }
        });
        if (row_n >= g.rows) break;
        row = row_n; seg = seg_n; c = c_n;
    }
    // nothing may land in LDS after the wave has gone
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// bf16 storage (rows of whole 16-byte granules, L % 8 == 0): the same in-place scheme on v_mfma_f32_16x16x16_bf16 with
// the raw bf16 window in LDS (2 bytes per position: a wave needs 2.25 KiB).  The window layout is that of the dY
// window of bwd_fused_bf16_kernel (bf16_dy_pos: blocks permuted inside groups of four, the 16-byte halves of a block
// swapped when bit 3 of the block index is set), which keeps the 8-byte operand reads of sixteen consecutive blocks
// conflict-free.  Loads of a segment in issue order: g0 g1 (512 positions each), gt (128-position tail, two positions
// per lane); 256-position chunk 0 needs g0, chunks 1 and 2 need g1, chunk 3 needs gt; positions [0, 512) are dead
// after chunk 1, the rest after chunk 3.
// ROWS: short rows, the unit of work is a segment of the virtual row of a channel (see RowsMap; pitch a multiple of 8 and
// row length even: a 16-byte granule lies in one row or in one gap, or holds the last two, four or six elements of a row,
// in which case the rest of it is cleared in LDS once it has landed: rows_granule8_byte_offset): the walk's "row" is the virtual segment, its
// "segment" the channel (walk_segs = segs_per_row = C), every lane translates the position of its granule on the memory
// side of the loads, and the outputs of a group of four go to their row or nowhere.
template <int ND, bool ROWS = false>
__global__ __launch_bounds__(64 * kCorrWavesPerBlock, kMfmaWavesPerSimd) void corr_direct_bf16_kernel(
    const bf16_t *__restrict__ in, const bf16_t *__restrict__ f, bf16_t *__restrict__ out, const CorrGeom g,
    const RowsMap rm)
{
    static_assert(ND >= 2 && 16 * (ND - 1) <= 128, "window tail is one 128-element load");
    constexpr int XWE = kSegLen + 16 * (ND - 1);   // elements of the window that are ever read
    __shared__ __align__(16) short s_in[kCorrWavesPerBlock][kBf16FusedWin];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i16 = lane & 15, kg = lane >> 4;

    const int wg = (int)blockIdx.x * kCorrWavesPerBlock + __builtin_amdgcn_readfirstlane(wave);
    // Wave n_light + w takes segments w, w + n_main, ... of the memory order (row, segment), over the first walk_segs
    // segments of every row: at any moment the chip then reads one contiguous stretch of memory (waves that walk along
    // rows of their own, 4096 scattered streams, measured 8 to 12 % slower).  walk_segs is all segments of a row, or all
    // but the last when that one holds few positions: a nearly empty segment costs a wave as much as a memory round
    // trip and would tie the number of waves to an awkward number of segments per row, so such segments go to n_light
    // waves of their own (the first of the launch: wave w takes the last segment of rows w, w + n_light, ...).
    const bool light = wg < g.n_light;
    const int wm = wg - g.n_light;
    int row = __builtin_amdgcn_readfirstlane(light ? wg : wm / g.walk_segs);                 // b * C + c
    int seg = __builtin_amdgcn_readfirstlane(light ? g.segs_per_row - 1 : wm % g.walk_segs);
    int c = ROWS ? seg : __builtin_amdgcn_readfirstlane(row % g.C);
    if (wg >= g.n_waves || row >= g.rows) return;      // (the last block may hold spare waves)

    const short *sg = s_in[wave];
    const unsigned lds_g = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) const void *)sg);

    // Toeplitz operands: A[d][e] (lane (r, kg)) = f_eff[16 (dmin + d) + 4 kg + e - r + pad]
    shortx4 A[ND];
    auto load_filter = [&](int ch) {
        const bf16_t *f_c = f + (size_t)ch * (size_t)g.K;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = 16 * (g.dmin + d) + 4 * kg + e - i16 + g.pad;
                const bool ok = j >= 0 && j < g.K;
                const int jc = ok ? (g.reverse ? (g.K - 1 - j) : j) : 0;
                const uint16_t bits = f_c[jc].bits;
                A[d][e] = ok ? (short)bits : (short)0;
            }
    };
    const short *gx[ND];            // operand: elements 4 kg .. 4 kg + 3 of window block i16 + d (the chunk in the immediate offset)
#pragma unroll
    for (int d = 0; d < ND; ++d) gx[d] = sg + bf16_dy_pos(i16 + d, 4 * kg);
    // memory side of the loads (bytes): what belongs in the lane's LDS slot
    const int pb = lane >> 1;                                           // position block of the lane's 16-byte granule
    const int off_g = 32 * bf16_block_pos(pb) + 16 * ((lane & 1) ^ ((pb >> 3) & 1));
    const int tnb = 64 + bf16_block_pos(lane >> 3);                     // tail: LDS elements 1024 + 2 lane, + 1
    const int te = 2 * (lane & 7);
    const int tail_g = 16 * tnb + 4 * ((te >> 2) ^ (2 * ((tnb >> 3) & 1))) + (te & 3);
    const int off_gt = tail_g < XWE ? 2 * tail_g : kOutOfRow;

    uintx4 rg;
    int g_shift;
    int vg0 = 0;            // ROWS: virtual position of the first element of the window
    auto aim = [&](int prow, int pseg) {
        if constexpr (ROWS) {
            g_shift = 0;
            if (prow < g.rows) {
                vg0 = prow * kSegLen + 16 * g.dmin;
                const unsigned long long a0 = reinterpret_cast<unsigned long long>(in + (size_t)pseg * (size_t)g.L);
                rg = uintx4{(unsigned)a0, (unsigned)(a0 >> 32) & 0xffffu, rm.bytes - (unsigned)(pseg * g.L) * 2u, kBufferFlags};
            } else {
                rg = uintx4{0u, 0u, 0u, kBufferFlags};
            }
        } else if (prow < g.rows) {
            const int v0 = 2 * (pseg * kSegLen + 16 * g.dmin);
            g_shift = v0 < 0 ? v0 : 0;
            rg = row_tail_resource(in + (size_t)prow * (size_t)g.L, g.L, v0 > 0 ? v0 : 0);
        } else {
            g_shift = 0;
            rg = uintx4{0u, 0u, 0u, kBufferFlags};
        }
    };
    int live_next[2] = {8, 8}, live_cur[2] = {8, 8};   // ROWS: see rows_granule8_byte_offset
    auto load_half = [&](auto hc) {
        constexpr int h = decltype(hc)::value;
        if constexpr (ROWS)
            buffer_load_x4_to_lds_keep(rg, rows_granule8_byte_offset(rm, vg0 + (off_g >> 1) + 512 * h, live_next[h]),
                                       lds_g + 1024u * (unsigned)h);
        else
            buffer_load_x4_to_lds_keep(rg, off_g + (1024 * h + g_shift), lds_g + 1024u * (unsigned)h);
    };
    auto load_tail = [&]() {
        if constexpr (ROWS)
            buffer_load_x1_to_lds_keep(rg, off_gt == kOutOfRow ? kOutOfRow : rows_byte_offset<2>(rm, vg0 + (off_gt >> 1)), lds_g + 2048u);
        else
            buffer_load_x1_to_lds_keep(rg, off_gt == kOutOfRow ? kOutOfRow : off_gt + g_shift, lds_g + 2048u);
    };

    aim(row, seg);
    load_half(std::integral_constant<int, 0>{});
    load_half(std::integral_constant<int, 1>{});
    load_tail();
    load_filter(c);
    int cur_c = c;

    for (;;) {
        int seg_n, row_n, c_n;
        if (light) {
            seg_n = seg;
            row_n = row + g.n_light;
            c_n = c + g.step_c_light;
            c_n -= c_n >= g.C ? g.C : 0;
        } else {
            seg_n = seg + g.step_seg;
            const int carry = seg_n >= g.walk_segs ? 1 : 0;
            seg_n -= carry ? g.walk_segs : 0;
            row_n = row + g.step_rows + carry;
            c_n = c + g.step_c + carry;
            c_n -= c_n >= g.C ? g.C : 0;
            c_n -= c_n >= g.C ? g.C : 0;
            if constexpr (ROWS) c_n = seg_n;
        }
        bf16_t *out_seg = ROWS ? out + (size_t)c * (size_t)g.L                         // (ROWS: the channel's first row)
                               : out + (size_t)row * (size_t)g.L + (size_t)(seg * kSegLen);   // wave-uniform
        const bool whole = ROWS ? false : (seg + 1) * kSegLen <= g.L;
        const int t_seg = ROWS ? row * kSegLen : seg * kSegLen;
        aim(row_n, seg_n);
        if (c != cur_c) {
            load_filter(c);
            cur_c = c;
        }
        if constexpr (ROWS) { live_cur[0] = live_next[0]; live_cur[1] = live_next[1]; }
        static_for<0, 4>([&](auto cc) {
            constexpr int c4 = decltype(cc)::value;
            // three loads per segment (g0 g1 gt); one load of the next segment is out after chunk 1
            constexpr int need = c4 == 0 ? 0 : (c4 < 3 ? 1 : 2), issued = c4 >= 2 ? 1 : 0;
            wait_vmcnt_at_most<(2 - need) + issued>();
            if constexpr (ROWS && c4 < 2) zero_slot_tail(sg + 512 * c4 + 8 * lane, live_cur[c4]);     // g_{c4} has just landed
            // (a chunk wholly past the end of the row has no outputs: its matrix work is skipped)
            const bool live = ROWS || whole || t_seg + 256 * c4 < g.L;
            floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
            if (live) {
                shortx4 bv[ND];
#pragma unroll
                for (int d = 0; d < ND; ++d) bv[d] = *reinterpret_cast<const shortx4 *>(gx[d] + 256 * c4);
#pragma unroll
                for (int d = 0; d < ND; ++d) acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(A[d], bv[d], acc, 0, 0, 0);
            }
            if constexpr (c4 == 1 || c4 == 3) {
                // half c4 / 2 of the window is dead: refill it for the next segment
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                load_half(std::integral_constant<int, c4 / 2>{});
                if constexpr (c4 == 3) load_tail();
            }
            // lane (block j = i16, row group kg) owns outputs 16 j + 4 kg + 0..3 of the chunk
            const int lt = 256 * c4 + 16 * i16 + 4 * kg;
            if constexpr (ROWS) {
                int n;
                const int e = rows_element_group(rm, t_seg + lt, n);    // four outputs: one row, one gap, or the end of a row
                if (e >= 0) st_rows_group(out_seg + e, make_float4(acc[0], acc[1], acc[2], acc[3]), n);
            } else {
                if (whole) st_elem4_stream(out_seg + lt, make_float4(acc[0], acc[1], acc[2], acc[3]));
                else if (live) st_elem4_stream_upto(out_seg + lt, make_float4(acc[0], acc[1], acc[2], acc[3]), t_seg + lt, g.L);
            }
        });
        if (row_n >= g.rows) break;
        row = row_n; seg = seg_n; c = c_n;
    }
    // nothing may land in LDS after the wave has gone
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

}  // namespace dwconv
