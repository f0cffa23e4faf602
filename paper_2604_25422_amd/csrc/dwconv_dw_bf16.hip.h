// Stage 1 of the weight gradient (Sec. IV-A eq. (dk_def)) for bf16 storage on the bf16 matrix instruction
// (v_mfma_f32_16x16x16_bf16): products of two bf16 are exact in fp32, sums are fp32.
//
//     G_d[q'][q] += sum over 16 consecutive 16-blocks n of X[n + dmin + d][q'] * dY[n][q]
// is ONE instruction per block offset d and 256 positions (the fp32 instruction needs four per 64 positions),
// so this kernel is bound by memory alone.  Operand layout: lane (i = lane % 16, kg = lane / 16) holds the
// contraction entries k = 4 kg + v, v = 0..3, i.e. element i of blocks n0 + 4 kg + v (+ d): four 2-byte LDS reads
// per operand, two into the low and two into the high halves of a register pair.
//
// The raw bf16 rows go from memory straight into LDS (16 bytes = 8 elements per lane), refilled in place for the
// next segment as soon as a half of the windows is dead, with compile-time wait counts as in
// dw_partial_direct_kernel.  Inside every group of four 16-blocks the blocks are stored permuted
// (block nb at nb ^ ((nb >> 2) & 3) within its group): the four lane groups of a read touch blocks 4 apart, which
// would otherwise fall on the same LDS banks.  The permutation is applied on the memory side of the loads.
// Loads of a segment in issue order: x0 g0 x1 g1 xt (x_h, g_h: elements [512 h, 512 h + 512) of the x window and
// of the dY tile; xt: 128 elements of x tail, two per lane; a second such load above eight block offsets).
// Needs L % 8 == 0 and 16-byte aligned tensors.  Up to sixteen block offsets fit 128 registers; above six the
// diagonal image of the accumulators (18 KB of LDS per wave at sixteen) is what limits the waves per compute unit.
#pragma once
#include "dwconv_bwd_fused.hip.h"

namespace dwconv {

constexpr int dw_bf16_tail_loads(int ND) { return (16 * ND + 127) / 128; }      // 128-element loads of x tail
constexpr int dw_bf16_win_x(int ND) { return kSegLen + 128 * dw_bf16_tail_loads(ND); }   // elements of the staged x window
constexpr int dw_bf16_wave_floats(int ND)
{
    const int stage = (dw_bf16_win_x(ND) + kSegLen) / 2, diag = ((16 * ND + 15) * 17 + 3) / 4 * 4;
    return stage > diag ? stage : diag;
}
// taps a wave hands to the block-level sum (see dw_direct_row_floats: a launch over part of the offsets owns up to 16 ND + 15)
constexpr int dw_bf16_row_floats(int ND) { return 16 * ND + (ND >= 9 ? 16 : 0); }
constexpr size_t dw_bf16_lds_bytes(int ND, int W) { return (size_t)W * (size_t)(dw_bf16_wave_floats(ND) + dw_bf16_row_floats(ND)) * sizeof(float); }

// position of logical 16-block nb inside the staged windows
__host__ __device__ constexpr int bf16_block_pos(int nb) { return (nb & ~3) | ((nb & 3) ^ ((nb >> 2) & 3)); }

// ROWS: short rows, the wave walks the virtual row of its channel (see RowsMap; pitch a multiple of 8 and row length a
// row length even: a 16-byte granule lies in one row or in one gap, or holds the last two, four or six elements of a row, in
// which case the rest of it is cleared in LDS once it has landed: rows_granule8_byte_offset); B is then 1 and segs_per_row the number of segments of the
// virtual row.  Every lane translates the position of its granule on the memory side of the loads.
template <int ND, int W, bool ROWS = false>
__global__ __launch_bounds__(64 * W, kMfmaWavesPerSimd) void dw_partial_bf16_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy, float *__restrict__ part, bf16_t *__restrict__ dw_out,
    int B, int C, int L, int K, int pad, int dmin, int segs_per_row, int j0, int j1, int seg0, int own_only,
    const RowsMap rm)
{
    // seg0, own_only: as in dw_partial_direct_kernel (the first segment of every row this launch walks; write the
    // owned taps only)
    // [j0, j1): the taps this launch owns (0, K unless the block offsets of the filter are split over two launches);
    // the other taps of its slices are written as zeros
    static_assert(ND >= 2 && 16 * ND <= 256, "the x tail is one or two 128-element loads");
    constexpr int NT = dw_bf16_tail_loads(ND);     // tail loads per segment
    constexpr int NLOADS = 4 + NT;                 // loads per segment
    constexpr int WINX = dw_bf16_win_x(ND);
    constexpr int XWE = kSegLen + 16 * ND;         // elements of the x window that are ever read
    constexpr int WREG = dw_bf16_wave_floats(ND);
    extern __shared__ __align__(16) float dyn_lds[];
    float (*s_mem)[WREG] = reinterpret_cast<float (*)[WREG]>(dyn_lds);
    constexpr int ROWF = dw_bf16_row_floats(ND);
    float (*s_dw)[ROWF] = reinterpret_cast<float (*)[ROWF]>(dyn_lds + W * WREG);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i16 = lane & 15, kg = lane >> 4;
    // ROWS, rows that are not whole 128-byte cache lines: neighbouring channels behind one L2, loads without the
    // non-temporal hint (the line a row shares with the next channel's row is then fetched once; measured on B8192 C128
    // L136 K48: weight gradient 132 -> 107 us; rows of whole lines keep the hint, they lose without it)
    const bool keep_lines = ROWS && ((L * 2) & 127) != 0;
    const int c = keep_lines ? die_run_channel((int)blockIdx.x, C) : (int)blockIdx.x;
    const int stride = (int)gridDim.y * W;
    const int ws = (int)blockIdx.y * W + __builtin_amdgcn_readfirstlane(wave);
    const int step_b = stride / segs_per_row, step_seg = stride % segs_per_row;
    int b = ws / segs_per_row, seg = ws % segs_per_row;

    const short *sx = reinterpret_cast<const short *>(s_mem[wave]);     // x window, element e of block nb at 16 pos(nb) + e
    const short *sg = sx + WINX;                                        // dY tile, same block order
    const unsigned lds_x = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) const void *)sx);
    const unsigned lds_g = lds_x + 2u * WINX;

    // ---- loop constants
    // LDS read addresses (elements).  x: block 16 c4 + 4 kg + m, m = v + d = 4 mh + ml, sits at
    // 16 c4 + 4 (kg + mh) + (ml ^ ((kg + mh) & 3)); dY: block 16 c4 + 4 kg + v sits at 16 c4 + 4 kg + (v ^ kg).
    const short *ax[ND + 3];
#pragma unroll
    for (int m = 0; m < ND + 3; ++m) {
        const int hi = kg + (m >> 2);
        ax[m] = sx + 16 * (4 * hi + ((m & 3) ^ (hi & 3))) + i16;
    }
    const short *ag[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) ag[v] = sg + 16 * (4 * kg + (v ^ kg)) + i16;
    // memory-side byte offsets of the loads: LDS granule slot `lane` of a 512-element load holds half (lane & 1)
    // of the block whose position is lane >> 1
    const int off_main = 32 * bf16_block_pos(lane >> 1) + 16 * (lane & 1);
    // tail load t: LDS elements 1024 + 128 t + 2 lane, + 1: block position 64 + 8 t + (lane >> 3), elements 2 (lane & 7), + 1
    int off_tail[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tail_elem = 16 * (64 + bf16_block_pos(8 * t + (lane >> 3))) + 2 * (lane & 7);
        off_tail[t] = tail_elem < XWE ? 2 * tail_elem : kOutOfRow;
    }

    floatx4 G[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) G[d] = floatx4{0.f, 0.f, 0.f, 0.f};

    uintx4 rx, rg;
    int x_shift;        // negative when the x window starts before the row: added to the lane offsets
    int vx0 = 0, vg0 = 0;   // ROWS: virtual positions of the first elements of the two windows
    auto aim = [&](int pb, int pseg) {
        if constexpr (ROWS) {
            x_shift = 0;
            if (pb < B) {
                // (virtual segments are walked downwards, like the batches below)
                const int t0 = (segs_per_row - 1 - pseg) * kSegLen;
                vx0 = t0 + 16 * dmin;
                vg0 = t0;
                const unsigned nbytes = rm.bytes - (unsigned)(c * L) * 2u;
                const unsigned long long ax0 = reinterpret_cast<unsigned long long>(x + (size_t)c * (size_t)L);
                const unsigned long long ag0 = reinterpret_cast<unsigned long long>(dy + (size_t)c * (size_t)L);
                rx = uintx4{(unsigned)ax0, (unsigned)(ax0 >> 32) & 0xffffu, nbytes, kBufferFlags};
                rg = uintx4{(unsigned)ag0, (unsigned)(ag0 >> 32) & 0xffffu, nbytes, kBufferFlags};
            } else {
                rx = uintx4{0u, 0u, 0u, kBufferFlags};
                rg = rx;
            }
        } else if (pb < B) {
            // batches are walked from the last to the first (the rows the input-gradient call touched last are
            // still in the last-level cache)
            const size_t row = ((size_t)(B - 1 - pb) * (size_t)C + (size_t)c) * (size_t)L;
            const int t0 = (seg0 + pseg) * kSegLen;
            const int u0 = 2 * (t0 + 16 * dmin);
            x_shift = u0 < 0 ? u0 : 0;
            // (a window that starts past the end of the row - the second of two launches - gets an empty resource)
            rx = row_tail_resource(x + row, L, u0 > 0 ? min(u0, 2 * L) : 0);
            rg = row_tail_resource(dy + row, L, 2 * t0);
        } else {
            x_shift = 0;
            rx = uintx4{0u, 0u, 0u, kBufferFlags};
            rg = rx;
        }
    };
    // ROWS: elements of the lane's granules x0 g0 x1 g1 that belong to a row which ends inside them (rows_granule8_byte_offset)
    int live_next[4] = {8, 8, 8, 8}, live_cur[4] = {8, 8, 8, 8};
    auto load_half = [&](auto hc) {         // x_h then g_h
        constexpr int h = decltype(hc)::value;
        if constexpr (ROWS) {
            const int e = (off_main >> 1) + 512 * h;        // the lane's granule: elements e .. e + 7 of the windows
            buffer_load_x4_to_lds_sel(keep_lines, rx, rows_granule8_byte_offset(rm, vx0 + e, live_next[2 * h]), lds_x + 1024u * (unsigned)h);
            buffer_load_x4_to_lds_sel(keep_lines, rg, rows_granule8_byte_offset(rm, vg0 + e, live_next[2 * h + 1]), lds_g + 1024u * (unsigned)h);
        } else {
            buffer_load_x4_to_lds(rx, off_main + (1024 * h + x_shift), lds_x + 1024u * (unsigned)h);
            buffer_load_x4_to_lds(rg, off_main + 1024 * h, lds_g + 1024u * (unsigned)h);
        }
    };
    auto tail_offset = [&](int t) {
        if constexpr (ROWS) return off_tail[t] == kOutOfRow ? kOutOfRow : rows_byte_offset<2>(rm, vx0 + (off_tail[t] >> 1));
        else return off_tail[t] + x_shift;
    };
    auto load_tail = [&]() {
        buffer_load_x1_to_lds(rx, tail_offset(0), lds_x + 2048u);
        if constexpr (NT > 1) buffer_load_x1_to_lds(rx, tail_offset(NT - 1), lds_x + 2048u + 256u);
    };

    aim(b, seg);
    load_half(std::integral_constant<int, 0>{});
    load_half(std::integral_constant<int, 1>{});
    load_tail();

    while (b < B) {
        int seg_n = seg + step_seg;
        const int carry = seg_n >= segs_per_row ? 1 : 0;
        seg_n -= carry ? segs_per_row : 0;
        const int b_n = b + step_b + carry;
        aim(b_n, seg_n);
        if constexpr (ROWS) {
#pragma unroll
            for (int i = 0; i < 4; ++i) live_cur[i] = live_next[i];
        }
        // 256-position chunk c4 (x blocks 16 c4 .. 16 c4 + 15 + ND + 2): before it, load number need(c4) of this
        // segment has landed
        //   c4 = 0: g0 (1)   c4 = 1: x1 (2)   c4 = 2: g1 (3)   c4 = 3: the last tail;   two next-segment loads are out after chunk 1
        static_for<0, 4>([&](auto cc) {
            constexpr int c4 = decltype(cc)::value;
            constexpr int need = c4 == 3 ? NLOADS - 1 : c4 + 1, issued = c4 >= 2 ? 2 : 0;
            wait_vmcnt_at_most<(NLOADS - 1 - need) + issued>();
            if constexpr (ROWS) {
                // what has just landed: x0 and g0 before chunk 0, x1 before chunk 1, g1 before chunk 2
                if constexpr (c4 == 0) { zero_slot_tail(sx + 8 * lane, live_cur[0]); zero_slot_tail(sg + 8 * lane, live_cur[1]); }
                if constexpr (c4 == 1) zero_slot_tail(sx + 512 + 8 * lane, live_cur[2]);
                if constexpr (c4 == 2) zero_slot_tail(sg + 512 + 8 * lane, live_cur[3]);
            }
            shortx4 bq;
#pragma unroll
            for (int v = 0; v < 4; ++v) bq[v] = ag[v][256 * c4];
            short e[ND + 3];
#pragma unroll
            for (int m = 0; m < ND + 3; ++m) e[m] = ax[m][256 * c4];
#pragma unroll
            for (int d = 0; d < ND; ++d) {
                const shortx4 aq = {e[d], e[d + 1], e[d + 2], e[d + 3]};
                G[d] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(aq, bq, G[d], 0, 0, 0);
            }
            if constexpr (c4 == 1 || c4 == 3) {
                // half c4 / 2 of both windows is dead: refill it for the next segment
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                load_half(std::integral_constant<int, c4 / 2>{});
                if constexpr (c4 == 3) load_tail();
            }
        });
        b = b_n; seg = seg_n;
    }
    // nothing may land in LDS after this point
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    wave_lds_fence();

    // ---- per-wave diagonal sums, then the waves of the block in wave order
    dw_wave_diagonal_sums<ND>(G, s_mem[wave], s_dw[wave], lane, j0, j1, pad, dmin);
    __syncthreads();
    for (int j = own_only ? j0 + tid : tid; j < (own_only ? j1 : K); j += 64 * W) {
        float sum = 0.f;
        if (j >= j0 && j < j1) {
#pragma unroll
            for (int w = 0; w < W; ++w) sum += s_dw[w][j - j0];
        }
        if (dw_out) st_elem(dw_out + (size_t)c * (size_t)K + (size_t)j, sum);
        else part[((size_t)blockIdx.y * (size_t)C + (size_t)c) * (size_t)K + (size_t)j] = sum;
    }
}

}  // namespace dwconv
