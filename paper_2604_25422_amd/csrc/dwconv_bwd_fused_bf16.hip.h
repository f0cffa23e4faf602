// Fused backward pass for bf16 storage: input gradient and stage 1 of the weight gradient from one pass over dY,
// both on v_mfma_f32_16x16x16_bf16 (exact products, fp32 sums), raw bf16 rows loaded straight into LDS.
// The two halves are those of corr_mfma_bf16_kernel (dX: D[r][n] += Toep'_d[r][k] dY[n + dmin' + d][k], one
// instruction per block offset and 256 outputs) and dw_partial_bf16_kernel (dW: G_d[q'][q] += sum over 16 blocks n
// of X[n + dmin + d][q'] dY[n][q]); dX out of this kernel is bit-identical to the separate call.
//
// The dY window [t0 + 16 dmin', + 1024 + 16 ND) serves two read patterns:
//   dX operand: lane (j, kg) reads the 8 bytes of elements 4 kg .. 4 kg + 3 of block j + d        (16 blocks per read)
//   dW operand: lane (i, kg) gathers element i of blocks 4 kg + v (+ offset), v = 0..3           (blocks 4 apart)
// Stored plainly, the first puts blocks 8 apart and the second blocks 4 apart on the same banks.  Layout used:
// inside every group of four blocks the blocks are permuted (nb at nb ^ ((nb >> 2) & 3), as in
// dw_partial_bf16_kernel), and the two 16-byte halves of a block are swapped when bit 3 of the block index is
// set; both are whole 16-byte granules, so the memory side of the loads applies them.  The x window uses the block
// permutation only.
//
// A segment is four 256-position chunks: chunk c4 = dX tile c4, then dW chunk c4.  Elements [0, 512) of both
// windows are dead after chunk 1, the rest after chunk 3; loads of a segment in issue order: x0 g0 x1 g1 xt gt
// (xt, gt: 128-element tails, two elements per lane).  Needs L % 8 == 0 and 16-byte aligned tensors.
//
// ROWS: short rows, the wave walks the virtual row of its channel (see RowsMap; pitch a multiple of 8 and row length a
// row length even: a 16-byte granule lies in one row or in one gap, or holds the last two, four or six elements of a row, in
// which case the rest of it is cleared in LDS once it has landed: rows_granule8_byte_offset); B is then 1 and segs_per_row the number of segments of the
// virtual row.  Every lane translates the position of its granule on the memory side of the loads, and the position of
// its four outputs at the stores.
#pragma once
#include "dwconv_dw_bf16.hip.h"

namespace dwconv {

constexpr int kBf16FusedWin = kSegLen + 128;        // elements per staged window
constexpr int bwd_fused_bf16_wave_floats(int ND)
{
    const int stage = kBf16FusedWin, diag = ((16 * ND + 15) * 17 + 3) / 4 * 4;      // two windows of 2-byte elements
    return stage > diag ? stage : diag;
}
constexpr size_t bwd_fused_bf16_lds_bytes(int ND, int W)
{
    return (size_t)W * (size_t)(bwd_fused_bf16_wave_floats(ND) + 16 * ND) * sizeof(float);
}

// element position of (logical block nb, element i) in the dY window
__host__ __device__ constexpr int bf16_dy_pos(int nb, int i)
{
    return 16 * bf16_block_pos(nb) + 4 * ((i >> 2) ^ (2 * ((nb >> 3) & 1))) + (i & 3);
}

template <int ND, int W, bool ROWS = false>
__global__ __launch_bounds__(64 * W, kMfmaWavesPerSimd) void bwd_fused_bf16_kernel(
    const bf16_t *__restrict__ dy, const bf16_t *__restrict__ x, const bf16_t *__restrict__ f, bf16_t *__restrict__ dx,
    float *__restrict__ part, bf16_t *__restrict__ dw_out, int B, int C, int L, int K, int pad, int dmin,
    int segs_per_row, const RowsMap rm)
{
    static_assert(ND >= 2 && 16 * ND <= 128, "window tails are one 128-element load each");
    constexpr int XWE = kSegLen + 16 * ND;         // elements of either window that are ever read
    constexpr int WREG = bwd_fused_bf16_wave_floats(ND);
    extern __shared__ __align__(16) float dyn_lds[];
    float (*s_mem)[WREG] = reinterpret_cast<float (*)[WREG]>(dyn_lds);
    float (*s_dw)[16 * ND] = reinterpret_cast<float (*)[16 * ND]>(dyn_lds + W * WREG);

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

    const int pad_x = K - 1 - pad;                 // pad of the input-gradient correlation
    const int dmin_x = -((pad_x + 15) / 16);       // its first block offset
    const short *sx = reinterpret_cast<const short *>(s_mem[wave]);     // x window  [t0 + 16 dmin,   ...)
    const short *sg = sx + kBf16FusedWin;                               // dY window [t0 + 16 dmin_x, ...)
    const unsigned lds_x = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) const void *)sx);
    const unsigned lds_g = lds_x + 2u * kBf16FusedWin;

    // ---- loop constants
    // Toeplitz operands of the input gradient: A[d][e] (lane (r, kg)) = w[c, K-1-j], j = 16 (dmin_x + d) + 4 kg + e - r + pad_x
    shortx4 A[ND];
    {
        const bf16_t *f_c = f + (size_t)c * (size_t)K;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = 16 * (dmin_x + d) + 4 * kg + e - i16 + pad_x;
                const bool ok = j >= 0 && j < K;
                const uint16_t bits = f_c[ok ? (K - 1 - j) : 0].bits;
                A[d][e] = ok ? (short)bits : (short)0;
            }
    }
    // LDS read addresses (elements; the 256-position chunk goes into the immediate offset)
    const short *gx[ND];            // dX operand: elements 4 kg .. 4 kg + 3 of window block i16 + d
#pragma unroll
    for (int d = 0; d < ND; ++d) gx[d] = sg + bf16_dy_pos(i16 + d, 4 * kg);
    const short *gw[4];             // dW operand from dY: element i16 of window block 4 kg + v - dmin_x
#pragma unroll
    for (int v = 0; v < 4; ++v) gw[v] = sg + bf16_dy_pos(4 * kg + v - dmin_x, i16);
    const short *ax[ND + 3];        // dW operand from x: element i16 of window block 4 kg + m, m = v + d
#pragma unroll
    for (int m = 0; m < ND + 3; ++m) ax[m] = sx + 16 * bf16_block_pos(4 * kg + m) + i16;
    // memory side of the loads (bytes): what belongs in the lane's LDS slot
    const int pb = lane >> 1;                                           // position block of the lane's 16-byte granule
    const int off_x = 32 * bf16_block_pos(pb) + 16 * (lane & 1);
    const int off_g = 32 * bf16_block_pos(pb) + 16 * ((lane & 1) ^ ((pb >> 3) & 1));
    // tails: LDS elements 1024 + 2 lane, + 1: position block 64 + (lane >> 3), elements 2 (lane & 7), + 1
    const int tnb = 64 + bf16_block_pos(lane >> 3);                     // logical block (64 is a multiple of 16)
    const int te = 2 * (lane & 7);
    const int tail_x = 16 * tnb + te;
    const int tail_g = 16 * tnb + 4 * ((te >> 2) ^ (2 * ((tnb >> 3) & 1))) + (te & 3);
    const int off_xt = tail_x < XWE ? 2 * tail_x : kOutOfRow;
    const int off_gt = tail_g < XWE ? 2 * tail_g : kOutOfRow;

    floatx4 G[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) G[d] = floatx4{0.f, 0.f, 0.f, 0.f};

    uintx4 rx, rg;
    int x_shift, g_shift;       // negative when a window starts before the row: added to the lane offsets
    int vx0 = 0, vg0 = 0;       // ROWS: virtual positions of the first elements of the two windows
    auto aim = [&](int pbat, int pseg) {
        if constexpr (ROWS) {
            x_shift = g_shift = 0;
            if (pbat < B) {
                const int t0 = pseg * kSegLen;
                vx0 = t0 + 16 * dmin;
                vg0 = t0 + 16 * dmin_x;
                const unsigned nbytes = rm.bytes - (unsigned)(c * L) * 2u;
                const unsigned long long ax0 = reinterpret_cast<unsigned long long>(x + (size_t)c * (size_t)L);
                const unsigned long long ag0 = reinterpret_cast<unsigned long long>(dy + (size_t)c * (size_t)L);
                rx = uintx4{(unsigned)ax0, (unsigned)(ax0 >> 32) & 0xffffu, nbytes, kBufferFlags};
                rg = uintx4{(unsigned)ag0, (unsigned)(ag0 >> 32) & 0xffffu, nbytes, kBufferFlags};
            } else {
                rx = uintx4{0u, 0u, 0u, kBufferFlags};
                rg = rx;
            }
        } else if (pbat < B) {
            const size_t row = ((size_t)pbat * (size_t)C + (size_t)c) * (size_t)L;
            const int t0 = pseg * kSegLen;
            const int u0 = 2 * (t0 + 16 * dmin), v0 = 2 * (t0 + 16 * dmin_x);
            x_shift = u0 < 0 ? u0 : 0;
            g_shift = v0 < 0 ? v0 : 0;
            rx = row_tail_resource(x + row, L, u0 > 0 ? u0 : 0);
            rg = row_tail_resource(dy + row, L, v0 > 0 ? v0 : 0);
        } else {
            x_shift = g_shift = 0;
            rx = uintx4{0u, 0u, 0u, kBufferFlags};
            rg = rx;
        }
    };
    // ROWS: elements of the lane's granules x0 g0 x1 g1 that belong to a row which ends inside them (rows_granule8_byte_offset)
    int live_next[4] = {8, 8, 8, 8}, live_cur[4] = {8, 8, 8, 8};
    auto load_half = [&](auto hc) {         // x_h then g_h
        constexpr int h = decltype(hc)::value;
        if constexpr (ROWS) {
            // the lane's granules: elements e .. e + 7 of the windows
            buffer_load_x4_to_lds_sel(keep_lines, rx, rows_granule8_byte_offset(rm, vx0 + (off_x >> 1) + 512 * h, live_next[2 * h]),
                                  lds_x + 1024u * (unsigned)h);
            buffer_load_x4_to_lds_sel(keep_lines, rg, rows_granule8_byte_offset(rm, vg0 + (off_g >> 1) + 512 * h, live_next[2 * h + 1]),
                                  lds_g + 1024u * (unsigned)h);
        } else {
            buffer_load_x4_to_lds(rx, off_x + (1024 * h + x_shift), lds_x + 1024u * (unsigned)h);
            buffer_load_x4_to_lds(rg, off_g + (1024 * h + g_shift), lds_g + 1024u * (unsigned)h);
        }
    };
    auto tail_offset = [&](int off, int v0, int shift) {
        if constexpr (ROWS) return off == kOutOfRow ? kOutOfRow : rows_byte_offset<2>(rm, v0 + (off >> 1));
        else return off == kOutOfRow ? kOutOfRow : off + shift;
    };
    auto load_tails = [&]() {               // xt gt
        buffer_load_x1_to_lds(rx, tail_offset(off_xt, vx0, x_shift), lds_x + 2048u);
        buffer_load_x1_to_lds(rg, tail_offset(off_gt, vg0, g_shift), lds_g + 2048u);
    };

    aim(b, seg);
    load_half(std::integral_constant<int, 0>{});
    load_half(std::integral_constant<int, 1>{});
    load_tails();

    while (b < B) {
        int seg_n = seg + step_seg;
        const int carry = seg_n >= segs_per_row ? 1 : 0;
        seg_n -= carry ? segs_per_row : 0;
        const int b_n = b + step_b + carry;
        bf16_t *out_seg = ROWS ? dx + (size_t)c * (size_t)L                                                  // wave-uniform
                               : dx + ((size_t)b * (size_t)C + (size_t)c) * (size_t)L + (size_t)(seg * kSegLen);
        const bool whole = !ROWS && (seg + 1) * kSegLen <= L;
        const int t_seg = seg * kSegLen;
        aim(b_n, seg_n);
        if constexpr (ROWS) {
#pragma unroll
            for (int i = 0; i < 4; ++i) live_cur[i] = live_next[i];
        }
        // loads of this segment: x0 g0 x1 g1 xt gt.  Chunk 0 needs g0, chunks 1 and 2 need g1, chunk 3 needs gt;
        // two loads of the next segment are out after chunk 1.
        static_for<0, 4>([&](auto cc) {
            constexpr int c4 = decltype(cc)::value;
            constexpr int need = c4 == 0 ? 1 : (c4 < 3 ? 3 : 5), issued = c4 >= 2 ? 2 : 0;
            wait_vmcnt_at_most<(5 - need) + issued>();
            if constexpr (ROWS) {
                // what has just landed: x0 and g0 before chunk 0, x1 and g1 before chunk 1
                if constexpr (c4 == 0) { zero_slot_tail(sx + 8 * lane, live_cur[0]); zero_slot_tail(sg + 8 * lane, live_cur[1]); }
                if constexpr (c4 == 1) { zero_slot_tail(sx + 512 + 8 * lane, live_cur[2]); zero_slot_tail(sg + 512 + 8 * lane, live_cur[3]); }
            }
            // ---- input gradient, tile c4
            shortx4 bv[ND];
#pragma unroll
            for (int d = 0; d < ND; ++d) bv[d] = *reinterpret_cast<const shortx4 *>(gx[d] + 256 * c4);
            floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int d = 0; d < ND; ++d) acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(A[d], bv[d], acc, 0, 0, 0);
            // ---- weight gradient, chunk c4
            shortx4 bq;
#pragma unroll
            for (int v = 0; v < 4; ++v) bq[v] = gw[v][256 * c4];
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
                if constexpr (c4 == 3) load_tails();
            }
            // ---- store tile c4: lane (block j = i16, row group kg) owns outputs 16 j + 4 kg + 0..3
            const int lt = 256 * c4 + 16 * i16 + 4 * kg;
            if constexpr (ROWS) {
                int n;
                const int eo = rows_element_group(rm, t_seg + lt, n);   // four outputs: one row, one gap, or the end of a row
                if (eo >= 0) st_rows_group(out_seg + eo, make_float4(acc[0], acc[1], acc[2], acc[3]), n);
            } else {
                if (whole) st_elem4_stream(out_seg + lt, make_float4(acc[0], acc[1], acc[2], acc[3]));
                else st_elem4_stream_upto(out_seg + lt, make_float4(acc[0], acc[1], acc[2], acc[3]), t_seg + lt, L);
            }
        });
        b = b_n; seg = seg_n;
    }
    // nothing may land in LDS after this point
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    wave_lds_fence();

    // ---- per-wave diagonal sums, then the waves of the block in wave order
    dw_wave_diagonal_sums<ND>(G, s_mem[wave], s_dw[wave], lane, K, pad, dmin);
    __syncthreads();
    for (int j = tid; j < K; j += 64 * W) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) sum += s_dw[w][j];
        if (dw_out) st_elem(dw_out + (size_t)c * (size_t)K + (size_t)j, sum);
        else part[((size_t)blockIdx.y * (size_t)C + (size_t)c) * (size_t)K + (size_t)j] = sum;
    }
}

}  // namespace dwconv
