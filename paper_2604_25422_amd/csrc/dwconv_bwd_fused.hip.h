// Fused backward pass, fp32 storage: input gradient (adjoint of Sec. IV-A eq. (dwconv), cf. eq. (dx_def)) and
// stage 1 of the weight gradient (eq. (dk_def)) in one pass that reads dY once.  The paper names kernel fusion
// as the remaining lever for the backward path (Sec. VI); separately the two calls read dY twice.
//
// Both halves are the blocked-Toeplitz contractions of dwconv_mfma.hip.h on v_mfma_f32_16x16x4_f32:
//     dX:  D[r][n]     += Toep'_d[r][4k+v] * dY[n + dmin' + d][4k+v]       (reversed filter, pad' = K-1-pad)
//     dW:  G_d[q'][q]  += X[n + dmin + d][q'] * dY[n][q]                  (contraction over 16-blocks n)
// with the same number ND of block offsets for both (dmin' = -dmax, dmax' = -dmin).
//
// A wave owns one channel for its whole life (grid (C, S), W waves per block, as in the weight-gradient
// kernels) and walks 1024-position segments.  Its private LDS region holds the x window [t0 + 16 dmin, + 1024 +
// 16 ND) in plain order and the dY window [t0 + 16 dmin', + 1024 + 16 ND) with the four 16-byte granules of every
// 16-block permuted (granule g of block nb sits at g ^ ((nb >> 1) & 3)): that keeps the strided 16-byte reads of
// the dX operand conflict-free, and the 4-byte reads of the dW operand, which cover whole blocks, do not care.
// Rows come from memory straight into LDS (buffer loads with the LDS bit; the permutation is applied on the
// memory side, each lane fetching the granule that belongs in its LDS slot; zeros outside the row come from the
// hardware range check).
//
// A segment is processed in four quarters.  Quarter i: dX tile i (256 outputs), then dW chunks 4i..4i+3; after
// it, floats [256 i, 256 i + 256) of both windows are dead and are refilled in place for the NEXT segment (the
// tails beyond float 1024 after quarter 3).  Loads of a segment in issue order: x0 g0 x1 g1 x2 g2 x3 g3, then
// four 4-byte-per-lane tail loads xa xb ga gb.  Quarter i reads at most 16 (ND-1) + 63 floats into region i + 1,
// so before quarter i everything up to g_{i+1} (all twelve before quarter 3) must have landed; the vector-memory
// counter retires in order, which turns that into one constant s_waitcnt per quarter.
#pragma once
#include "dwconv_dw_direct.hip.h"

namespace dwconv {

// One 4-byte-per-lane load into LDS: LDS[lds_base + 4 lane] <- resource[byte_off], zero outside the resource.
__device__ __forceinline__ void buffer_load_x1_to_lds(uintx4 rsrc, int byte_off, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen nt lds"
                 :: "s"(lds_base), "v"(byte_off), "s"(rsrc) : "memory");
}

constexpr int kFusedWin = kSegLen + 128;      // floats per staged window: 1024 + tail of two 64-float loads
constexpr int bwd_fused_wave_floats(int ND)
{
    const int stage = 2 * kFusedWin, diag = ((16 * ND + 15) * 17 + 3) / 4 * 4;
    return stage > diag ? stage : diag;
}
constexpr size_t bwd_fused_lds_bytes(int ND, int W) { return (size_t)W * (size_t)(bwd_fused_wave_floats(ND) + 16 * ND) * sizeof(float); }

// Position of logical float f of the dY window in LDS (granules permuted inside every 16-block).
__device__ __forceinline__ constexpr int swz_pos(int f)
{
    const int nb = f >> 4, g = (f >> 2) & 3, e = f & 3;
    return 16 * nb + 4 * (g ^ ((nb >> 1) & 3)) + e;
}

// ROWS: short rows, the wave walks the virtual row of its channel (see RowsMap); B is then 1 and segs_per_row the
// number of segments of the virtual row.
template <int ND, int W, bool ROWS>
__global__ __launch_bounds__(64 * W, kMfmaWavesPerSimd) void bwd_fused_kernel(
    const float *__restrict__ dy, const float *__restrict__ x, const float *__restrict__ f, float *__restrict__ dx,
    float *__restrict__ part, float *__restrict__ dw_out, int B, int C, int L, int K, int pad, int dmin,
    int segs_per_row, const RowsMap rm)
{
    static_assert(ND >= 2 && 16 * ND <= 128, "window tails are two 64-float loads");
    constexpr int XW = kSegLen + 16 * ND;          // floats of either window that are ever read
    constexpr int WREG = bwd_fused_wave_floats(ND);
    extern __shared__ __align__(16) float dyn_lds[];
    float (*s_mem)[WREG] = reinterpret_cast<float (*)[WREG]>(dyn_lds);
    float (*s_dw)[16 * ND] = reinterpret_cast<float (*)[16 * ND]>(dyn_lds + W * WREG);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i16 = lane & 15, k4 = lane >> 4;
    const int c = blockIdx.x;
    const int stride = (int)gridDim.y * W;
    const int ws = (int)blockIdx.y * W + __builtin_amdgcn_readfirstlane(wave);
    const int step_b = stride / segs_per_row, step_seg = stride % segs_per_row;
    int b = ws / segs_per_row, seg = ws % segs_per_row;

    const int pad_x = K - 1 - pad;                 // pad of the input-gradient correlation
    const int dmin_x = -((pad_x + 15) / 16);       // its first block offset (= -dmax of the weight gradient)
    float *sx = s_mem[wave];                       // sx[i] = x~[t0 + 16 dmin + i]
    float *sg = s_mem[wave] + kFusedWin;           // sg[swz_pos(i)] = dy~[t0 + 16 dmin_x + i]
    const unsigned lds_x = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) void *)sx);
    const unsigned lds_g = lds_x + 4u * kFusedWin;

    // ---- loop constants
    // Toeplitz operands of the input gradient: A[d][v] (lane (r, k)) = w[c, K-1-j], j = 16 (dmin_x + d) + 4k + v - r + pad_x
    float A[ND][4];
    {
        const float *f_c = f + (size_t)c * (size_t)K;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int j = 16 * (dmin_x + d) + 4 * k4 + v - i16 + pad_x;
                const bool ok = j >= 0 && j < K;
                const float a = f_c[ok ? (K - 1 - j) : 0];
                A[d][v] = ok ? a : 0.f;
            }
    }
    // LDS read addresses.  dX operand: granule k4 of window block 16 dt + i16 + d  (dt in the immediate offset)
    const float *gx[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) gx[d] = sg + 16 * (i16 + d) + 4 * (k4 ^ (((i16 + d) >> 1) & 3));
    // dW operand from dY: logical float 64 ch + lane - 16 dmin_x of the window; the permutation depends on ch & 1
    const float *gw[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) gw[h] = sg + swz_pos(64 * h + lane - 16 * dmin_x) - 64 * h;
    const float *xw = sx + lane;
    // offsets of the loads inside the windows (memory side), in floats
    const int fo_x = 4 * lane;                                                          // plain granule order
    const int fo_g = 4 * (4 * (lane >> 2) + ((lane & 3) ^ ((lane >> 3) & 3)));          // granule that belongs in slot `lane`
    int fo_xt[2], fo_gt[2];     // tails: the logical float that belongs in LDS float slot 1024 + 64 h + lane (-1: none)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int slot = kSegLen + 64 * h + lane;
        fo_xt[h] = slot < XW ? slot : -1;
        const int nb = slot >> 4, gp = (slot >> 2) & 3, e = slot & 3;
        const int fg = 16 * nb + 4 * (gp ^ ((nb >> 1) & 3)) + e;
        fo_gt[h] = fg < XW ? fg : -1;
    }

    floatx4 G[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) G[d] = floatx4{0.f, 0.f, 0.f, 0.f};

    // resources of the segment the next loads belong to (wave-uniform); empty past the last segment
    uintx4 rx, rg;
    int x_shift, g_shift;       // negative when a window starts before the row: added to the lane offsets
    int vx0 = 0, vg0 = 0;       // ROWS: virtual positions of the first floats of the two windows
    auto aim = [&](int pb, int pseg) {
        if (pb < B) {
            const int t0 = pseg * kSegLen;
            if constexpr (ROWS) {
                vx0 = t0 + 16 * dmin;
                vg0 = t0 + 16 * dmin_x;
                x_shift = g_shift = 0;
                const unsigned nbytes = rm.bytes - (unsigned)(c * L) * 4u;
                const unsigned long long ax = reinterpret_cast<unsigned long long>(x + (size_t)c * (size_t)L);
                const unsigned long long ag = reinterpret_cast<unsigned long long>(dy + (size_t)c * (size_t)L);
                rx = uintx4{(unsigned)ax, (unsigned)(ax >> 32) & 0xffffu, nbytes, kBufferFlags};
                rg = uintx4{(unsigned)ag, (unsigned)(ag >> 32) & 0xffffu, nbytes, kBufferFlags};
            } else {
                const size_t row = ((size_t)pb * (size_t)C + (size_t)c) * (size_t)L;
                const int u0 = 4 * (t0 + 16 * dmin), v0 = 4 * (t0 + 16 * dmin_x);
                x_shift = u0 < 0 ? u0 : 0;
                g_shift = v0 < 0 ? v0 : 0;
                rx = row_tail_resource(x + row, L, u0 > 0 ? u0 : 0);
                rg = row_tail_resource(dy + row, L, v0 > 0 ? v0 : 0);
            }
        } else {
            x_shift = g_shift = 0;
            rx = uintx4{0u, 0u, 0u, kBufferFlags};
            rg = rx;
        }
    };
    // ROWS: floats of the lane's granules x0 g0 x1 g1 x2 g2 x3 g3 that belong to a row which ends inside them
    // (rows_granule4_byte_offset; rows whose length is not a multiple of four)
    // (three bits per load, packed: the kernel has no registers to spare)
    const bool rag = ROWS && (rm.L & 3) != 0;
    unsigned live_next = 0u, live_cur = 0u;
    auto note_live = [&](int k, int live) { live_next |= (unsigned)live << (3 * k); };
    auto live_of = [&](int k) { return (int)((live_cur >> (3 * k)) & 7u); };
    auto load_region = [&](auto ic) {       // x_i then g_i, i = 0..3
        constexpr int i = decltype(ic)::value;
        if constexpr (ROWS) {
            int lx, lg;
            const int ox = rows_granule4_byte_offset(rm, vx0 + fo_x + 256 * i, lx), og = rows_granule4_byte_offset(rm, vg0 + fo_g + 256 * i, lg);
            note_live(2 * i, lx); note_live(2 * i + 1, lg);
            buffer_load_x4_to_lds(rx, ox, lds_x + 1024u * (unsigned)i);
            buffer_load_x4_to_lds(rg, og, lds_g + 1024u * (unsigned)i);
        } else {
            buffer_load_x4_to_lds(rx, 4 * fo_x + (1024 * i + x_shift), lds_x + 1024u * (unsigned)i);
            buffer_load_x4_to_lds(rg, 4 * fo_g + (1024 * i + g_shift), lds_g + 1024u * (unsigned)i);
        }
    };
    auto tail_offset = [&](int fo, int v0, int shift) {
        if constexpr (ROWS) return fo >= 0 ? rows_byte_offset<4>(rm, v0 + fo) : kOutOfRow;
        else return fo >= 0 ? 4 * fo + shift : kOutOfRow;
    };
    auto load_tails = [&]() {               // xa xb ga gb
        buffer_load_x1_to_lds(rx, tail_offset(fo_xt[0], vx0, x_shift), lds_x + 4096u);
        buffer_load_x1_to_lds(rx, tail_offset(fo_xt[1], vx0, x_shift), lds_x + 4096u + 256u);
        buffer_load_x1_to_lds(rg, tail_offset(fo_gt[0], vg0, g_shift), lds_g + 4096u);
        buffer_load_x1_to_lds(rg, tail_offset(fo_gt[1], vg0, g_shift), lds_g + 4096u + 256u);
    };

    aim(b, seg);
    static_for<0, 4>([&](auto ic) { load_region(ic); });
    load_tails();

    while (b < B) {
        int seg_n = seg + step_seg;
        const int carry = seg_n >= segs_per_row ? 1 : 0;
        seg_n -= carry ? segs_per_row : 0;
        const int b_n = b + step_b + carry;
        // where this segment's input gradient goes (wave-uniform)
        float *out_seg = ROWS ? dx + (size_t)c * (size_t)L
                              : dx + ((size_t)b * (size_t)C + (size_t)c) * (size_t)L + (size_t)(seg * kSegLen);
        const bool whole = !ROWS && (seg + 1) * kSegLen <= L;
        const int t_seg = seg * kSegLen;
        aim(b_n, seg_n);
        if constexpr (ROWS) { live_cur = live_next; live_next = 0u; }

        static_for<0, 4>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            // twelve loads per segment; before quarter i everything up to g_{i+1} (i < 3) or all of them has landed
            constexpr int need = i < 3 ? 2 * i + 3 : 11;
            wait_vmcnt_at_most<(11 - need) + 2 * i>();
            if constexpr (ROWS) {
                // what has just landed: x0 g0 x1 g1 before quarter 0, x2 g2 before quarter 1, x3 g3 before quarter 2
                if (rag && i == 0) {
                    zero_slot_tail(sx + 4 * lane, live_of(0)); zero_slot_tail(sg + 4 * lane, live_of(1));
                    zero_slot_tail(sx + 256 + 4 * lane, live_of(2)); zero_slot_tail(sg + 256 + 4 * lane, live_of(3));
                }
                if (rag && (i == 1 || i == 2)) {
                    zero_slot_tail(sx + 256 * (i + 1) + 4 * lane, live_of(2 * (i + 1)));
                    zero_slot_tail(sg + 256 * (i + 1) + 4 * lane, live_of(2 * (i + 1) + 1));
                }
            }

            // ---- input gradient, tile i: one chain of 4 ND matrix instructions
            float4 bv[ND];
#pragma unroll
            for (int d = 0; d < ND; ++d) bv[d] = *reinterpret_cast<const float4 *>(gx[d] + 256 * i);
            floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int d = 0; d < ND; ++d) {
                acc = mfma16x16x4(A[d][0], bv[d].x, acc);
                acc = mfma16x16x4(A[d][1], bv[d].y, acc);
                acc = mfma16x16x4(A[d][2], bv[d].z, acc);
                acc = mfma16x16x4(A[d][3], bv[d].w, acc);
            }
            // ---- weight gradient, chunks 4i .. 4i+3
            float gr[4], xr[4][ND];
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const int ch = 4 * i + cc;
                gr[cc] = gw[ch & 1][64 * ch];
#pragma unroll
                for (int d = 0; d < ND; ++d) xr[cc][d] = xw[64 * ch + 16 * d];
            }
#pragma unroll
            for (int cc = 0; cc < 4; ++cc)
#pragma unroll
                for (int d = 0; d < ND; ++d) G[d] = mfma16x16x4(xr[cc][d], gr[cc], G[d]);
            // ---- regions i of both windows are dead: refill them for the next segment
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            load_region(ic);
            if constexpr (i == 3) load_tails();
            // ---- store tile i: lane (block j = i16, row group k4) owns outputs 16 j + 4 k4 + 0..3
            const int lt = 256 * i + 16 * i16 + 4 * k4;
            if constexpr (ROWS) {
                int n;
                const int e = rows_element_group(rm, t_seg + lt, n);    // four outputs: one row, one gap, or the end of a row
                if (e >= 0) st_rows_group(out_seg + e, make_float4(acc[0], acc[1], acc[2], acc[3]), n);
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
        if (dw_out) dw_out[(size_t)c * (size_t)K + (size_t)j] = sum;
        else part[((size_t)blockIdx.y * (size_t)C + (size_t)c) * (size_t)K + (size_t)j] = sum;
    }
}

}  // namespace dwconv
