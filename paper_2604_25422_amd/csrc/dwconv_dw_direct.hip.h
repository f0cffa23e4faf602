// Stage 1 of the weight gradient (Sec. IV-A eq. (dk_def)) on the matrix cores, fp32 storage, with
// the operands brought from memory straight into LDS.
//
// Same contraction, same walk and same three ordered reduction levels as dw_partial_mfma_kernel
// (G_d[q'][q] += X[n+d][q'] dY[n][q] over 16-blocks n; diagonal sums per wave; waves in wave order;
// slices in slice order).  What differs is how a segment reaches LDS: buffer loads with the LDS
// bit write 16 bytes per lane into consecutive LDS slots, so the x window and the dY tile of the
// next segment are never held in registers, nothing is copied or masked by the vector ALU (which
// shares its issue slots with the matrix instructions on this part), and the zero padding of the
// operator is the hardware range check writing zeros.
//
// A wave refills its private LDS region in place while it contracts out of it.  The loads of a
// segment are, in issue order,  x0 g0 x1 g1 x2 g2 x3 g3 x4  (x_i: floats [256 i, 256 i + 256) of
// the x window, g_i: the same of the dY tile; x4 is the partial tail plus zeros into a slack
// area).  Region i is last read by 64-position chunk 4 i + 3, so x_i and g_i of the NEXT segment
// are issued right after that chunk; the vector-memory counter retires in order, so "load number s
// of this segment has landed" is  vmcnt <= (8 - s) + (loads of the next segment issued so far),
// a compile-time constant at every point of the unrolled chunk loop.  A wave past its last segment
// keeps issuing the same loads against an empty resource (zeros, no memory traffic) so that the
// counts hold.
#pragma once
#include <type_traits>

#include "dwconv_mfma.hip.h"

namespace dwconv {

// One 16-byte-per-lane load into LDS:  LDS[lds_base + 16 lane ..] <- resource[byte_off ..], zeros when
// byte_off is outside the resource.  M0 carries the LDS base of the instruction.  The loads carry the
// non-temporal hint: the kernels that use them are the last readers of x and dY in a training step, and lines
// that are not kept do not push out the rows still waiting in the last-level cache (measured: -8 % on the
// short-filter weight gradient, -11 % on its fused backward, neutral on the headline shape).
__device__ __forceinline__ void buffer_load_x4_to_lds(uintx4 rsrc, int byte_off, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen nt lds"
                 :: "s"(lds_base), "v"(byte_off), "s"(rsrc) : "memory");
}
template <int OFF>
__device__ __forceinline__ void buffer_load_x4_to_lds_imm(uintx4 rsrc, int byte_off, unsigned lds_base)
{
    // the immediate offset advances the memory side and the LDS side alike
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen offset:%3 nt lds"
                 :: "s"(lds_base), "v"(byte_off), "s"(rsrc), "n"(OFF) : "memory");
}
// The same loads without the non-temporal hint: the forward / input-gradient kernels (the weight-gradient call of the
// same step reads their rows again), and the weight-gradient and fused kernels on short rows that are not whole
// 128-byte cache lines, where the line in which one row ends and the next channel's row begins has a second reader
// behind the same L2 (see die_run_channel).
__device__ __forceinline__ void buffer_load_x4_to_lds_keep(uintx4 rsrc, int byte_off, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_base), "v"(byte_off), "s"(rsrc) : "memory");
}
__device__ __forceinline__ void buffer_load_x1_to_lds_keep(uintx4 rsrc, int byte_off, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :: "s"(lds_base), "v"(byte_off), "s"(rsrc) : "memory");
}
// One or the other (keep is wave-uniform): either way one load, so the wait counts do not depend on it.
__device__ __forceinline__ void buffer_load_x4_to_lds_sel(bool keep, uintx4 rsrc, int byte_off, unsigned lds_base)
{
    if (keep) buffer_load_x4_to_lds_keep(rsrc, byte_off, lds_base);
    else buffer_load_x4_to_lds(rsrc, byte_off, lds_base);
}
// s_waitcnt vmcnt(N)
template <int N>
__device__ __forceinline__ void wait_vmcnt_at_most()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// Compile-time loop: f(std::integral_constant<int, I>) for I = BEGIN .. END-1.  The chunk loop below must
// be unrolled with every index a constant (register arrays, wait counts), which a pragma does not guarantee.
template <int BEGIN, int END, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (BEGIN < END) {
        f(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(f);
    }
}

// Bookkeeping of the nine loads of a segment (issue order x0 g0 x1 g1 x2 g2 x3 g3 x4) against the reads of
// the chunk loop.  Ring read n = ch * ND + d of the x window touches floats [64 ch + 16 d, + 64).
template <int ND>
struct DirectSchedule {
    static constexpr int NCH = kSegLen / 64;
    static constexpr int NQ = NCH * ND;
    static constexpr int PFX = 6, PFG = 2;
    static constexpr int cmax(int a, int b) { return a > b ? a : b; }
    static constexpr int cmin(int a, int b) { return a < b ? a : b; }
    static constexpr int need_x(int n)      // load (in issue order) that x read n needs
    {
        const int i = (64 * (n / ND) + 16 * (n % ND) + 63) / 256;
        return i < 4 ? 2 * i : 8;
    }
    static constexpr int need_g(int ch) { return 2 * (ch / 4) + 1; }
    // loads of the next segment issued before the reads of step q (two after every fourth chunk)
    static constexpr int issued(int q) { return 2 * (q / (4 * ND)); }
    // highest load known landed before the x read of step q (reads before it: x reads up to q + PFX - 1,
    // dY reads up to chunk q / ND + PFG - 1)
    static constexpr int landed_before_x(int q)
    {
        return cmax(need_x(cmin(q + PFX - 1, NQ - 1)), need_g(cmin(q / ND + PFG - 1, NCH - 1)));
    }
    static constexpr int landed_before_g(int q)   // only asked at the last step of a chunk
    {
        return cmax(need_x(cmin(q + PFX, NQ - 1)), need_g(cmin(q / ND + PFG - 1, NCH - 1)));
    }
};

constexpr int kDirectSlackFloats = 256;   // x4 writes a full 1 KiB: the tail of the window, then zeros

// Per-wave LDS region (floats) and dynamic LDS bytes of a block of W waves.
constexpr int dw_direct_wave_floats(int ND)
{
    const int stage = 5 * 256 + kSegLen, gf = ND * 256, diag = ((16 * ND + 15) * 17 + 3) / 4 * 4;
    return stage > gf ? (stage > diag ? stage : diag) : (gf > diag ? gf : diag);
}
// Taps a wave hands to the block-level sum: all of them fit 16 ND when the offsets cover the whole filter; a launch over
// part of the offsets (nine and more, see the j0 / j1 arguments of the kernel) owns up to 16 ND + 15 taps.
constexpr int dw_direct_row_floats(int ND) { return 16 * ND + (ND >= 9 ? 16 : 0); }
constexpr size_t dw_direct_lds_bytes(int ND, int W) { return (size_t)W * (size_t)(dw_direct_wave_floats(ND) + dw_direct_row_floats(ND)) * sizeof(float); }

// W waves per block.  dw_out == nullptr: the block's sums go to slice blockIdx.y of part; otherwise (one
// block per channel, gridDim.y == 1) they are the weight gradient itself and go to dw_out.
// ROWS: short rows, the wave walks the virtual row of its channel (see RowsMap); B is then 1 and segs_per_row the
// number of segments of the virtual row.
// [j0, j1): the taps this launch owns, at most dw_direct_row_floats(ND) of them (0, K unless the block offsets of the
// filter are split over several launches); the other taps of its slices are written as zeros, or, with own_only set,
// left alone (filters with hundreds of block offsets: dozens of launches share two zero-filled sets of slices).
// seg0: the first 1024-position segment of every row this launch walks (segs_per_row of them): a launch over offsets
// far from lag 0 skips the segments whose x window lies outside the row.
template <int ND, int W, bool ROWS>
__global__ __launch_bounds__(64 * W, kMfmaWavesPerSimd) void dw_partial_direct_kernel(
    const float *__restrict__ x, const float *__restrict__ dy, float *__restrict__ part, float *__restrict__ dw_out,
    int B, int C, int L, int K, int pad, int dmin, int segs_per_row, const RowsMap rm, int j0, int j1, int seg0,
    int own_only)
{
    constexpr int XW = kSegLen + 16 * ND;          // staged x window (floats)
    constexpr int NGX = XW / 4;                    // its 16-byte granules: 4 full loads and a tail
    static_assert(NGX > 256 && NGX <= 320, "five loads per x window");
    constexpr int XREG = 5 * 256;                  // x window plus slack for the tail load
    static_assert(XREG - XW <= kDirectSlackFloats, "slack");
    constexpr int GF = ND * 256;                   // floats of one wave's G
    constexpr int STAGE = XREG + kSegLen;
    constexpr int WREG = dw_direct_wave_floats(ND);   // per-wave LDS region: the staged windows, or the epilogue's images
    static_assert(WREG >= STAGE && WREG >= GF, "the staged windows fit the wave's region");
    extern __shared__ __align__(16) float dyn_lds[];
    float (*s_mem)[WREG] = reinterpret_cast<float (*)[WREG]>(dyn_lds);
    constexpr int ROWF = dw_direct_row_floats(ND);
    float (*s_dw)[ROWF] = reinterpret_cast<float (*)[ROWF]>(dyn_lds + W * WREG);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int c = blockIdx.x;
    const int stride = (int)gridDim.y * W;
    const int ws = (int)blockIdx.y * W + __builtin_amdgcn_readfirstlane(wave);
    const int step_b = stride / segs_per_row, step_seg = stride % segs_per_row;
    int b = ws / segs_per_row, seg = ws % segs_per_row;
    float *sx = s_mem[wave];            // sx[i] = x~[t0 + 16 dmin + i]
    float *sg = s_mem[wave] + XREG;     // sg[i] = dy[t0 + i]
    const unsigned lds_x = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) void *)sx);
    const unsigned lds_g = lds_x + 4u * XREG;

    floatx4 G[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) G[d] = floatx4{0.f, 0.f, 0.f, 0.f};

    // per-lane byte offsets inside the staged windows (loop constants)
    const int off_lane = 16 * lane;
    const int off_tail = (lane + 256 < NGX) ? 16 * (lane + 256) : kOutOfRow;

    // resources of the segment the next loads belong to (wave-uniform); empty past the last segment
    uintx4 rx, rg;
    int x_shift;        // negative when the x window starts before the row: added to the lane offsets
    int vx0 = 0, vg0 = 0;   // ROWS: virtual positions of the first floats of the two windows
    auto aim = [&](int pb, int pseg) {
        if (pb < B) {
            if constexpr (ROWS) {
                // (virtual segments are walked downwards, like the batches below)
                const int t0 = (segs_per_row - 1 - pseg) * kSegLen;
                vx0 = t0 + 16 * dmin;
                vg0 = t0;
                x_shift = 0;
                const unsigned nbytes = rm.bytes - (unsigned)(c * L) * 4u;
                rx = uintx4{0u, 0u, nbytes, kBufferFlags};
                rg = rx;
                const unsigned long long ax = reinterpret_cast<unsigned long long>(x + (size_t)c * (size_t)L);
                const unsigned long long ag = reinterpret_cast<unsigned long long>(dy + (size_t)c * (size_t)L);
                rx[0] = (unsigned)ax; rx[1] = (unsigned)(ax >> 32) & 0xffffu;
                rg[0] = (unsigned)ag; rg[1] = (unsigned)(ag >> 32) & 0xffffu;
            } else {
                // batches are walked from the last to the first: the input-gradient call that usually runs just
                // before this one walks them upwards, so its last rows of dY are still in the last-level cache
                const size_t row = ((size_t)(B - 1 - pb) * (size_t)C + (size_t)c) * (size_t)L;
                const int t0 = (seg0 + pseg) * kSegLen;
                const int u0 = 4 * (t0 + 16 * dmin);
                x_shift = u0 < 0 ? u0 : 0;
                // (a window that starts past the end of the row - possible when dmin > 0, the second of two passes
                // over the block offsets - gets an empty resource: every load returns zero)
                rx = row_tail_resource(x + row, L, u0 > 0 ? min(u0, 4 * L) : 0);
                rg = row_tail_resource(dy + row, L, 4 * t0);
            }
        } else {
            x_shift = 0;
            rx = uintx4{0u, 0u, 0u, kBufferFlags};
            rg = rx;
        }
    };
    // (no immediate offsets on the x side: a window that starts before the row has negative lane offsets,
    // and the chunk loop stays one straight-line block without a second code path)
    // ROWS, rows whose length is not a multiple of four (rag): floats of the lane's granules x0 .. x4 (fields 0 .. 4) and
    // g0 .. g3 (fields 5 .. 8) that belong to a row which ends inside them (rows_granule4_byte_offset), three bits per load
    const bool rag = ROWS && (rm.L & 3) != 0;
    unsigned live_next = 0u, live_cur = 0u;
    auto load_x = [&](auto ic) {        // ic = 0..4
        constexpr int i = decltype(ic)::value;
        if constexpr (ROWS) {
            int live = 4;
            const int off = (i < 4 || lane + 256 < NGX) ? rows_granule4_byte_offset(rm, vx0 + 4 * (lane + 64 * i), live) : kOutOfRow;
            live_next |= (unsigned)live << (3 * i);
            buffer_load_x4_to_lds(rx, off, lds_x + 1024u * (unsigned)i);
        } else {
            if constexpr (i < 4) buffer_load_x4_to_lds(rx, off_lane + (1024 * i + x_shift), lds_x + 1024u * (unsigned)i);
            else buffer_load_x4_to_lds(rx, off_tail + x_shift, lds_x + 4096u);
        }
    };
    auto load_g = [&](auto ic) {        // ic = 0..3
        constexpr int i = decltype(ic)::value;
        if constexpr (ROWS) {
            int live;
            const int off = rows_granule4_byte_offset(rm, vg0 + 4 * (lane + 64 * i), live);
            live_next |= (unsigned)live << (3 * (5 + i));
            buffer_load_x4_to_lds(rg, off, lds_g + 1024u * (unsigned)i);
        } else {
            buffer_load_x4_to_lds_imm<1024 * i>(rg, off_lane, lds_g);
        }
    };

    // first segment: all nine loads, in the order every later segment uses
    aim(b, seg);
    static_for<0, 4>([&](auto ic) { load_x(ic); load_g(ic); });
    load_x(std::integral_constant<int, 4>{});

    typedef DirectSchedule<ND> Sch;
    constexpr int NQ = Sch::NQ, PFX = Sch::PFX, PFG = Sch::PFG;
    while (b < B) {
        // the segment after this one
        int seg_n = seg + step_seg;
        const int carry = seg_n >= segs_per_row ? 1 : 0;
        seg_n -= carry ? segs_per_row : 0;
        const int b_n = b + step_b + carry;
        aim(b_n, seg_n);
        if constexpr (!ROWS && ND <= 6) {
            // (up to six block offsets: beyond, this second body costs the kernel registers it does not have)
            // A last segment that holds at most 768 positions of its row (rows that are not whole segments): dY is zero
            // beyond them, so only the first 4 lr chunks can add anything, lr = 1..3 the 256-position regions that hold
            // positions of the row; they need the loads up to x_lr (x0 g0 x1 g1 ... in issue order, the nine loads of this
            // segment being the last nine issued).  Then all nine loads of the next segment go out in the usual order.
            const int left = L - (seg0 + seg) * kSegLen;
            if (left <= 3 * 256) {
                const int lr = left <= 256 ? 1 : (left <= 512 ? 2 : 3);
                if (lr == 1) wait_vmcnt_at_most<6>();
                else if (lr == 2) wait_vmcnt_at_most<4>();
                else wait_vmcnt_at_most<2>();
#pragma unroll 1
                for (int ch = 0; ch < 4 * lr; ++ch) {
                    const float gv = sg[64 * ch + lane];
                    float xv[ND];
#pragma unroll
                    for (int d = 0; d < ND; ++d) xv[d] = sx[64 * ch + 16 * d + lane];
#pragma unroll
                    for (int d = 0; d < ND; ++d) G[d] = mfma16x16x4(xv[d], gv, G[d]);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                static_for<0, 4>([&](auto ic) { load_x(ic); load_g(ic); });
                load_x(std::integral_constant<int, 4>{});
                b = b_n; seg = seg_n;
                continue;
            }
        }
        if constexpr (ROWS) {
            live_cur = live_next; live_next = 0u;
            if (rag) {
                // rows that end inside a granule: all nine loads of this segment have to land before the elements of the
                // next row they brought along are cleared (the waits below then find nothing left to wait for)
                wait_vmcnt_at_most<0>();
#pragma unroll
                for (int i = 0; i < 5; ++i) zero_slot_tail(sx + 256 * i + 4 * lane, (int)((live_cur >> (3 * i)) & 7u));
#pragma unroll
                for (int i = 0; i < 4; ++i) zero_slot_tail(sg + 256 * i + 4 * lane, (int)((live_cur >> (3 * (5 + i))) & 7u));
            }
        }
        // 64-position chunk ch, block offset d:  G_d += X[n0 + k + dmin + d][q'] * dY[n0 + k][q]
        //   A operand sx[64 ch + 16 d + lane],  B operand sg[64 ch + lane].
        // LDS reads run ahead of the matrix instructions in two small rings.
        float xr[PFX], gr[PFG];
        wait_vmcnt_at_most<8 - Sch::need_g(PFG - 1)>();          // x0 and g0 have landed
        static_assert(Sch::need_x(PFX - 1) <= Sch::need_g(PFG - 1), "the first reads stay inside x0, g0");
        static_for<0, PFG>([&](auto cc) { constexpr int ch = decltype(cc)::value; gr[ch] = sg[64 * ch + lane]; });
        static_for<0, PFX>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            xr[q] = sx[64 * (q / ND) + 16 * (q % ND) + lane];
        });
        static_for<0, NQ>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            constexpr int ch = q / ND, d = q % ND;
            G[d] = mfma16x16x4(xr[q % PFX], gr[ch % PFG], G[d]);
            if constexpr (q + PFX < NQ) {
                constexpr int n = q + PFX;
                if constexpr (Sch::need_x(n) > Sch::landed_before_x(q))
                    wait_vmcnt_at_most<8 - Sch::need_x(n) + Sch::issued(q)>();
                xr[q % PFX] = sx[64 * (n / ND) + 16 * (n % ND) + lane];
            }
            if constexpr (d == ND - 1 && ch + PFG < Sch::NCH) {
                if constexpr (Sch::need_g(ch + PFG) > Sch::landed_before_g(q))
                    wait_vmcnt_at_most<8 - Sch::need_g(ch + PFG) + Sch::issued(q)>();
                gr[ch % PFG] = sg[64 * (ch + PFG) + lane];
            }
            if constexpr (d == ND - 1 && ch % 4 == 3) {
                // regions ch/4 of both windows have been read for the last time: refill them for the next
                // segment once every LDS read issued so far has returned
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                load_x(std::integral_constant<int, ch / 4>{});
                load_g(std::integral_constant<int, ch / 4>{});
                if constexpr (ch == Sch::NCH - 1) load_x(std::integral_constant<int, 4>{});
            }
        });
        // pin the interleaving: the first reads, then (1 matrix instruction, its ring refills) per step
        static_for<0, PFX + PFG>([&](auto) { __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); });
        static_for<0, NQ>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if constexpr (q + PFX < NQ) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if constexpr (q % ND == ND - 1 && q / ND + PFG < Sch::NCH) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        });
        b = b_n; seg = seg_n;
    }
    // nothing may land in LDS after this point
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    wave_lds_fence();

    // ---- per-wave diagonal sums, then the waves of the block in wave order
    static_assert(WREG >= ((16 * ND + 15) * 17 + 3) / 4 * 4, "diagonal image fits the wave's region");
    dw_wave_diagonal_sums<ND>(G, s_mem[wave], s_dw[wave], lane, j0, j1, pad, dmin);
    __syncthreads();
    for (int j = own_only ? j0 + tid : tid; j < (own_only ? j1 : K); j += 64 * W) {
        float sum = 0.f;
        if (j >= j0 && j < j1) {
#pragma unroll
            for (int w = 0; w < W; ++w) sum += s_dw[w][j - j0];
        }
        if (dw_out) dw_out[(size_t)c * (size_t)K + (size_t)j] = sum;
        else part[((size_t)blockIdx.y * (size_t)C + (size_t)c) * (size_t)K + (size_t)j] = sum;
    }
}

}  // namespace dwconv
