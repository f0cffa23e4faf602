// Rows of 129 to 512 positions with filters of the order of the row length, sixteen rows at a time (fp32, or bf16
// storage widened to fp32 on the way into LDS).  Rows need to start on a dword only (bf16: even L): a last granule of
// four that holds elements of the next row gets zeros in their place on the way into LDS, and the last group of
// outputs of such a row is stored by element (see dwconv_rowbatch.hip.h).
//
// The sixteen-row formulation of dwconv_rowbatch.hip.h (Sec. IV-A eqs. (dwconv), (dk_def): the sixteen columns of a
// matrix tile are sixteen ROWS (b, c) of one channel at the same block position, and only block pairs inside the row
// are contracted) for rows of m = 9 .. 32 blocks, where neither the Toeplitz operands of up to 2 m - 1 block offsets
// nor the accumulators of all output blocks fit the registers:
//   forward / input gradient:  the filter window of the channel sits in LDS beside the image of the unit, the
//       operands of offset d are four 4-byte reads of it; one output block at a time is accumulated over its in-row
//       input blocks and stored straight from the accumulator layout;
//   weight gradient:  the accumulators are indexed by the relative block offset, fifteen per launch window (grid z);
//       every window walks the batch on its own and owns the taps its offsets reach, its slices hold zeros elsewhere,
//       and stage 2 adds the slices of all windows.
// Units are loaded without prefetch across the contraction (a few granules per lane at a time, waited for at once); two
// or three workgroups per compute unit, where LDS allows, hide the load of one behind the matrix work of another.
#pragma once
#include "dwconv_rowbatch.hip.h"

namespace dwconv {

constexpr int kRtMinBlocks = 9;        // rows of fewer blocks take the kernels of dwconv_rowbatch.hip.h
constexpr int kRtMaxBlocks = 32;       // rows of at most 512 positions
constexpr int kRtWaves = 4;            // waves per workgroup, each with a unit of its own
constexpr int kRtWindow = 15;          // relative block offsets per weight-gradient window

struct RowTallGeom {
    int B, C, L, K;
    int pad;            // effective pad of this correlation (weight gradient: the forward pad)
    int reverse;        // filter index reversed (input gradient)
    int dmin, dmax;     // block offsets inside a row (cropped to -(m-1) .. m-1)
    int m;              // 16-blocks per row
    int n_units;        // correlate: ceil(B / 16); weight gradient: ceil(B / 4)
    int J;              // correlate: waves per channel, wave (c, j) walks units j, j + J, ...
    int win;            // weight gradient: relative block offsets per window (at most kRtWindow; the windows are of equal size)
    unsigned lg_recip;  // floor(2^32 / ceil(L / 4)) + 1: granule index -> (row of the unit, granule of the row)
};

__host__ __device__ constexpr int rt_corr_pitch(int m) { return 16 * m + 4; }
__host__ __device__ constexpr int rt_filter_floats(int m) { return 32 * m + 32; }
__host__ __device__ constexpr size_t rt_corr_lds_bytes(int m)
{
    return (size_t)kRtWaves * (size_t)(kRbRows * rt_corr_pitch(m) + rt_filter_floats(m)) * sizeof(float);
}

// out[b, c, t] = sum_j in~[b, c, t + j - pad] * f_eff[c, j] for sixteen rows b of channel c at a time.
// Grid: C * J waves, channel fastest, four waves to a block (neighbouring channels: their rows are neighbours in memory).
template <typename T>
__global__ __launch_bounds__(64 * kRtWaves, 2) void corr_rowtall_kernel(const T *__restrict__ in, const T *__restrict__ f,
                                                                         T *__restrict__ out, const RowTallGeom g)
{
    constexpr int ES = (int)sizeof(T);
    extern __shared__ __align__(16) float dyn_lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int i16 = lane & 15;      // A: output position r;  B/D: row of the unit
    const int k4 = lane >> 4;       // contraction sub-index;  D: position group
    const int Lo = rt_corr_pitch(g.m);
    const int FW = rt_filter_floats(g.m);
    float *sw = dyn_lds + wave * (kRbRows * Lo + FW);
    float *fw = sw + kRbRows * Lo;

    const int id = (int)blockIdx.x * kRtWaves + wave;
    const int c = id % g.C;
    int unit = id / g.C;
    if (unit >= g.J) return;                    // (no workgroup barrier below)

    // filter window: fw[i] = f_eff[i + jbase]; offset d, lane (r, k), element v reads i = 16 (d + m - 1) + 4 k + v - r + 15
    {
        const T *f_c = f + (size_t)c * (size_t)g.K;
        const int jbase = g.pad - 16 * (g.m - 1) - 15;
        for (int i = lane; i < FW; i += 64) {
            const int j = i + jbase;
            float v = 0.f;
            if (j >= 0 && j < g.K) v = ld_elem(f_c + (g.reverse ? (g.K - 1 - j) : j));
            fw[i] = v;
        }
    }
    for (int i = lane; i < kRbRows * Lo / 4; i += 64)
        *reinterpret_cast<float4 *>(sw + 4 * i) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_fence();

    const int CL = g.C * g.L;
    const int Lg = (g.L + 3) >> 2;              // granules per row (the last one partial when L % 4 != 0)
    const int rem_last = g.L & 3;
    const int NG = kRbRows * Lg;                // granules per unit
    const float *a_lane = fw + 16 * (g.m - 1) + 4 * k4 - i16 + 15;
    const float *sp = sw + i16 * Lo + 4 * k4;

    // A unit is loaded eight granules per lane at a time and the loads are waited for before anything else happens:
    // registers that loads the compiler does not track are still writing must not stay live across the contraction
    // loop below (a variant that prefetched the next unit there faulted: nothing keeps the compiler from copying such
    // registers and reusing the originals).  Two or three workgroups per compute unit overlap one wave's loads with
    // another's matrix work instead.
    for (; unit < g.n_units; unit += g.J) {
        const int b0 = kRbRows * unit;
        const int nr = g.B - b0 < kRbRows ? g.B - b0 : kRbRows;        // rows past the batch read as zeros
        {
            const uintx4 r = rb_unit_resource(in + ((size_t)b0 * (size_t)g.C + (size_t)c) * (size_t)g.L, nr, CL, g.L);
            for (int g0 = 0; g0 < NG; g0 += 8 * 64) {
                typename Raw4<T>::type pre[8];
                int idx[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int gi = g0 + 64 * i + lane;
                    const int row = (int)__umulhi((unsigned)gi, g.lg_recip);
                    const int cg = gi - row * Lg;
                    // (low bits of idx: elements of a partial last granule, as in the sixteen-row kernels)
                    idx[i] = gi < NG ? ((row * Lo + 4 * cg) | (cg == Lg - 1 ? rem_last : 0)) : -1;
                    pre[i] = Raw4<T>::load(r, gi < NG ? ES * (row * CL + 4 * cg) : kOutOfRow);
                }
                wait_untracked_loads();
                release_after_wait(pre);
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (idx[i] >= 0) *reinterpret_cast<float4 *>(sw + (idx[i] & ~3)) = rb_granule<T>(pre[i], idx[i] & 3);
            }
        }
        wave_lds_fence();
        // lane (row i16 of the unit, position group k4) owns outputs 16 mo + 4 k4 + 0..3 of block mo
        T *out_lane = out + ((size_t)(b0 + i16) * (size_t)g.C + (size_t)c) * (size_t)g.L + 4 * k4;
        const bool row_ok = i16 < nr;
        for (int mo = 0; mo < g.m; ++mo) {
            const int mi_lo = mo + g.dmin > 0 ? mo + g.dmin : 0;
            const int mi_hi = mo + g.dmax < g.m - 1 ? mo + g.dmax : g.m - 1;
            // (two chains of dependent matrix instructions, even and odd input blocks, added at the end; reading the next
            // pair's operands ahead by hand, or advancing the addresses by pointer increments, measured no faster)
            floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f}, acc2 = acc;
            auto pair = [&](int mi, floatx4 &a) {
                const float *ap = a_lane + 16 * (mi - mo);
                const float a0 = ap[0], a1 = ap[1], a2 = ap[2], a3 = ap[3];
                const float4 cur = *reinterpret_cast<const float4 *>(sp + 16 * mi);
                a = mfma16x16x4(a0, cur.x, a);
                a = mfma16x16x4(a1, cur.y, a);
                a = mfma16x16x4(a2, cur.z, a);
                a = mfma16x16x4(a3, cur.w, a);
            };
            int mi = mi_lo;
            for (; mi + 1 <= mi_hi; mi += 2) {
                pair(mi, acc);
                pair(mi + 1, acc2);
            }
            if (mi <= mi_hi) pair(mi, acc);
            acc += acc2;
            if (row_ok)
                st_elem4_stream_upto(out_lane + 16 * mo, make_float4(acc[0], acc[1], acc[2], acc[3]), 16 * mo + 4 * k4, g.L);
        }
        wave_lds_fence();       // (the image is rewritten by the next unit's loads)
    }
}

// Stage 1 of the weight gradient for such rows.  grid = (C, S, windows), W = 4 waves per block; wave w of slice s takes
// the units W s + w, W s + w + W S, ... of four rows of its channel (walked from the last batch to the first, like the
// other weight-gradient kernels).  Window z owns the relative block offsets wlo = dmin + 15 z .. wlo + 14: accumulator e
// is offset wlo + e,  G_e[q'][q] += x[b][16 (mo + wlo + e) + q'] * dY[b][16 mo + q]  over the four rows b of a unit (the
// contraction index of one matrix instruction) and all output blocks mo whose partner lies inside the row.  The block
// writes slice z * S + s of part: the taps its window reaches, zeros elsewhere.
__host__ __device__ constexpr int rt_dw_pitch(int m)
{
    int p = 16 * m;
    while (p % 64 != 16 && p % 64 != 48) p += 16;
    return p;
}
__host__ __device__ constexpr int rt_dw_wave_floats(int m)
{
    const int stage = 2 * 4 * rt_dw_pitch(m);
    const int diag = ((16 * kRtWindow + 15) * 17 + 3) / 4 * 4;
    return stage > diag ? stage : diag;
}
__host__ __device__ constexpr size_t rt_dw_lds_bytes(int m)
{
    return (size_t)kRtWaves * (size_t)(rt_dw_wave_floats(m) + rb_tap_floats(kRtWindow)) * sizeof(float);
}

template <typename T>
__global__ __launch_bounds__(64 * kRtWaves, 2) void dw_rowtall_kernel(const T *__restrict__ x, const T *__restrict__ dy,
                                                                       float *__restrict__ part, const RowTallGeom g)
{
    constexpr int ES = (int)sizeof(T);
    constexpr int NE = kRtWindow;
    constexpr int RU = 4;                       // rows per unit: the contraction of one matrix instruction
    constexpr int NLD = RU * (16 * kRtMaxBlocks / 4) / 64;      // granule loads per lane, unit and tensor, at most (8)
    extern __shared__ __align__(16) float dyn_lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, k4 = lane >> 4;
    const int c = (int)blockIdx.x;
    const int wreg = rt_dw_wave_floats(g.m);
    float *s_wave = dyn_lds + wave * wreg;
    float *s_dw = dyn_lds + kRtWaves * wreg;          // [wave][rb_tap_floats(NE)]
    const int Lp = rt_dw_pitch(g.m);
    float *sx = s_wave, *sg = s_wave + RU * Lp;
    const int wlo = g.dmin + g.win * (int)blockIdx.z;  // first relative offset of this window
    const int whi = min(g.dmax, wlo + g.win - 1);      // ... and its last

    floatx4 G[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) G[e] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int i = lane; i < 2 * RU * Lp / 4; i += 64)
        *reinterpret_cast<float4 *>(s_wave + 4 * i) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_fence();

    const int CL = g.C * g.L;
    const int Lg = (g.L + 3) >> 2;              // (the last granule of a row partial when L % 4 != 0)
    const int NG = RU * Lg;                     // granules of a unit, per tensor
    const int nld = (NG + 63) >> 6;             // loads per lane (wave-uniform)
    int gl_off[NLD], idx[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int gi = lane + 64 * i;
        const int row = (int)__umulhi((unsigned)gi, g.lg_recip);
        const int cg = gi - row * Lg;
        gl_off[i] = gi < NG ? ES * (row * CL + 4 * cg) : kOutOfRow;
        idx[i] = gi < NG ? ((row * Lp + 4 * cg) | (cg == Lg - 1 ? (g.L & 3) : 0)) : -1;      // (low bits: see corr_rowtall_kernel)
    }
    const int stride = (int)gridDim.y * kRtWaves;
    int unit = (int)blockIdx.y * kRtWaves + wave;
    // A unit is loaded and waited for before it is contracted (no registers that untracked loads are still writing stay
    // live across the contraction: see corr_rowtall_kernel); two workgroups per compute unit overlap instead.
    auto load_unit = [&](int u) {
        const int b0 = RU * (g.n_units - 1 - u);
        const int nr = g.B - b0 < RU ? g.B - b0 : RU;
        const size_t first = ((size_t)b0 * (size_t)g.C + (size_t)c) * (size_t)g.L;
        const uintx4 rx = rb_unit_resource(x + first, nr, CL, g.L);
        const uintx4 rg = rb_unit_resource(dy + first, nr, CL, g.L);
        typename Raw4<T>::type px[NLD], pg[NLD];
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (i < nld) {
                px[i] = Raw4<T>::load(rx, gl_off[i]);
                pg[i] = Raw4<T>::load(rg, gl_off[i]);
            }
        wait_untracked_loads();
        release_after_wait(px);
        release_after_wait(pg);
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (i < nld && idx[i] >= 0) {
                *reinterpret_cast<float4 *>(sx + (idx[i] & ~3)) = rb_granule<T>(px[i], idx[i] & 3);
                *reinterpret_cast<float4 *>(sg + (idx[i] & ~3)) = rb_granule<T>(pg[i], idx[i] & 3);
            }
    };
    const float *xrow = sx + k4 * Lp + i16;     // lane (q' = i16, row k4): x[row][16 mi + q']
    const float *grow = sg + k4 * Lp + i16;     // lane (q = i16, row k4): dY[row][16 mo + q]
    for (; unit < g.n_units; unit += stride) {
        load_unit(unit);
        wave_lds_fence();
        // one relative offset at a time over the output blocks whose partner lies inside the row: no branch inside the
        // loops (a test per matrix instruction left the matrix pipe waiting on its LDS reads: 26 against 42 TFLOP/s at L = K = 256)
        static_for<0, NE>([&](auto ec) {
            constexpr int e = decltype(ec)::value;
            const int rel = wlo + e;
            if (rel <= whi) {
                const int mo_lo = rel < 0 ? -rel : 0;
                const int mo_hi = rel > 0 ? g.m - 1 - rel : g.m - 1;
                // (two chains of dependent matrix instructions, even and odd output blocks, added at the end)
                floatx4 acc = G[e], acc2 = floatx4{0.f, 0.f, 0.f, 0.f};
                const float *xp = xrow + 16 * rel;
                int mo = mo_lo;
#pragma unroll 2
                for (; mo + 1 <= mo_hi; mo += 2) {
                    acc = mfma16x16x4(xp[16 * mo], grow[16 * mo], acc);
                    acc2 = mfma16x16x4(xp[16 * mo + 16], grow[16 * mo + 16], acc2);
                }
                if (mo <= mo_hi) acc = mfma16x16x4(xp[16 * mo], grow[16 * mo], acc);
                G[e] = acc + acc2;
            }
        });
        wave_lds_fence();       // (the images are rewritten by the next unit's loads)
    }

    // ---- per-wave diagonal sums over this window's offsets, then the waves of the block in wave order
    // (rb_diagonal_sums with accumulator e = relative offset wlo + e: its M chosen so that e - (M - 1) is that offset)
    const int TF = rb_tap_floats(NE);
    rb_diagonal_sums<NE>(G, 1 - wlo, s_wave, s_dw + wave * TF, lane, g.K, g.pad, wlo, NE);
    wave_lds_fence();
    __syncthreads();
    const int j0 = rb_tap_j0(g.pad, wlo), j1 = rb_tap_j1(g.K, g.pad, wlo, NE);
    const size_t slice = (size_t)blockIdx.z * (size_t)gridDim.y + (size_t)blockIdx.y;
    for (int j = tid; j < g.K; j += 64 * kRtWaves) {
        float sum = 0.f;
        if (j >= j0 && j < j1) {
#pragma unroll
            for (int w = 0; w < kRtWaves; ++w) sum += s_dw[w * TF + (j - j0)];
        }
        part[(slice * (size_t)g.C + (size_t)c) * (size_t)g.K + (size_t)j] = sum;
    }
}

}  // namespace dwconv
