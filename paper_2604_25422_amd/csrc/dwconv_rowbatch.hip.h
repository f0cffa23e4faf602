// Short rows on the matrix cores, sixteen rows at a time (fp32, L <= 64, L % 4 == 0).
//
// The operator of Sec. IV-A eq. (dwconv) treats every row (b, c) on its own, and the paper's own workload
// (Sec. V: windows of 48 steps) has rows of three 16-blocks.  The blocked-Toeplitz contraction of
// dwconv_mfma.hip.h needs sixteen independent columns per matrix instruction; here they are sixteen ROWS of the
// same channel (b = 16 u .. 16 u + 15, one "unit") at the same block position instead of sixteen consecutive
// blocks of one row:
//     forward / input gradient:  D[r][b] += Toep_d[r][4k+v] * X[b][mi][4k+v],   mi = mo + d inside the row only,
//     weight gradient (eq. (dk_def)):  G_d[q'][q] += X[b][mo + d][q'] * dY[b][mo][q], contraction over b.
// Block pairs (mo, mi) whose input block lies outside the row are skipped (they hold the zero padding), so a row
// of m blocks costs (pairs inside the row) * 4 matrix instructions per unit and no position of a padded segment
// is computed: for L = 48, K = 48, pad = 24 that is 36 instructions per 768 outputs.
#pragma once
#include "dwconv_mfma.hip.h"

namespace dwconv {

constexpr int kRbRows = 16;       // rows of one channel per unit
constexpr int kRbMaxL = 64;       // longest row
constexpr int kRbMaxBlocks = 4;   // 16-blocks per row
constexpr int kRbMaxLoads = 4;    // 16 rows * (L / 4) granules over 64 lanes

// Pitch (floats) of a row in the weight-gradient kernel's LDS image: at least the row rounded up to whole blocks,
// and congruent to 16 or 48 modulo 64 so that the four rows one operand read touches (64 bytes each) fall into
// four different quarters of the LDS banks.
__host__ __device__ constexpr int rb_dw_pitch(int L)
{
    int p = (L + 15) / 16 * 16;
    while (p % 64 != 16 && p % 64 != 48) p += 16;
    return p;
}
// Floats of one wave's LDS region in the weight-gradient kernel: both operands, or the diagonal image of the epilogue.
__host__ __device__ constexpr int rb_dw_wave_floats(int L, int ND)
{
    const int stage = 2 * kRbRows * rb_dw_pitch(L);
    const int diag = ((16 * ND + 15) * 17 + 3) / 4 * 4;
    return stage > diag ? stage : diag;
}

struct RowBatchGeom {
    int B, C, L, K;
    int pad;        // effective pad of this correlation
    int reverse;    // filter index reversed (input gradient)
    int dmin;       // first block offset
    int m;          // 16-blocks per row
    int n_units;    // ceil(B / 16)
    int J;          // waves per channel: wave (c, j) walks units j, j + J, ...
};

// Resource over rows b0 .. b0 + nr - 1 of channel c (row r of the unit starts r * C * L elements after the first).
__device__ __forceinline__ uintx4 rb_unit_resource(const float *base, int nr, int CL, int L)
{
    const unsigned long long a = reinterpret_cast<unsigned long long>(base);
    const uintx4 r = {(unsigned)a, (unsigned)(a >> 32) & 0xffffu, (unsigned)(((nr - 1) * CL + L) * 4), kBufferFlags};
    return r;
}

// Floats of one wave's LDS region in the correlate kernel: the input image (16-block mi of row r at float
// (mi * 16 + r) * kLdsBlockStride, the layout the strided 16-byte operand reads of the long-row kernel use), then
// the output image (row r at r * rb_out_pitch(L); the pitch is 4 modulo 8 floats so that the 16-byte tile writes
// of sixteen rows spread over the banks).
__host__ __device__ constexpr int rb_out_pitch(int L) { return (L % 8) == 0 ? L + 4 : L; }
__host__ __device__ constexpr int rb_corr_wave_floats(int L)
{
    return (L + 15) / 16 * 16 * kLdsBlockStride + kRbRows * rb_out_pitch(L);
}
constexpr int kRbCorrWaves = 4;   // waves per block: four neighbouring channels, whose rows share cache lines

// out[b, c, t] = sum_j in~[b, c, t + j - pad] * f_eff[c, j].   Grid = C * J waves, channel fastest, four to a
// block.  Per unit: the loads of the next unit are issued into registers, the current one is contracted, the
// D tiles go to the output image, the prefetch registers are drained into the input image, and the output image
// is stored with the lane-to-granule map of the loads (whole rows per store instruction; streaming stores, as in
// the long-row kernel).
template <int ND>
__global__ __launch_bounds__(64 * kRbCorrWaves, kMfmaWavesPerSimd) void corr_rowbatch_kernel(
    const float *__restrict__ in, const float *__restrict__ f, float *__restrict__ out, const RowBatchGeom g)
{
    extern __shared__ __align__(16) float dyn_lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int i16 = lane & 15;      // A: output position r;  B/D: row of the unit
    const int k4 = lane >> 4;       // contraction sub-index;  D: position group
    float *sw = dyn_lds + wave * rb_corr_wave_floats(g.L);
    float *so = sw + g.m * 16 * kLdsBlockStride;
    const int Lo = rb_out_pitch(g.L);

    const int id = (int)blockIdx.x * kRbCorrWaves + wave;
    const int c = id % g.C;
    int unit = id / g.C;
    if (unit >= g.J) return;                    // (no workgroup barrier below)

    const int CL = g.C * g.L;
    const int Lg = g.L >> 2;                    // granules per row
    const int NG = kRbRows * Lg;                // granules per unit
    const int nld = (NG + 63) >> 6;             // loads per lane (wave-uniform)
    int gl_off[kRbMaxLoads], lds_idx[kRbMaxLoads], so_idx[kRbMaxLoads];
#pragma unroll
    for (int i = 0; i < kRbMaxLoads; ++i) {
        const int gi = lane + 64 * i;
        const int r = gi / Lg, cg = gi - r * Lg;
        gl_off[i] = gi < NG ? 4 * (r * CL + 4 * cg) : kOutOfRow;
        lds_idx[i] = gi < NG ? (((cg >> 2) * 16 + r) * kLdsBlockStride + 4 * (cg & 3)) : 0;
        so_idx[i] = gi < NG ? r * Lo + 4 * cg : 0;
    }
    // zeros once: the part of the last block past the end of the row is never written again
    for (int i = lane; i < g.m * 16 * kLdsBlockStride / 4; i += 64)
        *reinterpret_cast<float4 *>(sw + 4 * i) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_fence();

    uintx4 pre[kRbMaxLoads];
    auto prefetch = [&](int u) {
        const int b0 = kRbRows * u;
        const int nr = g.B - b0 < kRbRows ? g.B - b0 : kRbRows;        // rows past the batch read as zeros
        const uintx4 r = rb_unit_resource(in + ((size_t)b0 * (size_t)g.C + (size_t)c) * (size_t)g.L, nr, CL, g.L);
#pragma unroll
        for (int i = 0; i < kRbMaxLoads; ++i)
            if (i < nld) pre[i] = buffer_load_x4_untracked(r, gl_off[i]);
    };
    auto drain = [&]() {
        wait_untracked_loads();
        release_after_wait(pre);
#pragma unroll
        for (int i = 0; i < kRbMaxLoads; ++i)
            if (i < nld && lane + 64 * i < NG)
                *reinterpret_cast<float4 *>(sw + lds_idx[i]) = Raw4<float>::widen(pre[i]);
    };
    prefetch(unit);
    drain();
    wave_lds_fence();

    // Toeplitz operands: A[d][v] (lane (r, k)) = f_eff[16 (dmin + d) + 4k + v - r + pad]
    float A[ND][4];
    {
        const float *f_c = f + (size_t)c * (size_t)g.K;
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
    }
    const float *sp = sw + i16 * kLdsBlockStride + 4 * k4;
    float *so_lane = so + i16 * Lo + 4 * k4;

    for (;;) {
        const int unit_n = unit + g.J;
        const bool more = unit_n < g.n_units;
        if (more) prefetch(unit_n);
        // lane (row i16 of the unit, position group k4) owns outputs 16 mo + 4 k4 + 0..3 of block mo
#pragma unroll
        for (int mo = 0; mo < kRbMaxBlocks; ++mo) {
            if (mo < g.m) {
                floatx4 a4 = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int d = 0; d < ND; ++d) {
                    const int mi = mo + g.dmin + d;
                    if (mi >= 0 && mi < g.m) {
                        const float4 cur = *reinterpret_cast<const float4 *>(sp + mi * 16 * kLdsBlockStride);
                        a4 = mfma16x16x4(A[d][0], cur.x, a4);
                        a4 = mfma16x16x4(A[d][1], cur.y, a4);
                        a4 = mfma16x16x4(A[d][2], cur.z, a4);
                        a4 = mfma16x16x4(A[d][3], cur.w, a4);
                    }
                }
                if (16 * mo + 4 * k4 < g.L)
                    *reinterpret_cast<float4 *>(so_lane + 16 * mo) = make_float4(a4[0], a4[1], a4[2], a4[3]);
            }
        }
        wave_lds_fence();
        if (more) drain();
        {
            const int b0 = kRbRows * unit;
            const int nr = g.B - b0 < kRbRows ? g.B - b0 : kRbRows;
            const int lim = 4 * nr * CL;                                                   // byte offsets of real rows
            float *out_u = out + ((size_t)b0 * (size_t)g.C + (size_t)c) * (size_t)g.L;      // wave-uniform
#pragma unroll
            for (int i = 0; i < kRbMaxLoads; ++i)
                if (i < nld && gl_off[i] < lim)
                    st_elem4_stream(out_u + (gl_off[i] >> 2), *reinterpret_cast<const float4 *>(so + so_idx[i]));
        }
        wave_lds_fence();
        if (!more) break;
        unit = unit_n;
    }
}

// Stage 1 of the weight gradient for short rows.  grid = (C, S), W waves per block; wave w of slice s takes the
// units W s + w, W s + w + W S, ... of its channel (walked from the last batch to the first, see the long-row
// kernel) and keeps ND 16x16 accumulators G_d for its whole life.  LDS image of a unit: rows of x, then rows
// of dY, pitch rb_dw_pitch(L) floats, zeros between the end of a row and the end of its last block.  One matrix
// instruction contracts four rows: A operand x[row 4 g + k][16 (mo + d) + q'], B operand dY[row 4 g + k][16 mo + q].
// dw_out == nullptr: the block's sums go to slice blockIdx.y of part; otherwise (gridDim.y == 1) they are the
// weight gradient itself.
template <int ND, int W>
__global__ __launch_bounds__(64 * W, kMfmaWavesPerSimd) void dw_rowbatch_kernel(
    const float *__restrict__ x, const float *__restrict__ dy, float *__restrict__ part, float *__restrict__ dw_out,
    int B, int C, int L, int K, int pad, int dmin, int n_units)
{
    extern __shared__ __align__(16) float dyn_lds[];
    const int wreg = rb_dw_wave_floats(L, ND);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, k4 = lane >> 4;
    const int c = blockIdx.x;
    float *s_wave = dyn_lds + wave * wreg;
    float *s_dw = dyn_lds + W * wreg + wave * (16 * ND);
    const int Lp = rb_dw_pitch(L);
    const int m = (L + 15) >> 4;
    float *sx = s_wave, *sg = s_wave + kRbRows * Lp;

    const int CL = C * L;
    const int Lg = L >> 2;
    const int NG = kRbRows * Lg;
    const int nld = (NG + 63) >> 6;
    int gl_off[kRbMaxLoads], lds_idx[kRbMaxLoads];
#pragma unroll
    for (int i = 0; i < kRbMaxLoads; ++i) {
        const int gi = lane + 64 * i;
        const int r = gi / Lg, cg = gi - r * Lg;
        gl_off[i] = gi < NG ? 4 * (r * CL + 4 * cg) : kOutOfRow;
        lds_idx[i] = gi < NG ? r * Lp + 4 * cg : 0;
    }
    for (int i = lane; i < 2 * kRbRows * Lp / 4; i += 64)
        *reinterpret_cast<float4 *>(s_wave + 4 * i) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_fence();

    floatx4 G[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) G[d] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int stride = (int)gridDim.y * W;
    int unit = (int)blockIdx.y * W + wave;
    uintx4 px[kRbMaxLoads], pg[kRbMaxLoads];
    auto prefetch = [&](int u) {
        const int b0 = kRbRows * (n_units - 1 - u);
        const int nr = B - b0 < kRbRows ? B - b0 : kRbRows;
        const size_t first = ((size_t)b0 * (size_t)C + (size_t)c) * (size_t)L;
        const uintx4 rx = rb_unit_resource(x + first, nr, CL, L);
        const uintx4 rg = rb_unit_resource(dy + first, nr, CL, L);
#pragma unroll
        for (int i = 0; i < kRbMaxLoads; ++i)
            if (i < nld) {
                px[i] = buffer_load_x4_untracked(rx, gl_off[i]);
                pg[i] = buffer_load_x4_untracked(rg, gl_off[i]);
            }
    };
    auto drain = [&]() {
        wait_untracked_loads();
        release_after_wait(px);
        release_after_wait(pg);
#pragma unroll
        for (int i = 0; i < kRbMaxLoads; ++i)
            if (i < nld && lane + 64 * i < NG) {
                *reinterpret_cast<float4 *>(sx + lds_idx[i]) = Raw4<float>::widen(px[i]);
                *reinterpret_cast<float4 *>(sg + lds_idx[i]) = Raw4<float>::widen(pg[i]);
            }
    };
    if (unit < n_units) {
        prefetch(unit);
        drain();
        wave_lds_fence();
    }
    while (unit < n_units) {
        const int unit_n = unit + stride;
        const bool more = unit_n < n_units;
        if (more) prefetch(unit_n);
#pragma unroll
        for (int g4 = 0; g4 < kRbRows / 4; ++g4) {
            const float *xrow = sx + (4 * g4 + k4) * Lp + i16;
            const float *grow = sg + (4 * g4 + k4) * Lp + i16;
            for (int mo = 0; mo < m; ++mo) {
                const float bq = grow[16 * mo];
#pragma unroll
                for (int d = 0; d < ND; ++d) {
                    const int mi = mo + dmin + d;
                    if (mi >= 0 && mi < m) G[d] = mfma16x16x4(xrow[16 * mi], bq, G[d]);
                }
            }
        }
        wave_lds_fence();
        if (more) {
            drain();
            wave_lds_fence();
        }
        unit = unit_n;
    }

    // ---- per-wave diagonal sums, then the waves of the block in wave order
    dw_wave_diagonal_sums<ND>(G, s_wave, s_dw, lane, K, pad, dmin);
    __syncthreads();
    for (int j = tid; j < K; j += 64 * W) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) sum += dyn_lds[W * wreg + w * (16 * ND) + j];
        if (dw_out) dw_out[(size_t)c * (size_t)K + (size_t)j] = sum;
        else part[((size_t)blockIdx.y * (size_t)C + (size_t)c) * (size_t)K + (size_t)j] = sum;
    }
}

}  // namespace dwconv
