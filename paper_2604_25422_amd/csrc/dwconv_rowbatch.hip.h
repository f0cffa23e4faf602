// Short rows on the matrix cores, sixteen rows at a time (L <= 128; fp32, or bf16 storage widened to fp32 on the way
// into LDS: fp32 matrix instructions and sums either way, one rounding at the store).  Rows are moved in granules of
// four elements; a row that is not whole granules (L % 4 != 0, one channel per wave) ends in a granule whose last
// elements belong to the next row: they are replaced by zeros on the way into LDS, and on the way out only the
// elements of the row are stored.  Rows need to start on a dword only (buffer loads; bf16: even L).
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
#include "dwconv_dw_direct.hip.h"   // static_for
#include "dwconv_mfma.hip.h"

namespace dwconv {

constexpr int kRbRows = 16;       // rows of one channel per unit
constexpr int kRbMaxL = 128;      // longest row
constexpr int kRbMaxBlocks = 8;   // 16-blocks per row

// Weight-gradient kernel: a wave owns NC neighbouring channels and works on units of 16 / NC rows (b), so a unit
// is the same number of bytes either way.  Pitch (floats) of a row (b, c0 .. c0 + NC - 1) in the LDS image: every
// channel rounded up to whole 16-blocks, the sum congruent to 16 or 48 modulo 64 so that the four rows one operand
// read touches (64 bytes each) fall into four different quarters of the LDS banks.
__host__ __device__ constexpr int rb_dw_pitch(int L, int NC)
{
    int p = NC * ((L + 15) / 16 * 16);
    while (p % 64 != 16 && p % 64 != 48) p += 16;
    return p;
}
// Floats of one wave's LDS region in the weight-gradient kernel: both operands, or the diagonal image of the epilogue.
// Rows (b) of a weight-gradient unit: 16 / NC, or 4 for rows of more than four blocks (one row group; the
// accumulators, one per relative block offset, leave fewer registers for staging).
__host__ __device__ constexpr int rb_dw_unit_rows(int L, int NC) { return (L + 15) / 16 > 4 ? 4 : kRbRows / NC; }
__host__ __device__ constexpr int rb_dw_wave_floats(int L, int ND, int NC)
{
    const int stage = 2 * rb_dw_unit_rows(L, NC) * rb_dw_pitch(L, NC);
    const int diag = ((16 * ND + 15) * 17 + 3) / 4 * 4;
    return stage > diag ? stage : diag;
}
// Taps the nd block offsets of a kernel can reach: 16 nd + 15 (all K of them when the offsets cover the filter; with
// the offsets cropped to those inside a row, a window [j0, j1) of a longer filter: the other taps are zero).
__host__ __device__ constexpr int rb_tap_floats(int ND) { return 16 * ND + 16; }
__host__ __device__ constexpr size_t rb_dw_lds_bytes(int L, int ND, int W, int NC)
{
    return (size_t)W * (size_t)(rb_dw_wave_floats(L, ND, NC) + NC * rb_tap_floats(ND)) * sizeof(float);
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
template <typename T>
__device__ __forceinline__ uintx4 rb_unit_resource(const T *base, int nr, int CL, int L)
{
    const unsigned long long a = reinterpret_cast<unsigned long long>(base);
    const uintx4 r = {(unsigned)a, (unsigned)(a >> 32) & 0xffffu, (unsigned)(((nr - 1) * CL + L) * (int)sizeof(T)),
                      kBufferFlags};
    return r;
}

// A granule on its way into LDS: rem = 0 for a whole one, else the number of its elements (1..3) that belong to the
// row; the others become the zeros the image holds behind the end of a row.
template <typename T>
__device__ __forceinline__ float4 rb_granule(typename Raw4<T>::type raw, int rem)
{
    float4 v = Raw4<T>::widen(raw);
    if (rem) {
        v.w = 0.f;
        if (rem < 3) v.z = 0.f;
        if (rem < 2) v.y = 0.f;
    }
    return v;
}
// ... and on its way out: whole granules as one streaming store, the last one of a ragged row by element.
template <typename T>
__device__ __forceinline__ void rb_store_granule(T *p, float4 v, int rem)
{
    if (!rem) {
        st_elem4_stream(p, v);
    } else {
        st_elem(p, v.x);
        if (rem > 1) st_elem(p + 1, v.y);
        if (rem > 2) st_elem(p + 2, v.z);
    }
}

// LDS image of a unit in the correlate kernel, one per wave: row r of the unit at float r * pitch; inside it the
// NC channels the wave owns, each rounded up to whole 16-blocks (the floats between the end of a row and the end
// of its last block stay zero).  The pitch is 4 modulo 8 floats, so the 16-byte operand reads and tile writes of
// sixteen rows spread over the banks.  The outputs of a unit replace its inputs in the same image.
__host__ __device__ constexpr int rb_corr_pitch(int L, int NC) { return NC * ((L + 15) / 16 * 16) + 4; }
__host__ __device__ constexpr int rb_corr_wave_floats(int L, int NC) { return kRbRows * rb_corr_pitch(L, NC); }
constexpr int kRbCorrWaves = 4;   // waves per block: neighbouring channels, whose rows share cache lines

// out[b, c, t] = sum_j in~[b, c, t + j - pad] * f_eff[c, j].
// A wave owns NC neighbouring channels (NC divides C): their rows (b, c0 .. c0 + NC - 1) are one contiguous piece
// of NC * L elements, so with NC = 2 a wave touches whole cache lines where rows of 48 elements would share them
// with the neighbouring channel's wave.  Grid = (C / NC) * J waves, channel group fastest, four waves to a block.
// Per unit: the loads of the next unit are issued into registers; the current one is contracted out of the LDS
// image, channel by channel, and the tiles of a channel replace its inputs; then every lane swaps its granules of
// the image (the lane-to-granule map of the loads): the outputs go out as whole rows (streaming stores, as in the
// long-row kernel), the prefetched inputs of the next unit come in.
// RAG: rows that are not whole granules (one channel per wave; the code for the partial granule is compiled only there).
template <typename T, int ND, int NC, int MB, bool RAG>
__global__ __launch_bounds__(64 * kRbCorrWaves, (ND > 9 ? 2 : (MB > 4 || RAG || ND > 6) ? 3 : kMfmaWavesPerSimd)) void corr_rowbatch_kernel(
    const T *__restrict__ in, const T *__restrict__ f, T *__restrict__ out, const RowBatchGeom g)
{
    constexpr int ES = (int)sizeof(T);          // bf16 storage is widened on the way into LDS; fp32 arithmetic
    // MB: 16-blocks per row the kernel is compiled for (two channels per wave: 3, the register budget)
    static_assert(MB >= 1 && MB <= kRbMaxBlocks && (NC == 1 || MB <= 3) && (NC == 1 || !RAG), "row blocks");
    constexpr int NLD = NC * MB;                 // 16 rows * NC * 4 MB granules over 64 lanes
    extern __shared__ __align__(16) float dyn_lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int i16 = lane & 15;      // A: output position r;  B/D: row of the unit
    const int k4 = lane >> 4;       // contraction sub-index;  D: position group
    const int Lc = 16 * g.m;
    const int Lo = NC * Lc + 4;
    float *sw = dyn_lds + wave * (kRbRows * Lo);

    const int Cg = g.C / NC;                    // channel groups
    const int id = (int)blockIdx.x * kRbCorrWaves + wave;
    const int c0 = NC * (id % Cg);
    int unit = id / Cg;
    if (unit >= g.J) return;                    // (no workgroup barrier below)

    const int CL = g.C * g.L;
    const int Lg = (g.L + 3) >> 2;              // granules per row (the last one partial when L % 4 != 0: NC is 1 then)
    const int NG = kRbRows * NC * Lg;           // granules per unit
    const int nld = (NG + 63) >> 6;             // loads per lane (wave-uniform)
    int gl_off[NLD], img[NLD];                  // img: float index in the image (a multiple of 4) + elements of a partial granule
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int gi = lane + 64 * i;
        const int r = gi / (NC * Lg), cg = gi - r * (NC * Lg);
        const int h = (NC > 1 && cg >= Lg) ? 1 : 0;
        static_assert(NC <= 2, "one or two channels per wave");
        gl_off[i] = gi < NG ? ES * (r * CL + 4 * cg) : kOutOfRow;
        img[i] = gi < NG ? (r * Lo + h * Lc + 4 * (cg - h * Lg)) | (RAG && cg == Lg - 1 ? (g.L & 3) : 0) : 0;
    }
    for (int i = lane; i < kRbRows * Lo / 4; i += 64)
        *reinterpret_cast<float4 *>(sw + 4 * i) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_fence();

    typename Raw4<T>::type pre[NLD];
    auto prefetch = [&](int u) {
        const int b0 = kRbRows * u;
        const int nr = g.B - b0 < kRbRows ? g.B - b0 : kRbRows;        // rows past the batch read as zeros
        const uintx4 r = rb_unit_resource(in + ((size_t)b0 * (size_t)g.C + (size_t)c0) * (size_t)g.L, nr, CL, NC * g.L);
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (i < nld) pre[i] = Raw4<T>::load(r, gl_off[i]);
    };
    auto drain = [&]() {
        wait_untracked_loads();
        release_after_wait(pre);
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (i < nld && lane + 64 * i < NG) {
                const int rem = RAG ? (img[i] & 3) : 0;
                *reinterpret_cast<float4 *>(sw + (img[i] - rem)) = rb_granule<T>(pre[i], rem);
            }
    };
    prefetch(unit);
    drain();
    wave_lds_fence();

    // Toeplitz operands: A[h][d][v] (lane (r, k)) = f_eff[c0 + h][16 (dmin + d) + 4k + v - r + pad]
    float A[NC][ND][4];
#pragma unroll
    for (int h = 0; h < NC; ++h) {
        const T *f_c = f + (size_t)(c0 + h) * (size_t)g.K;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int j = 16 * (g.dmin + d) + 4 * k4 + v - i16 + g.pad;
                const bool ok = j >= 0 && j < g.K;
                const int jc = ok ? (g.reverse ? (g.K - 1 - j) : j) : 0;
                const float a = ld_elem(f_c + jc);
                A[h][d][v] = ok ? a : 0.f;
            }
    }
    float *sp = sw + i16 * Lo + 4 * k4;

    for (;;) {
        const int unit_n = unit + g.J;
        const bool more = unit_n < g.n_units;
        if (more) prefetch(unit_n);
        // lane (row i16 of the unit, position group k4) owns outputs 16 mo + 4 k4 + 0..3 of block mo; one channel
        // at a time: its tiles replace its own inputs once all of them are computed
#pragma unroll
        for (int h = 0; h < NC; ++h) {
            floatx4 acc[MB];
#pragma unroll
            for (int mo = 0; mo < MB; ++mo) {
                floatx4 a4 = floatx4{0.f, 0.f, 0.f, 0.f};
                if (mo < g.m) {
#pragma unroll
                    for (int d = 0; d < ND; ++d) {
                        const int mi = mo + g.dmin + d;
                        if (mi >= 0 && mi < g.m) {
                            const float4 cur = *reinterpret_cast<const float4 *>(sp + h * Lc + 16 * mi);
                            a4 = mfma16x16x4(A[h][d][0], cur.x, a4);
                            a4 = mfma16x16x4(A[h][d][1], cur.y, a4);
                            a4 = mfma16x16x4(A[h][d][2], cur.z, a4);
                            a4 = mfma16x16x4(A[h][d][3], cur.w, a4);
                        }
                    }
                }
                acc[mo] = a4;
            }
            wave_lds_fence();
#pragma unroll
            for (int mo = 0; mo < MB; ++mo)
                if (mo < g.m && 16 * mo + 4 * k4 < g.L)
                    *reinterpret_cast<float4 *>(sp + h * Lc + 16 * mo) = make_float4(acc[mo][0], acc[mo][1], acc[mo][2], acc[mo][3]);
        }
        wave_lds_fence();
        // every lane swaps its granules of the image: outputs out (stored as whole rows), inputs of the next unit in
        wait_untracked_loads();
        release_after_wait(pre);
        {
            const int b0 = kRbRows * unit;
            const int nr = g.B - b0 < kRbRows ? g.B - b0 : kRbRows;
            const int lim = ES * nr * CL;                                                  // byte offsets of real rows
            T *out_u = out + ((size_t)b0 * (size_t)g.C + (size_t)c0) * (size_t)g.L;     // wave-uniform
#pragma unroll
            for (int i = 0; i < NLD; ++i)
                if (i < nld && lane + 64 * i < NG) {
                    const int rem = RAG ? (img[i] & 3) : 0;
                    const float4 ov = *reinterpret_cast<const float4 *>(sw + (img[i] - rem));
                    if (more) *reinterpret_cast<float4 *>(sw + (img[i] - rem)) = rb_granule<T>(pre[i], rem);
                    if (gl_off[i] < lim) rb_store_granule(out_u + gl_off[i] / ES, ov, rem);
                }
        }
        wave_lds_fence();
        if (!more) break;
        unit = unit_n;
    }
}

// First and one-past-last tap that the block offsets dmin .. dmin + nd - 1 reach: j = 16 d + q' - q + pad.
__host__ __device__ constexpr int rb_tap_j0(int pad, int dmin) { return pad + 16 * dmin - 15 > 0 ? pad + 16 * dmin - 15 : 0; }
__host__ __device__ constexpr int rb_tap_j1(int K, int pad, int dmin, int nd)
{
    const int e = pad + 16 * (dmin + nd - 1) + 16;
    const int j0 = rb_tap_j0(pad, dmin);
    return e < j0 ? j0 : (e < K ? e : K);
}

// Diagonal sums of accumulators that are indexed by the RELATIVE block offset rel = mi - mo = e - (M - 1)
// (the run-time counterpart of dw_wave_diagonal_sums: which offsets exist, dmin .. dmax, is known at run time only).
// sw: the wave's LDS region, at least ((16 nd + 15) * 17 + 3) / 4 * 4 floats; dw_wave[j], j < K, receives the sums.
template <int NR>
__device__ __forceinline__ void rb_diagonal_sums(const floatx4 (&G)[NR], int M, float *sw, float *dw_wave, int lane, int K,
                                                 int pad, int dmin, int nd)
{
    constexpr int RS = 17;
    const int rows = 16 * nd + 15;
    const int n4 = (rows * RS + 3) / 4;
    for (int i = lane; i < n4; i += 64) *reinterpret_cast<float4 *>(sw + 4 * i) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_fence();
    const int q = lane & 15, k4 = lane >> 4;
#pragma unroll
    for (int e = 0; e < NR; ++e) {
        const int d = e - (M - 1) - dmin;            // slot of this relative offset among dmin .. dmax
        if (d >= 0 && d < nd) {
#pragma unroll
            for (int v = 0; v < 4; ++v) sw[(16 * d + 4 * k4 + v - q + 15) * RS + q] = G[e][v];
        }
    }
    wave_lds_fence();
    // taps the offsets reach: j0 .. j1 - 1 (rb_tap_window), dw_wave[j - j0]
    const int j0 = rb_tap_j0(pad, dmin), j1 = rb_tap_j1(K, pad, dmin, nd);
    for (int j = j0 + lane; j < j1; j += 64) {
        const int jl = j - pad - 16 * dmin + 15;
        float sum = 0.f;
        if (jl >= 0 && jl < rows) {
            float t[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) t[i] = sw[jl * RS + i];
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += t[i];
        }
        dw_wave[j - j0] = sum;
    }
}

// Stage 1 of the weight gradient for short rows of M 16-blocks.  grid = (C / NC, S), W waves per block; wave w of
// slice s takes the units W s + w, W s + w + W S, ... of its channel group (walked from the last batch to the
// first, see the long-row kernel).  A unit is 16 / NC rows of NC neighbouring channels (NC = 2 makes whole cache
// lines of rows of 48 elements, see corr_rowbatch_kernel).  LDS image of a unit: rows of x, then rows of dY, pitch
// rb_dw_pitch floats, zeros between the end of a row and the end of its last block.  One matrix instruction
// contracts four rows:  A operand x[row 4 g + k][c0 + h][16 mi + q'],  B operand dY[row 4 g + k][c0 + h][16 mo + q],
// for every block pair (mo, mi) of the row whose offset mi - mo is one of the nd offsets dmin .. dmin + nd - 1 of
// the filter.  The accumulators are indexed by that relative offset (2 M - 1 per channel, compile-time indices;
// which of them exist is a wave-uniform run-time test), so the 2 M operand reads of a row group are issued
// together, ahead of its matrix instructions.
// dw_out == nullptr: the block's sums go to slice blockIdx.y of part; otherwise (gridDim.y == 1) they are the
// weight gradient itself.
// RAG: rows that are not whole granules (one channel per wave).
template <typename T, int M, int W, int NC, bool RAG>
__global__ __launch_bounds__(64 * W, kMfmaWavesPerSimd) void dw_rowbatch_kernel(
    const T *__restrict__ x, const T *__restrict__ dy, float *__restrict__ part, T *__restrict__ dw_out,
    int B, int C, int L, int K, int pad, int dmin, int nd, int n_units)
{
    constexpr int ES = (int)sizeof(T);
    static_assert(NC == 1 || NC == 2, "one or two channels per wave");
    static_assert(M >= 1 && M <= kRbMaxBlocks && (NC == 1 || M <= 3) && (NC == 1 || !RAG), "rows of at most 128 (two channels: 48) positions");
    constexpr int RU = M > 4 ? 4 : kRbRows / NC;              // rows per unit (rb_dw_unit_rows)
    constexpr int NLD = (RU * NC * 4 * M + 63) / 64;          // 16-byte granules of a unit over 64 lanes
    constexpr int NR = 2 * M - 1;                             // relative block offsets -(M-1) .. M-1
    extern __shared__ __align__(16) float dyn_lds[];
    const int wreg = rb_dw_wave_floats(L, nd, NC);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, k4 = lane >> 4;
    const int c0 = NC * (int)blockIdx.x;
    float *s_wave = dyn_lds + wave * wreg;
    float *s_dw = dyn_lds + W * wreg;                         // [wave][h][16 nd]
    const int Lp = rb_dw_pitch(L, NC);
    constexpr int Lc = 16 * M;
    float *sx = s_wave, *sg = s_wave + RU * Lp;
    const int dmax = dmin + nd - 1;

    const int CL = C * L;
    const int Lg = (L + 3) >> 2;                              // (the last granule partial when L % 4 != 0: NC is 1 then)
    const int NG = RU * NC * Lg;
    const int nld = (NG + 63) >> 6;
    int gl_off[NLD], lds_idx[NLD];                            // lds_idx: float index (a multiple of 4) + elements of a partial granule
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int gi = lane + 64 * i;
        const int r = gi / (NC * Lg), cg = gi - r * (NC * Lg);
        const int h = (NC > 1 && cg >= Lg) ? 1 : 0;
        gl_off[i] = gi < NG ? ES * (r * CL + 4 * cg) : kOutOfRow;
        lds_idx[i] = gi < NG ? (r * Lp + h * Lc + 4 * (cg - h * Lg)) | (RAG && cg == Lg - 1 ? (L & 3) : 0) : 0;
    }
    for (int i = lane; i < 2 * RU * Lp / 4; i += 64)
        *reinterpret_cast<float4 *>(s_wave + 4 * i) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_fence();

    floatx4 G[NC][NR];
#pragma unroll
    for (int h = 0; h < NC; ++h)
#pragma unroll
        for (int e = 0; e < NR; ++e) G[h][e] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int stride = (int)gridDim.y * W;
    int unit = (int)blockIdx.y * W + wave;
    typename Raw4<T>::type px[NLD], pg[NLD];
    auto prefetch = [&](int u) {
        const int b0 = RU * (n_units - 1 - u);
        const int nr = B - b0 < RU ? B - b0 : RU;
        const size_t first = ((size_t)b0 * (size_t)C + (size_t)c0) * (size_t)L;
        const uintx4 rx = rb_unit_resource(x + first, nr, CL, NC * L);
        const uintx4 rg = rb_unit_resource(dy + first, nr, CL, NC * L);
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (i < nld) {
                px[i] = Raw4<T>::load(rx, gl_off[i]);
                pg[i] = Raw4<T>::load(rg, gl_off[i]);
            }
    };
    auto drain = [&]() {
        wait_untracked_loads();
        release_after_wait(px);
        release_after_wait(pg);
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (i < nld && lane + 64 * i < NG) {
                const int rem = RAG ? (lds_idx[i] & 3) : 0;
                *reinterpret_cast<float4 *>(sx + (lds_idx[i] - rem)) = rb_granule<T>(px[i], rem);
                *reinterpret_cast<float4 *>(sg + (lds_idx[i] - rem)) = rb_granule<T>(pg[i], rem);
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
        // (template recursion instead of unroll pragmas: every accumulator index has to be a constant)
        static_for<0, (RU / 4) * NC>([&](auto gc) {
            constexpr int g4 = decltype(gc)::value / NC, h = decltype(gc)::value % NC;
            const float *xrow = sx + (4 * g4 + k4) * Lp + h * Lc + i16;
            const float *grow = sg + (4 * g4 + k4) * Lp + h * Lc + i16;
            float xa[M], gb[M];
            static_for<0, M>([&](auto bc) {
                constexpr int b = decltype(bc)::value;
                xa[b] = xrow[16 * b];
                gb[b] = grow[16 * b];
            });
            static_for<0, M * M>([&](auto pc) {
                constexpr int mo = decltype(pc)::value / M, mi = decltype(pc)::value % M;
                constexpr int rel = mi - mo;
                if (rel >= dmin && rel <= dmax) G[h][rel + M - 1] = mfma16x16x4(xa[mi], gb[mo], G[h][rel + M - 1]);
            });
        });
        wave_lds_fence();
        if (more) {
            drain();
            wave_lds_fence();
        }
        unit = unit_n;
    }

    // ---- per-wave diagonal sums, then the waves of the block in wave order
    const int TF = rb_tap_floats(nd);
#pragma unroll
    for (int h = 0; h < NC; ++h) {
        rb_diagonal_sums<NR>(G[h], M, s_wave, s_dw + (wave * NC + h) * TF, lane, K, pad, dmin, nd);
        wave_lds_fence();
    }
    __syncthreads();
    const int j0 = rb_tap_j0(pad, dmin), j1 = rb_tap_j1(K, pad, dmin, nd);      // (the other taps of a longer filter are zero)
    for (int e = tid; e < NC * K; e += 64 * W) {
        const int h = e / K, j = e - h * K;
        float sum = 0.f;
        if (j >= j0 && j < j1) {
#pragma unroll
            for (int w = 0; w < W; ++w) sum += s_dw[(w * NC + h) * TF + (j - j0)];
        }
        const size_t o = (size_t)(c0 + h) * (size_t)K + (size_t)j;
        if (dw_out) st_elem(dw_out + o, sum);
        else part[(size_t)blockIdx.y * (size_t)C * (size_t)K + o] = sum;
    }
}

// Fused backward for short rows: dx = correlate(dY, reversed w, pad' = K - 1 - pad) and stage 1 of the weight
// gradient from ONE pass over dY (units of sixteen rows of one channel).  grid = (ceil(C / 4), S): the four waves
// of a block own four neighbouring channels (their rows share cache lines) and slice blockIdx.y of the units,
// walked from the last batch to the first; every wave writes its own slice of part (or dw itself when S == 1), so
// there is no workgroup barrier.  Per unit a wave holds two LDS images: dY (row pitch
// 16 m + 4 floats, the layout of corr_rowbatch_kernel: 16-byte operand reads for dx, the tiles of dx replace dY in
// place) and x (pitch rb_dw_pitch).  Order per unit: prefetch of the next unit's dY and x rows into registers;
// G_d += x * dY; D tiles of dx from the dY image with the arithmetic of corr_rowbatch_kernel (same instruction
// order per output, so dx is bit-identical to the separate call); the tiles replace dY; every lane swaps its
// granules (dx out as whole rows, next dY in) and drains the next x rows.
constexpr int kRbBwdMaxL = 48;
__host__ __device__ constexpr int rb_bwd_dy_pitch(int L) { return (L + 15) / 16 * 16 + 4; }
__host__ __device__ constexpr int rb_bwd_wave_floats(int L, int ND)
{
    const int stage = kRbRows * (rb_bwd_dy_pitch(L) + rb_dw_pitch(L, 1));
    const int diag = ((16 * ND + 15) * 17 + 3) / 4 * 4;
    return stage > diag ? stage : diag;
}
constexpr int kRbBwdWaves = 4;
__host__ __device__ constexpr size_t rb_bwd_lds_bytes(int L, int ND)
{
    return (size_t)kRbBwdWaves * (size_t)(rb_bwd_wave_floats(L, ND) + rb_tap_floats(ND)) * sizeof(float);
}

// RAG: rows that are not whole granules (the masks and element stores of the partial granule cost registers this
// kernel does not have at four waves per SIMD, so that variant runs three).
template <typename T, int ND, int M, bool RAG>
__global__ __launch_bounds__(64 * kRbBwdWaves, (RAG ? 3 : kMfmaWavesPerSimd)) void bwd_rowbatch_kernel(
    const T *__restrict__ dy, const T *__restrict__ x, const T *__restrict__ w, T *__restrict__ dx,
    float *__restrict__ part, T *__restrict__ dw_out, int B, int C, int L, int K, int pad, int dmin, int n_units)
{
    constexpr int ES = (int)sizeof(T);
    // rows of at most kRbBwdMaxL positions (register budget: two prefetched tensors, Toeplitz operands, accumulators)
    static_assert(M >= 1 && 16 * M <= kRbBwdMaxL, "rows of M 16-blocks");
    constexpr int NLD = (kRbRows * 4 * M + 63) / 64;
    constexpr int MB = M;
    constexpr int NR = 2 * M - 1;                             // relative block offsets of the weight gradient
    extern __shared__ __align__(16) float dyn_lds[];
    const int wreg = rb_bwd_wave_floats(L, ND);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, k4 = lane >> 4;
    const int c = kRbBwdWaves * (int)blockIdx.x + wave;
    if (c >= C) return;                                       // (no workgroup barrier below)
    float *s_wave = dyn_lds + wave * wreg;
    float *s_dw = dyn_lds + kRbBwdWaves * wreg + wave * rb_tap_floats(ND);
    constexpr int m = M;
    const int Ld = 16 * m + 4;                                // pitch of the dY image
    const int Lp = rb_dw_pitch(L, 1);                         // pitch of the x image
    float *sd = s_wave, *sx = s_wave + kRbRows * Ld;
    // input-gradient geometry: pad' = K - 1 - pad, offsets -(dmin + ND - 1) .. -dmin
    const int padx = K - 1 - pad;
    const int dminx = -(dmin + ND - 1);

    const int CL = C * L;
    const int Lg = (L + 3) >> 2;                              // (the last granule partial when L % 4 != 0)
    const int NG = kRbRows * Lg;
    const int nld = (NG + 63) >> 6;
    int gl_off[NLD], img_d[NLD], img_x[NLD];                  // img_d: float index (a multiple of 4) + elements of a partial granule
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int gi = lane + 64 * i;
        const int r = gi / Lg, cg = gi - r * Lg;
        gl_off[i] = gi < NG ? ES * (r * CL + 4 * cg) : kOutOfRow;
        img_d[i] = gi < NG ? (r * Ld + 4 * cg) | (RAG && cg == Lg - 1 ? (L & 3) : 0) : 0;
        img_x[i] = gi < NG ? r * Lp + 4 * cg : 0;
    }
    for (int i = lane; i < kRbRows * (Ld + Lp) / 4; i += 64)
        *reinterpret_cast<float4 *>(s_wave + 4 * i) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_fence();

    floatx4 G[NR];
#pragma unroll
    for (int e = 0; e < NR; ++e) G[e] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int dmax = dmin + ND - 1;
    // Toeplitz operands of the input gradient: A[d][v] (lane (r, k)) = w[K - 1 - (16 (dminx + d) + 4k + v - r + padx)]
    float A[ND][4];
    {
        const T *f_c = w + (size_t)c * (size_t)K;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int j = 16 * (dminx + d) + 4 * k4 + v - i16 + padx;
                const bool ok = j >= 0 && j < K;
                const float a = ld_elem(f_c + (ok ? K - 1 - j : 0));
                A[d][v] = ok ? a : 0.f;
            }
    }

    const int stride = (int)gridDim.y;
    int unit = (int)blockIdx.y;
    typename Raw4<T>::type pd[NLD], px[NLD];
    auto prefetch = [&](int u) {
        const int b0 = kRbRows * (n_units - 1 - u);
        const int nr = B - b0 < kRbRows ? B - b0 : kRbRows;
        const size_t first = ((size_t)b0 * (size_t)C + (size_t)c) * (size_t)L;
        const uintx4 rd = rb_unit_resource(dy + first, nr, CL, L);
        const uintx4 rx = rb_unit_resource(x + first, nr, CL, L);
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (i < nld) {
                pd[i] = Raw4<T>::load(rd, gl_off[i]);
                px[i] = Raw4<T>::load(rx, gl_off[i]);
            }
    };
    if (unit < n_units) {
        prefetch(unit);
        wait_untracked_loads();
        release_after_wait(pd);
        release_after_wait(px);
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (i < nld && lane + 64 * i < NG) {
                const int rem = RAG ? (img_d[i] & 3) : 0;
                *reinterpret_cast<float4 *>(sd + (img_d[i] - rem)) = rb_granule<T>(pd[i], rem);
                *reinterpret_cast<float4 *>(sx + img_x[i]) = rb_granule<T>(px[i], rem);
            }
        wave_lds_fence();
    }
    float *sp = sd + i16 * Ld + 4 * k4;
    while (unit < n_units) {
        const int unit_n = unit + stride;
        const bool more = unit_n < n_units;
        if (more) prefetch(unit_n);
        // weight gradient: four rows per instruction, accumulators by relative block offset (see dw_rowbatch_kernel)
        static_for<0, kRbRows / 4>([&](auto gc) {
            constexpr int g4 = decltype(gc)::value;
            const float *xrow = sx + (4 * g4 + k4) * Lp + i16;
            const float *grow = sd + (4 * g4 + k4) * Ld + i16;
            float xa[M], gb[M];
            static_for<0, M>([&](auto bc) {
                constexpr int b = decltype(bc)::value;
                xa[b] = xrow[16 * b];
                gb[b] = grow[16 * b];
            });
            static_for<0, M * M>([&](auto pc) {
                constexpr int mo = decltype(pc)::value / M, mi = decltype(pc)::value % M;
                constexpr int rel = mi - mo;
                if (rel >= dmin && rel <= dmax) G[rel + M - 1] = mfma16x16x4(xa[mi], gb[mo], G[rel + M - 1]);
            });
        });
        // input gradient: lane (row i16, position group k4) owns outputs 16 mo + 4 k4 + 0..3 of block mo
        floatx4 acc[MB];
#pragma unroll
        for (int mo = 0; mo < MB; ++mo) {
            floatx4 a4 = floatx4{0.f, 0.f, 0.f, 0.f};
            if (mo < m) {
#pragma unroll
                for (int d = 0; d < ND; ++d) {
                    const int mi = mo + dminx + d;
                    if (mi >= 0 && mi < m) {
                        const float4 cur = *reinterpret_cast<const float4 *>(sp + 16 * mi);
                        a4 = mfma16x16x4(A[d][0], cur.x, a4);
                        a4 = mfma16x16x4(A[d][1], cur.y, a4);
                        a4 = mfma16x16x4(A[d][2], cur.z, a4);
                        a4 = mfma16x16x4(A[d][3], cur.w, a4);
                    }
                }
            }
            acc[mo] = a4;
        }
        wave_lds_fence();
#pragma unroll
        for (int mo = 0; mo < MB; ++mo)
            if (mo < m && 16 * mo + 4 * k4 < L)
                *reinterpret_cast<float4 *>(sp + 16 * mo) = make_float4(acc[mo][0], acc[mo][1], acc[mo][2], acc[mo][3]);
        wave_lds_fence();
        wait_untracked_loads();
        release_after_wait(pd);
        release_after_wait(px);
        {
            const int b0 = kRbRows * (n_units - 1 - unit);
            const int nr = B - b0 < kRbRows ? B - b0 : kRbRows;
            const int lim = ES * nr * CL;
            T *dx_u = dx + ((size_t)b0 * (size_t)C + (size_t)c) * (size_t)L;
#pragma unroll
            for (int i = 0; i < NLD; ++i)
                if (i < nld && lane + 64 * i < NG) {
                    const int rem = RAG ? (img_d[i] & 3) : 0;
                    const float4 ov = *reinterpret_cast<const float4 *>(sd + (img_d[i] - rem));
                    if (more) {
                        *reinterpret_cast<float4 *>(sd + (img_d[i] - rem)) = rb_granule<T>(pd[i], rem);
                        *reinterpret_cast<float4 *>(sx + img_x[i]) = rb_granule<T>(px[i], rem);
                    }
                    if (gl_off[i] < lim) rb_store_granule(dx_u + gl_off[i] / ES, ov, rem);
                }
        }
        wave_lds_fence();
        unit = unit_n;
    }

    // ---- diagonal sums of this wave's accumulators: its slice of the partial sums
    rb_diagonal_sums<NR>(G, M, s_wave, s_dw, lane, K, pad, dmin, ND);
    wave_lds_fence();
    const int j0 = rb_tap_j0(pad, dmin), j1 = rb_tap_j1(K, pad, dmin, ND);      // (the other taps of a longer filter are zero)
    for (int j = lane; j < K; j += 64) {
        const size_t o = (size_t)c * (size_t)K + (size_t)j;
        const float v = (j >= j0 && j < j1) ? s_dw[j - j0] : 0.f;
        if (dw_out) st_elem(dw_out + o, v);
        else part[(size_t)blockIdx.y * (size_t)C * (size_t)K + o] = v;
    }
}

}  // namespace dwconv
