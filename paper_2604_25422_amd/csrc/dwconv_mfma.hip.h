// Matrix-core (MFMA) kernels for filters of moderate length (16*ND-30 >= K).
//
// The time axis is cut into blocks of 16:  t = 16 n + r.  With input index
// u = t + j - pad = 16 (n + d) + q, the tap is j = 16 d + q - r + pad, so for each
// block offset d the operator of Sec. IV-A eq. (dwconv) is a 16x16 Toeplitz block
//     Toep_d[r][q] = w[16 d + q - r + pad]      (zero outside [0, K))
// and   Y[n][r] = sum_d sum_q Toep_d[r][q] X[n + d][q].
// d runs over ND = dmax - dmin + 1 values, dmin = ceil((-pad-15)/16),
// dmax = floor((K-1-pad+15)/16).  That is a dense contraction whose left operand
// depends on the channel only, so it maps on v_mfma_f32_16x16x4_f32 with the
// Toeplitz blocks held in registers for the whole life of a wave:
//     forward / input gradient:  D[r][n] += Toep_d[r][4k+v] * X[n+d][4k+v]
//     weight gradient (eq. (dk_def)):  G_d[q'][q] += X[n+d][q'] * dY[n][q]  (contraction over n),
//         dw[j] = sum of G_d[q'][q] over 16 d + q' - q + pad = j.
// fp32 products and sums throughout (the matrix core computes fp32 FMA here),
// so results carry the same error bound as a sequential fp32 sum of K terms.
//
// Register layout of v_mfma_f32_16x16x4_f32 (wave64), lane = 16*k + i:
//   A (16x4):  lane holds A[i][k]          B (4x16): lane holds B[k][i]
//   D (16x16): lane holds D[4*k + v][i] in vector element v = 0..3
#pragma once
#include "dwconv_common.hip.h"

namespace dwconv {

typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ floatx4 mfma16x16x4(float a, float b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

constexpr int kLdsBlockStride = 20;   // floats per staged 16-block: 16 + 4 pad (bank spread for strided b128 reads)

// Geometry the host computes once per call for the correlate kernel.
struct CorrGeom {
    int C, L, K, B;
    int pad;            // effective pad of this correlation
    int reverse;        // filter index reversed (input gradient)
    int dmin;           // first block offset
    int segs_per_row;   // segments of SEGBLK*16 outputs per row
    int rows_per_block; // rows a block covers when a row has fewer segments than the block has waves
    int groups_per_row; // blocks per row otherwise
};

// out[row, t] = sum_j in~[row, t + j - pad] * f_eff[c, j]
// One wave = one segment of SEGBLK*16 consecutive outputs of one (b,c) row; the waves of a
// block share the channel.  Each wave stages its segment plus halo into its own LDS region.
template <typename T, int ND, int WAVES, int SEGBLK>
__global__ __launch_bounds__(64 * WAVES) void corr_mfma_kernel(const T *__restrict__ in, const T *__restrict__ f,
                                                                T *__restrict__ out, const CorrGeom g)
{
    constexpr int NIB = SEGBLK + ND - 1;           // input blocks staged per segment
    constexpr int NDT = SEGBLK / 16;               // D tiles (16 blocks = 256 outputs) per segment
    static_assert(SEGBLK % 16 == 0, "segment is a whole number of D tiles");
    __shared__ __align__(16) float s_in[WAVES][NIB * kLdsBlockStride];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i16 = lane & 15;      // A: output position r;  B/D: block j
    const int k4 = lane >> 4;       // contraction sub-index;  D: row group

    // ---- which segment is this wave's
    const unsigned bx = blockIdx.x;
    const int grp = (int)(bx % (unsigned)g.groups_per_row);
    const int c = (int)((bx / (unsigned)g.groups_per_row) % (unsigned)g.C);
    const int bg = (int)(bx / ((unsigned)g.groups_per_row * (unsigned)g.C));
    int b, seg;
    if (g.segs_per_row >= WAVES) {
        b = bg;
        seg = grp * WAVES + wave;
    } else {
        const int sub = wave / g.segs_per_row;
        b = bg * g.rows_per_block + sub;
        seg = wave % g.segs_per_row;
        if (sub >= g.rows_per_block) b = g.B;   // idle wave
    }
    const bool active = (b < g.B) && (seg < g.segs_per_row);

    // ---- Toeplitz operands: A[d][v] (lane (r, k)) = f_eff[16 (dmin + d) + 4k + v - r + pad]
    float A[ND][4];
    {
        const T *f_c = f + (size_t)c * (size_t)g.K;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int j = 16 * (g.dmin + d) + 4 * k4 + v - i16 + g.pad;
                float a = 0.f;
                if (j >= 0 && j < g.K) a = ld_elem(f_c + (g.reverse ? (g.K - 1 - j) : j));
                A[d][v] = a;
            }
    }

    const size_t row = (size_t)(active ? b : 0) * (size_t)g.C + (size_t)c;
    const T *in_row = in + row * (size_t)g.L;
    const int t0 = seg * (SEGBLK * 16);

    // ---- stage the segment: LDS block lb holds in~[16 (t0/16 + dmin + lb) + 0..15]
    if (active) {
        const int u0 = t0 + 16 * g.dmin;
        float *sw = s_in[wave];
        for (int gi = lane; gi < NIB * 4; gi += 64) {
            const int u = u0 + 4 * gi;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (u >= 0 && u + 3 < g.L) v = ld_elem4(in_row + u);
            *reinterpret_cast<float4 *>(sw + (gi >> 2) * kLdsBlockStride + (gi & 3) * 4) = v;
        }
    }
    __syncthreads();
    if (!active) return;

    // ---- contraction: NDT independent accumulators
    floatx4 acc[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) acc[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    const float *sp = s_in[wave] + i16 * kLdsBlockStride + 4 * k4;
#pragma unroll
    for (int d = 0; d < ND; ++d) {
        float4 bv[NDT];
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
            bv[dt] = *reinterpret_cast<const float4 *>(sp + (16 * dt + d) * kLdsBlockStride);
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            acc[dt] = mfma16x16x4(A[d][0], bv[dt].x, acc[dt]);
            acc[dt] = mfma16x16x4(A[d][1], bv[dt].y, acc[dt]);
            acc[dt] = mfma16x16x4(A[d][2], bv[dt].z, acc[dt]);
            acc[dt] = mfma16x16x4(A[d][3], bv[dt].w, acc[dt]);
        }
    }

    // ---- store: lane (block j = i16, row group k4) owns outputs 16 j + 4 k4 + 0..3 of each D tile
    T *out_row = out + row * (size_t)g.L;
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) {
        const int t = t0 + 256 * dt + 16 * i16 + 4 * k4;
        if (t + 3 < g.L) st_elem4(out_row + t, make_float4(acc[dt][0], acc[dt][1], acc[dt][2], acc[dt][3]));
    }
}

// Stage 1 of the weight gradient on the matrix cores.
// grid = (C, S).  A block walks the (b, tile) items of its slice; a tile is TT positions.
// Wave w takes the 64-position chunks w, w+WAVES, ... of every tile and keeps ND 16x16
// accumulators G_d for its whole life; at the end the diagonals of all G_d of all waves are
// summed through LDS in a fixed order.
template <typename T, int ND, int WAVES, int TT>
__global__ __launch_bounds__(64 * WAVES) void dw_partial_mfma_kernel(const T *__restrict__ x, const T *__restrict__ dy,
                                                                      float *__restrict__ part, int B, int C, int L,
                                                                      int K, int pad, int dmin, int tiles_per_row,
                                                                      int items_per_slice)
{
    constexpr int XW = TT + 16 * ND;                      // staged x window (floats)
    constexpr int STAGE = XW + TT;
    constexpr int RED = WAVES * ND * 256;
    constexpr int LDSF = STAGE > RED ? STAGE : RED;
    static_assert(TT % (64 * WAVES) == 0, "tile is a whole number of chunk rounds");
    __shared__ __align__(16) float s_mem[LDSF];
    float *s_x = s_mem;
    float *s_dy = s_mem + XW;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int c = blockIdx.x;
    const int s = blockIdx.y;
    const int items = B * tiles_per_row;
    const int it_begin = s * items_per_slice;
    const int it_end = min(items, it_begin + items_per_slice);

    floatx4 G[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) G[d] = floatx4{0.f, 0.f, 0.f, 0.f};

    for (int it = it_begin; it < it_end; ++it) {
        const int b = it / tiles_per_row;
        const int t0 = (it % tiles_per_row) * TT;
        const size_t row = ((size_t)b * (size_t)C + (size_t)c) * (size_t)L;
        const T *x_row = x + row;
        const T *dy_row = dy + row;
        __syncthreads();
        // s_dy[i] = dy[t0 + i];  s_x[i] = x~[t0 + 16 dmin + i]   (16-byte granules, zero outside the row)
        for (int gi = tid; gi < TT / 4; gi += 64 * WAVES) {
            const int t = t0 + 4 * gi;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (t + 3 < L) v = ld_elem4(dy_row + t);
            *reinterpret_cast<float4 *>(s_dy + 4 * gi) = v;
        }
        const int u0 = t0 + 16 * dmin;
        for (int gi = tid; gi < XW / 4; gi += 64 * WAVES) {
            const int u = u0 + 4 * gi;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (u >= 0 && u + 3 < L) v = ld_elem4(x_row + u);
            *reinterpret_cast<float4 *>(s_x + 4 * gi) = v;
        }
        __syncthreads();
        const int nch = min(TT, L - t0 + 63) / 64;        // chunks that hold at least one position < L
        for (int ch = wave; ch < nch; ch += WAVES) {
            const float gq = s_dy[64 * ch + lane];        // B operand: dY[n0 + k][q]
#pragma unroll
            for (int d = 0; d < ND; ++d)                  // A operand: X[n0 + k + dmin + d][q']
                G[d] = mfma16x16x4(s_x[64 * ch + 16 * d + lane], gq, G[d]);
        }
    }

    // ---- ordered reduction: red[w][d][q'][q]; lane (q = lane%16, k = lane/16) holds q' = 4k + v
    __syncthreads();
    float *red = s_mem;
#pragma unroll
    for (int d = 0; d < ND; ++d)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            red[((wave * ND + d) * 16 + 4 * (lane >> 4) + v) * 16 + (lane & 15)] = G[d][v];
    __syncthreads();
    for (int j = tid; j < K; j += 64 * WAVES) {
        float sum = 0.f;
        for (int d = 0; d < ND; ++d) {
            const int e = j - pad - 16 * (dmin + d);      // q' - q on this diagonal
            if (e < -15 || e > 15) continue;
            const int q_lo = e > 0 ? e : 0, q_hi = e > 0 ? 15 : 15 + e;
            for (int qp = q_lo; qp <= q_hi; ++qp)
                for (int w = 0; w < WAVES; ++w) sum += red[((w * ND + d) * 16 + qp) * 16 + (qp - e)];
        }
        part[((size_t)s * (size_t)C + (size_t)c) * (size_t)K + (size_t)j] = sum;
    }
}

}  // namespace dwconv
