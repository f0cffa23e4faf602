// Generic vector-ALU kernels (any B, C, L, K, pad; fp32 or bf16 storage).
//
// corr_valu_kernel      forward (Sec. IV-A eq. (dwconv)) and, with the filter
//                       index reversed and pad' = K-1-pad, the input gradient
//                       (adjoint of eq. (dwconv), cf. eq. (dx_def)).
// dw_partial_valu_kernel stage 1 of the weight gradient (eq. (dk_def)): per-block
//                       partial sums over a slice of (b, t), reduced in registers,
//                       then through LDS in a fixed order (no atomics).
// dw_finalize_kernel    stage 2: ordered sum of the partial slices.
//
// Both staged kernels keep the input window of a tile (tile + K-1 halo, zero
// filled outside the row) in LDS and slide a register window over it, so each
// LDS read feeds several fused multiply-adds.
#pragma once
#include "dwconv_common.hip.h"

namespace dwconv {

// out[row, t] = sum_j in~[row, t + j - pad] * f_eff[c, j],  f_eff[j] = reverse ? f[K-1-j] : f[j]
// One block = one tile of R*THREADS consecutive outputs of one (b,c) row.
// Taps are consumed in chunks of KCH so LDS stays bounded for any K; each chunk
// has its own accumulator that is added to the running total (bounds the length
// of any sequential fp32 sum by KCH + K/KCH).
// VROWS (short rows, see RowsMap): a tile is TILE consecutive positions of the VIRTUAL row of a channel - its B rows
// laid end to end with zeros between them - instead of a tile of one real row that is mostly padding; blockIdx.x / tiles_per_row
// is then the channel, and positions are translated where the window is staged and where outputs are stored.
template <typename T, int R, int THREADS, int KCH, bool VROWS>
__global__ __launch_bounds__(THREADS) void corr_valu_kernel(const T *__restrict__ in, const T *__restrict__ f,
                                                            T *__restrict__ out, int C, int L, int K, int pad,
                                                            int reverse, int tiles_per_row, const RowsMap rm)
{
    static_assert(R % 4 == 0 && KCH % 4 == 0, "vector width");
    constexpr int TILE = R * THREADS;
    __shared__ __align__(16) float s_in[TILE + KCH];
    __shared__ __align__(16) float s_f[KCH];

    const int tid = threadIdx.x;
    const size_t row = blockIdx.x / (unsigned)tiles_per_row;
    const int tile = blockIdx.x % (unsigned)tiles_per_row;
    const int c = VROWS ? (int)row : (int)(row % (size_t)C);
    const int t0 = tile * TILE;
    const T *in_row = in + row * (size_t)L;          // VROWS: row (0, c), the first of the channel
    const T *f_c = f + (size_t)c * (size_t)K;

    float total[R];
#pragma unroll
    for (int r = 0; r < R; ++r) total[r] = 0.f;

    for (int jc = 0; jc < K; jc += KCH) {
        const int kc = min(KCH, K - jc);
        const int kc4 = (kc + 3) & ~3;
        __syncthreads();
        for (int i = tid; i < kc4; i += THREADS) {
            const int j = jc + i;
            s_f[i] = (i < kc) ? ld_elem(f_c + (reverse ? (K - 1 - j) : j)) : 0.f;
        }
        const int g0 = t0 + jc - pad;
        for (int i = tid; i < TILE + kc4; i += THREADS) {
            const int g = g0 + i;
            if constexpr (VROWS) {
                const int e = rows_element(rm, g);
                s_in[i] = e >= 0 ? ld_elem(in_row + e) : 0.f;
            } else {
                s_in[i] = (g >= 0 && g < L) ? ld_elem(in_row + g) : 0.f;
            }
        }
        __syncthreads();

        float acc[R];
        float win[R + 4];
        const float *sp = s_in + R * tid;
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r] = 0.f;
#pragma unroll
        for (int r = 0; r < R; r += 4) {
            const float4 v = *reinterpret_cast<const float4 *>(sp + r);
            win[r] = v.x; win[r + 1] = v.y; win[r + 2] = v.z; win[r + 3] = v.w;
        }
        for (int j = 0; j < kc4; j += 4) {
            const float4 nx = *reinterpret_cast<const float4 *>(sp + R + j);
            const float4 wv = *reinterpret_cast<const float4 *>(s_f + j);
            win[R] = nx.x; win[R + 1] = nx.y; win[R + 2] = nx.z; win[R + 3] = nx.w;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                acc[r] = fmaf(win[r], wv.x, acc[r]);
                acc[r] = fmaf(win[r + 1], wv.y, acc[r]);
                acc[r] = fmaf(win[r + 2], wv.z, acc[r]);
                acc[r] = fmaf(win[r + 3], wv.w, acc[r]);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) win[r] = win[r + 4];
        }
#pragma unroll
        for (int r = 0; r < R; ++r) total[r] += acc[r];
    }

    const int t = t0 + R * tid;
    T *out_row = out + row * (size_t)L;
    if constexpr (VROWS) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int e = rows_element(rm, t + r);
            if (e >= 0) st_elem(out_row + e, total[r]);
        }
    } else if (t + R <= L && (L % 4) == 0) {
#pragma unroll
        for (int r = 0; r < R; r += 4)
            st_elem4(out_row + t + r, make_float4(total[r], total[r + 1], total[r + 2], total[r + 3]));
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (t + r < L) st_elem(out_row + t + r, total[r]);
    }
}

// part[s, c, j] = sum over the (b, tile) items of slice s of sum_t dy[b,c,t] * x~[b,c,t+j-pad]
// grid = (C, S).  Thread (jg, tg): taps 4*jg..4*jg+3 of the current tap chunk, positions
// [tg*SUB, (tg+1)*SUB) of each tile.  Items of a channel are (b, tile) pairs in row-major
// order; slice s owns the contiguous range [s*per, (s+1)*per).
// VROWS (short rows, see RowsMap): the items are the tiles_per_row tiles of the virtual row of the channel (B is 1).
template <typename T, int THREADS, int TT, int KCH, bool VROWS>
__global__ __launch_bounds__(THREADS) void dw_partial_valu_kernel(const T *__restrict__ x, const T *__restrict__ dy,
                                                                  float *__restrict__ part, int B, int C, int L, int K,
                                                                  int pad, int tiles_per_row, int items_per_slice,
                                                                  const RowsMap rm)
{
    constexpr int NJ = KCH / 4;
    constexpr int NT = THREADS / NJ;
    constexpr int SUB = TT / NT;
    static_assert(THREADS % NJ == 0 && TT % NT == 0 && SUB % 4 == 0, "thread layout");
    static_assert(NT * KCH <= TT + KCH, "reduction scratch fits the x window");
    __shared__ __align__(16) float s_x[TT + KCH];
    __shared__ __align__(16) float s_dy[TT];

    const int tid = threadIdx.x;
    const int jg = tid % NJ;
    const int tg = tid / NJ;
    const int c = blockIdx.x;
    const int s = blockIdx.y;
    const int items = B * tiles_per_row;
    const int it_begin = s * items_per_slice;
    const int it_end = min(items, it_begin + items_per_slice);

    for (int jc = 0; jc < K; jc += KCH) {
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int it = it_begin; it < it_end; ++it) {
            const int b = it / tiles_per_row;
            const int t0 = (it % tiles_per_row) * TT;
            const size_t row = ((size_t)b * (size_t)C + (size_t)c) * (size_t)L;      // VROWS: b is 0
            __syncthreads();
            for (int i = tid; i < TT; i += THREADS) {
                const int t = t0 + i;
                if constexpr (VROWS) {
                    const int e = rows_element(rm, t);
                    s_dy[i] = e >= 0 ? ld_elem(dy + row + e) : 0.f;
                } else {
                    s_dy[i] = (t < L) ? ld_elem(dy + row + t) : 0.f;
                }
            }
            const int g0 = t0 + jc - pad;
            for (int i = tid; i < TT + KCH; i += THREADS) {
                const int g = g0 + i;
                if constexpr (VROWS) {
                    const int e = rows_element(rm, g);
                    s_x[i] = e >= 0 ? ld_elem(x + row + e) : 0.f;
                } else {
                    s_x[i] = (g >= 0 && g < L) ? ld_elem(x + row + g) : 0.f;
                }
            }
            __syncthreads();

            const float *dp = s_dy + tg * SUB;
            const float *xp = s_x + tg * SUB + 4 * jg;
            float win[8];
            {
                const float4 v = *reinterpret_cast<const float4 *>(xp);
                win[0] = v.x; win[1] = v.y; win[2] = v.z; win[3] = v.w;
            }
#pragma unroll 2
            for (int t = 0; t < SUB; t += 4) {
                const float4 nx = *reinterpret_cast<const float4 *>(xp + t + 4);
                const float4 g = *reinterpret_cast<const float4 *>(dp + t);
                win[4] = nx.x; win[5] = nx.y; win[6] = nx.z; win[7] = nx.w;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    acc[jj] = fmaf(g.x, win[jj], acc[jj]);
                    acc[jj] = fmaf(g.y, win[jj + 1], acc[jj]);
                    acc[jj] = fmaf(g.z, win[jj + 2], acc[jj]);
                    acc[jj] = fmaf(g.w, win[jj + 3], acc[jj]);
                }
                win[0] = win[4]; win[1] = win[5]; win[2] = win[6]; win[3] = win[7];
            }
        }
        // ordered cross-thread reduction through LDS: s_x reused as red[NT][KCH]
        __syncthreads();
        *reinterpret_cast<float4 *>(s_x + tg * KCH + 4 * jg) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        __syncthreads();
        for (int j = tid; j < KCH; j += THREADS) {
            if (jc + j < K) {
                float sum = 0.f;
                for (int g = 0; g < NT; ++g) sum += s_x[g * KCH + j];
                part[((size_t)s * (size_t)C + (size_t)c) * (size_t)K + (size_t)(jc + j)] = sum;
            }
        }
    }
}

// dw[i] = sum_{s=0}^{S-1} part[s, i] in increasing s; i over C*K.
template <typename T>
__global__ __launch_bounds__(256) void dw_finalize_kernel(const float *__restrict__ part, T *__restrict__ dw, int S,
                                                          size_t CK)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= CK) return;
    float sum = 0.f;
    int s = 0;
    for (; s + 4 <= S; s += 4) {           // four independent loads in flight, added in slice order
        const float p0 = part[(size_t)s * CK + i], p1 = part[(size_t)(s + 1) * CK + i];
        const float p2 = part[(size_t)(s + 2) * CK + i], p3 = part[(size_t)(s + 3) * CK + i];
        sum = (((sum + p0) + p1) + p2) + p3;
    }
    for (; s < S; ++s) sum += part[(size_t)s * CK + i];
    st_elem(dw + i, sum);
}

// The same sum, in the same order, for many slices of few coefficients (few channels: the slices are what fills the
// chip in stage 1).  One thread per coefficient would wait a memory round trip for every four slices (B6666 C1 L3000 K7,
// 1000 slices: 61 us); here 256 threads bring 128 slices of sixteen coefficients into LDS at a time, and the threads
// that own the coefficients add them in slice order.
template <typename T>
__global__ __launch_bounds__(256) void dw_finalize_many_kernel(const float *__restrict__ part, T *__restrict__ dw, int S,
                                                               size_t CK)
{
    constexpr int NI = 16, TS = 16, U = 8, SB = TS * U;
    __shared__ float buf[SB][NI + 1];
    const int ti = threadIdx.x % NI, ts = threadIdx.x / NI;
    const size_t i = (size_t)blockIdx.x * NI + ti;
    const bool ok = i < CK;
    float sum = 0.f;
    for (int s0 = 0; s0 < S; s0 += SB) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int sl = s0 + ts + TS * u;
            v[u] = (ok && sl < S) ? part[(size_t)sl * CK + i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) buf[ts + TS * u][ti] = v[u];
        __syncthreads();
        if (ts == 0) {
            const int n = S - s0 < SB ? S - s0 : SB;
            for (int k = 0; k < n; ++k) sum += buf[k][ti];
        }
        __syncthreads();
    }
    if (ts == 0 && ok) st_elem(dw + i, sum);
}

}  // namespace dwconv
