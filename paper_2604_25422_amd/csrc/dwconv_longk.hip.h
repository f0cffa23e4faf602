// Matrix-core kernels for filters whose length is of the order of the sequence (K up to 8192,
// L up to 8192): the blocked-Toeplitz form of dwconv_mfma.hip.h with a long loop over block offsets.
//
//   Y[n][r] = sum_{d = dmin..dmax} sum_q Toep_d[r][q] X[n + d][q],   Toep_d[r][q] = w[16 d + q - r + pad]
//
// Here neither the Toeplitz operands (4 registers per offset, hundreds of offsets) nor the inputs fit
// in registers, so a workgroup keeps the whole filter of its channel and whole rows in LDS:
//   forward / input gradient:  grid (C, ceil(B/R)); a workgroup of 16 waves stages w[c,:] (with zero
//       margins) and R rows x[b,c,:] (16-blocks padded to 24 floats, 15 zero blocks on both sides;
//       R = 2 for rows of 8192, more for shorter rows so that the waves have about 32 (row pair, tile) items
//       to share).  A wave owns items in alternating order (longk_item), which balances the
//       triangular cost of a causal filter, and for each walks d over the offsets that touch the row:
//       4 LDS dwords of Toeplitz operand, one 16-byte LDS read per row, 4 matrix instructions per row.
//   weight gradient: see dw_longk_kernel below.
// Sums are fp32; a chain never runs longer than 64 offsets (1024 terms) before it is folded into a
// second accumulator.
#pragma once
#include "dwconv_common.hip.h"
#include "dwconv_mfma.hip.h"

namespace dwconv {

constexpr int kLkWaves = 16;            // waves per workgroup (1024 threads)
constexpr int kLkRows = 2;              // rows staged together
constexpr int kLkMaxBlocks = 512;       // 16-blocks per row: L <= 8192
constexpr int kLkMaxK = 8192;
constexpr int kLkMargin = 15;           // zero 16-blocks on both sides of a staged row
constexpr int kLkWMargin = 48;          // zero taps on both sides of the staged filter
constexpr int kLkFold = 64;             // offsets per inner accumulation chain

struct LongKGeom {
    int B, C, L, K;
    int pad;        // effective pad of this correlation
    int reverse;    // filter index reversed (input gradient)
    int dmin, dmax; // block offsets that can hold a tap
    int NB;         // 16-blocks per row, ceil(L / 16)
    int NT;         // D tiles per row, ceil(NB / 16)
    int R;          // rows staged per workgroup (even): R / 2 row pairs x NT tiles are the items its 16 waves share
};

__host__ __device__ inline int longk_filter_floats(int K) { return (K + 2 * kLkWMargin + 3) & ~3; }
__host__ __device__ inline int longk_row_floats(int NB) { return (NB + 2 * kLkMargin) * kLdsBlockStride; }
inline size_t longk_corr_lds_bytes(int K, int NB, int R)
{
    return sizeof(float) * ((size_t)longk_filter_floats(K) + (size_t)R * longk_row_floats(NB));
}
// Item number `round` of wave `wave`.  Under a causal pad tile t costs about t + 1, so the items (row pair rp, tile t)
// are numbered dearest first, q = (NT - 1 - t) * RP + rp, and dealt to the 16 waves in rounds of 16, every other
// round in reverse order: a wave (and with it a SIMD, which runs waves w, w + 4, ...) that gets a dear tile in one
// round gets a cheap one in the next (one row pair of 32 tiles: tiles 31 - w and w).
__device__ __forceinline__ int longk_item(int round, int wave)
{
    return round * kLkWaves + ((round & 1) ? kLkWaves - 1 - wave : wave);
}

// out[row, t] = sum_j in~[row, t + j - pad] * f_eff[c, j]
template <typename T>
__global__ __launch_bounds__(64 * kLkWaves) void corr_longk_kernel(const T *__restrict__ in, const T *__restrict__ f,
                                                                    T *__restrict__ out, const LongKGeom g)
{
    extern __shared__ __align__(16) float lk_smem[];
    float *fw = lk_smem;                                     // fw[kLkWMargin + j] = f_eff[j], zero outside [0, K)
    float *xr = lk_smem + longk_filter_floats(g.K);
    const int XR = longk_row_floats(g.NB);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15;
    const int k4 = lane >> 4;
    const int c = blockIdx.x;
    const int b0 = blockIdx.y * g.R;

    // ---- stage the filter and the rows
    {
        const T *f_c = f + (size_t)c * (size_t)g.K;
        const int FW = longk_filter_floats(g.K);
        for (int i = tid; i < FW; i += 64 * kLkWaves) {
            const int j = i - kLkWMargin;
            float v = 0.f;
            if (j >= 0 && j < g.K) v = ld_elem(f_c + (g.reverse ? (g.K - 1 - j) : j));
            fw[i] = v;
        }
        for (int rb = 0; rb < g.R; ++rb) {
            float *xrow = xr + rb * XR;
            const int b = b0 + rb;
            // zero margins (16 useful floats of each of the 15 + 15 blocks)
            for (int i = tid; i < 2 * kLkMargin * 16; i += 64 * kLkWaves) {
                const int blk = i >> 4, q = i & 15;
                const int lb = blk < kLkMargin ? blk : g.NB + blk;
                xrow[lb * kLdsBlockStride + q] = 0.f;
            }
            const T *in_row = in + ((size_t)(b < g.B ? b : 0) * (size_t)g.C + (size_t)c) * (size_t)g.L;
            for (int gi = tid; gi < g.NB * 4; gi += 64 * kLkWaves) {
                const int u = 4 * gi;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (b < g.B && u + 3 < g.L) v = ld_elem4(in_row + u);
                *reinterpret_cast<float4 *>(xrow + (kLkMargin + (gi >> 2)) * kLdsBlockStride + (gi & 3) * 4) = v;
            }
        }
    }
    __syncthreads();

    // ---- items of this wave: (row pair, D tile), see longk_item
    const int n_items = (g.R / 2) * g.NT;
    {
        for (int round = 0; round * kLkWaves < n_items; ++round) {
            int item = longk_item(round, wave);
            if (item >= n_items) continue;
            // (a single round: cheapest first, wave w on tile w of one row pair of up to sixteen tiles; the other order
            // measured 3 % slower on B32 C256 L4096 K4096)
            if (n_items <= kLkWaves) item = n_items - 1 - item;
            const int RP = g.R / 2;
            const int t = g.NT - 1 - item / RP, rp = item % RP;
            const int bq = b0 + 2 * rp;                     // first row of the pair
            if (bq >= g.B) continue;
            // offsets d for which some block 16 t + j + d of the tile lies inside the row
            const int dlo = max(g.dmin, -(16 * t + 15));
            const int dhi = min(g.dmax, g.NB - 1 - 16 * t);
            floatx4 tot0 = floatx4{0.f, 0.f, 0.f, 0.f}, tot1 = floatx4{0.f, 0.f, 0.f, 0.f};
            if (dlo <= dhi) {
                // A: lane (r = i16, k4) reads f_eff[16 d + 4 k4 + v - r + pad];  B: lane (j = i16, k4) reads X[16 t + j + d][4 k4 ..]
                const float *ap = fw + kLkWMargin + 16 * dlo + 4 * k4 - i16 + g.pad;
                const float *bp = xr + 2 * rp * XR + (kLkMargin + 16 * t + i16 + dlo) * kLdsBlockStride + 4 * k4;
                for (int d0 = dlo; d0 <= dhi; d0 += kLkFold) {
                    const int n = min(kLkFold, dhi - d0 + 1);
                    floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
                    for (int i = 0; i < n; ++i) {
                        const float a0 = ap[0], a1 = ap[1], a2 = ap[2], a3 = ap[3];
                        const float4 x0 = *reinterpret_cast<const float4 *>(bp);
                        const float4 x1 = *reinterpret_cast<const float4 *>(bp + XR);
                        acc0 = mfma16x16x4(a0, x0.x, acc0);
                        acc1 = mfma16x16x4(a0, x1.x, acc1);
                        acc0 = mfma16x16x4(a1, x0.y, acc0);
                        acc1 = mfma16x16x4(a1, x1.y, acc1);
                        acc0 = mfma16x16x4(a2, x0.z, acc0);
                        acc1 = mfma16x16x4(a2, x1.z, acc1);
                        acc0 = mfma16x16x4(a3, x0.w, acc0);
                        acc1 = mfma16x16x4(a3, x1.w, acc1);
                        ap += 16;
                        bp += kLdsBlockStride;
                    }
                    tot0 += acc0;
                    tot1 += acc1;
                }
            }
            // lane (block j = i16, row group k4) owns outputs 16 j + 4 k4 + 0..3 of the tile
            const int to = 256 * t + 16 * i16 + 4 * k4;
            if (to + 3 < g.L) {
                T *o0 = out + ((size_t)bq * (size_t)g.C + (size_t)c) * (size_t)g.L + to;
                st_elem4(o0, make_float4(tot0[0], tot0[1], tot0[2], tot0[3]));
                if (bq + 1 < g.B)
                    st_elem4(o0 + (size_t)g.C * (size_t)g.L, make_float4(tot1[0], tot1[1], tot1[2], tot1[3]));
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Filters or rows beyond what LDS holds whole (K or L above 8192): the same kernel in tiles.
// A workgroup owns one PIECE of 4096 outputs of a row pair and walks the filter in CHUNKS of 4096 taps.  For chunk ck
// the operator restricted to taps [4096 ck, 4096 ck + 4096) is the operator of a 4096-tap filter with pad
// pad - 4096 ck (any integer: the block offsets that can hold one of its taps follow from the same inequalities),
// and its contribution to the piece needs the input window of 4096 + 4096 + 30 positions that those offsets reach:
// both are staged (the filter chunk with zero margins, so that the taps of the neighbouring chunks inside its edge
// blocks count as zeros here; the window with zeros outside the row), the sixteen waves add the chunk's
// contribution to the accumulators of their tile (256 outputs x 2 rows), and the next chunk is staged.  A chunk whose
// window misses the row is skipped, so a causal filter costs its triangle, not the square.
constexpr int kLkTilePiece = 4096;                       // outputs per workgroup and row
constexpr int kLkTileChunk = 4096;                       // taps staged at a time
constexpr int kLkTileWinBlocks = kLkTilePiece / 16 + kLkTileChunk / 16 + 4;    // 16-blocks of a staged window (516)

struct LongKTileGeom {
    int B, C, L, K;
    int pad;        // effective pad of this correlation
    int reverse;    // filter index reversed (input gradient)
    int NB;         // 16-blocks per row, ceil(L / 16)
    int NP;         // pieces per row
    int NCK;        // filter chunks
};
inline size_t longk_tiled_lds_bytes()
{
    return sizeof(float) * ((size_t)(kLkTileChunk + 2 * kLkWMargin) + (size_t)kLkRows * kLkTileWinBlocks * kLdsBlockStride);
}

template <typename T>
__global__ __launch_bounds__(64 * kLkWaves) void corr_longk_tiled_kernel(const T *__restrict__ in, const T *__restrict__ f,
                                                                          T *__restrict__ out, const LongKTileGeom g)
{
    extern __shared__ __align__(16) float lkt_smem[];
    constexpr int FWT = kLkTileChunk + 2 * kLkWMargin;
    constexpr int XR = kLkTileWinBlocks * kLdsBlockStride;
    float *fw = lkt_smem;                                    // fw[kLkWMargin + jj] = tap 4096 ck + jj, zero outside the chunk
    float *xr = lkt_smem + FWT;                              // two staged windows

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int t = __builtin_amdgcn_readfirstlane(tid >> 6);     // the wave's tile of the piece
    const int i16 = lane & 15;
    const int k4 = lane >> 4;
    const int c = blockIdx.x;
    const int a = g.NP - 1 - (int)(blockIdx.y % (unsigned)g.NP);     // piece (the dear ones of a causal filter first)
    const int b0 = 2 * (int)(blockIdx.y / (unsigned)g.NP);
    const int n0 = (kLkTilePiece / 16) * a + 16 * t;                 // row block of the tile's first output block
    const T *f_c = f + (size_t)c * (size_t)g.K;

    floatx4 tot0 = floatx4{0.f, 0.f, 0.f, 0.f}, tot1 = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int ck = 0; ck < g.NCK; ++ck) {
        const int klen = min(kLkTileChunk, g.K - ck * kLkTileChunk);
        const int padc = g.pad - ck * kLkTileChunk;
        // block offsets that can hold a tap of the chunk (arithmetic shifts: floor division)
        const int dminc = -((padc + 15) >> 4), dmaxc = (klen - padc + 14) >> 4;
        const int wlo = (kLkTilePiece / 16) * a + dminc;             // row block of window block 0
        const int nwb = kLkTilePiece / 16 + (dmaxc - dminc);         // window blocks
        if (wlo + nwb - 1 < 0 || wlo >= g.NB) continue;              // the window misses the row (block-uniform)
        __syncthreads();                                             // everyone is done with the previous chunk
        for (int i = tid; i < FWT; i += 64 * kLkWaves) {
            const int jj = i - kLkWMargin;
            float v = 0.f;
            if (jj >= 0 && jj < klen) {
                const int j = ck * kLkTileChunk + jj;
                v = ld_elem(f_c + (g.reverse ? (g.K - 1 - j) : j));
            }
            fw[i] = v;
        }
        for (int rb = 0; rb < kLkRows; ++rb) {
            float *xrow = xr + rb * XR;
            const int b = b0 + rb;
            const T *in_row = in + ((size_t)(b < g.B ? b : 0) * (size_t)g.C + (size_t)c) * (size_t)g.L;
            for (int gi = tid; gi < nwb * 4; gi += 64 * kLkWaves) {
                const int m = wlo + (gi >> 2);
                const int u = 16 * m + 4 * (gi & 3);
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (b < g.B && m >= 0 && u + 3 < g.L) v = ld_elem4(in_row + u);
                *reinterpret_cast<float4 *>(xrow + (gi >> 2) * kLdsBlockStride + (gi & 3) * 4) = v;
            }
        }
        __syncthreads();
        // offsets for which some block n0 + j + d of the tile lies inside the row
        const int dlo = max(dminc, -(n0 + 15));
        const int dhi = min(dmaxc, g.NB - 1 - n0);
        if (dlo <= dhi && b0 < g.B) {
            // A: lane (r = i16, k4) reads chunk tap 16 d + 4 k4 + v - r + padc;  B: lane (j = i16, k4) reads window block 16 t + j + d - dminc
            const float *ap = fw + kLkWMargin + 16 * dlo + 4 * k4 - i16 + padc;
            const float *bp = xr + (16 * t + i16 + (dlo - dminc)) * kLdsBlockStride + 4 * k4;
            for (int d0 = dlo; d0 <= dhi; d0 += kLkFold) {
                const int n = min(kLkFold, dhi - d0 + 1);
                floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
                for (int i = 0; i < n; ++i) {
                    const float a0 = ap[0], a1 = ap[1], a2 = ap[2], a3 = ap[3];
                    const float4 x0 = *reinterpret_cast<const float4 *>(bp);
                    const float4 x1 = *reinterpret_cast<const float4 *>(bp + XR);
                    acc0 = mfma16x16x4(a0, x0.x, acc0);
                    acc1 = mfma16x16x4(a0, x1.x, acc1);
                    acc0 = mfma16x16x4(a1, x0.y, acc0);
                    acc1 = mfma16x16x4(a1, x1.y, acc1);
                    acc0 = mfma16x16x4(a2, x0.z, acc0);
                    acc1 = mfma16x16x4(a2, x1.z, acc1);
                    acc0 = mfma16x16x4(a3, x0.w, acc0);
                    acc1 = mfma16x16x4(a3, x1.w, acc1);
                    ap += 16;
                    bp += kLdsBlockStride;
                }
                tot0 += acc0;
                tot1 += acc1;
            }
        }
    }
    // lane (block j = i16, row group k4) owns outputs 16 j + 4 k4 + 0..3 of the tile
    const int to = 16 * n0 + 16 * i16 + 4 * k4;
    if (b0 < g.B && to + 3 < g.L) {
        T *o0 = out + ((size_t)b0 * (size_t)g.C + (size_t)c) * (size_t)g.L + to;
        st_elem4(o0, make_float4(tot0[0], tot0[1], tot0[2], tot0[3]));
        if (b0 + 1 < g.B) st_elem4(o0 + (size_t)g.C * (size_t)g.L, make_float4(tot1[0], tot1[1], tot1[2], tot1[3]));
    }
}

// ------------------------------------------------------------------------------------------------
// The same correlation for bf16 storage on the bf16 matrix instruction (v_mfma_f32_16x16x16_bf16): one
// instruction covers a whole block offset of one row (products of two bf16 are exact in fp32, sums fp32, one
// rounding at the store), so per offset a wave issues kLkRows instructions instead of 4 kLkRows.
// LDS holds raw bf16:
//   rows: 16-blocks of 32 bytes padded to 48 (as in corr_mfma_bf16_kernel), 15 zero blocks on both sides;
//   filter: FOUR copies, copy s shifted by s taps (copy_s[i] = fw[i + s]), because lane (r, kg) needs the four
//       consecutive taps fw[a .. a + 3], a = 16 d + 4 kg - r + pad (+ margin), as one aligned 8-byte read and
//       a mod 4 depends on the lane only: it reads copy (a mod 4) at a - (a mod 4), and a grows by 16 per offset.
//       The copies start 64 bytes apart modulo 256, which puts the sixteen r of a read on different banks.
constexpr int kLkBf16CopyPad = 32;         // bf16 elements: makes the stride of the copies 64 bytes modulo 256
__host__ __device__ constexpr int longk_bf16_copy_elems(int K)
{
    const int n = (K + 2 * kLkWMargin + 3) & ~3;                  // taps with margins, whole 8-byte granules
    return (n + 127) / 128 * 128 + kLkBf16CopyPad;                // stride = 64 bytes mod 256
}
__host__ __device__ inline int longk_bf16_row_bytes(int NB) { return (NB + 2 * kLkMargin) * kBf16BlockBytes; }
inline size_t longk_corr_bf16_lds_bytes(int K, int NB, int R)
{
    return (size_t)4 * longk_bf16_copy_elems(K) * 2 + (size_t)R * longk_bf16_row_bytes(NB);
}

template <int UNUSED = 0>   // (a template only so that the header can be included by several translation units)
__global__ __launch_bounds__(64 * kLkWaves) void corr_longk_bf16_kernel(const bf16_t *__restrict__ in,
                                                                         const bf16_t *__restrict__ f,
                                                                         bf16_t *__restrict__ out, const LongKGeom g)
{
    extern __shared__ __align__(16) unsigned char lkb_smem[];
    const int CE = longk_bf16_copy_elems(g.K);
    uint16_t *fwc = reinterpret_cast<uint16_t *>(lkb_smem);      // copy s at fwc + s * CE
    unsigned char *xr = lkb_smem + (size_t)4 * CE * 2;
    const int XR = longk_bf16_row_bytes(g.NB);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15;
    const int kg = lane >> 4;
    const int c = blockIdx.x;
    const int b0 = blockIdx.y * g.R;

    // ---- stage the filter copies and the rows
    {
        const bf16_t *f_c = f + (size_t)c * (size_t)g.K;
        const int FW = (g.K + 2 * kLkWMargin + 3) & ~3;
        for (int i = tid; i < 4 * FW; i += 64 * kLkWaves) {
            const int s = i / FW, e = i - s * FW;
            const int j = e + s - kLkWMargin;
            uint16_t v = 0;
            if (j >= 0 && j < g.K) v = f_c[g.reverse ? (g.K - 1 - j) : j].bits;
            fwc[s * CE + e] = v;
        }
        for (int rb = 0; rb < g.R; ++rb) {
            unsigned char *xrow = xr + rb * XR;
            const int b = b0 + rb;
            // zero margins (the 32 useful bytes of each of the 15 + 15 blocks, 8 bytes at a time)
            for (int i = tid; i < 2 * kLkMargin * 4; i += 64 * kLkWaves) {
                const int blk = i >> 2, q = i & 3;
                const int lb = blk < kLkMargin ? blk : g.NB + blk;
                *reinterpret_cast<uint2 *>(xrow + lb * kBf16BlockBytes + 8 * q) = make_uint2(0u, 0u);
            }
            const bf16_t *in_row = in + ((size_t)(b < g.B ? b : 0) * (size_t)g.C + (size_t)c) * (size_t)g.L;
            for (int gi = tid; gi < g.NB * 4; gi += 64 * kLkWaves) {
                const int u = 4 * gi;
                uint2 v = make_uint2(0u, 0u);
                if (b < g.B && u + 3 < g.L) v = *reinterpret_cast<const uint2 *>(in_row + u);
                *reinterpret_cast<uint2 *>(xrow + (kLkMargin + (gi >> 2)) * kBf16BlockBytes + (gi & 3) * 8) = v;
            }
        }
    }
    __syncthreads();

    // this lane's filter copy: a = kLkWMargin + 16 d + 4 kg - i16 + pad, copy a & 3 read at a - (a & 3)
    const int a0 = kLkWMargin + 4 * kg - i16 + g.pad;             // at d = 0; 16 d keeps a & 3
    const int sh = a0 & 3;
    const uint16_t *acopy = fwc + sh * CE + (a0 - sh);

    // ---- items of this wave: (row pair, D tile), see longk_item
    const int n_items = (g.R / 2) * g.NT;
    {
        for (int round = 0; round * kLkWaves < n_items; ++round) {
            int item = longk_item(round, wave);
            if (item >= n_items) continue;
            // (a single round: cheapest first, wave w on tile w of one row pair of up to sixteen tiles; the other order
            // measured 3 % slower on B32 C256 L4096 K4096)
            if (n_items <= kLkWaves) item = n_items - 1 - item;
            const int RP = g.R / 2;
            const int t = g.NT - 1 - item / RP, rp = item % RP;
            const int bq = b0 + 2 * rp;                     // first row of the pair
            if (bq >= g.B) continue;
            // offsets d for which some block 16 t + j + d of the tile lies inside the row
            const int dlo = max(g.dmin, -(16 * t + 15));
            const int dhi = min(g.dmax, g.NB - 1 - 16 * t);
            floatx4 tot0 = floatx4{0.f, 0.f, 0.f, 0.f}, tot1 = floatx4{0.f, 0.f, 0.f, 0.f};
            if (dlo <= dhi) {
                // A: lane (r = i16, kg) reads taps 16 d + 4 kg + e - r + pad;  B: lane (j = i16, kg) reads X[16 t + j + d][4 kg ..]
                const uint16_t *ap = acopy + 16 * dlo;
                const unsigned char *bp = xr + 2 * rp * XR + (kLkMargin + 16 * t + i16 + dlo) * kBf16BlockBytes + 8 * kg;
                for (int d0 = dlo; d0 <= dhi; d0 += kLkFold) {
                    const int n = min(kLkFold, dhi - d0 + 1);
                    floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = floatx4{0.f, 0.f, 0.f, 0.f};
                    // (one offset per trip, latency hidden by the four waves of a SIMD: four offsets per trip with all
                    // twelve reads issued first measured 429 us instead of 224 us on B8 C256 L8192 K8192, two offsets
                    // per trip on two register sets with the reads of one issued ahead of the other's instructions 266 us)
#pragma unroll 1
                    for (int i = 0; i < n; ++i) {
                        const shortx4 a = *reinterpret_cast<const shortx4 *>(ap);
                        const shortx4 x0 = *reinterpret_cast<const shortx4 *>(bp);
                        const shortx4 x1 = *reinterpret_cast<const shortx4 *>(bp + XR);
                        acc0 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, x0, acc0, 0, 0, 0);
                        acc1 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, x1, acc1, 0, 0, 0);
                        ap += 16;
                        bp += kBf16BlockBytes;
                    }
                    tot0 += acc0;
                    tot1 += acc1;
                }
            }
            // lane (block j = i16, row group kg) owns outputs 16 j + 4 kg + 0..3 of the tile
            const int to = 256 * t + 16 * i16 + 4 * kg;
            if (to + 3 < g.L) {
                bf16_t *o0 = out + ((size_t)bq * (size_t)g.C + (size_t)c) * (size_t)g.L + to;
                st_elem4(o0, make_float4(tot0[0], tot0[1], tot0[2], tot0[3]));
                if (bq + 1 < g.B)
                    st_elem4(o0 + (size_t)g.C * (size_t)g.L, make_float4(tot1[0], tot1[1], tot1[2], tot1[3]));
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// bf16 storage beyond what LDS holds whole: the tiles of corr_longk_tiled_kernel (pieces of 4096 outputs of a row pair,
// filter chunks of 4096 taps with pad - 4096 ck) on the operands of corr_longk_bf16_kernel (four shifted copies of the
// filter chunk, raw bf16 window blocks of 48 bytes, one v_mfma_f32_16x16x16_bf16 per block offset and row).
inline size_t longk_tiled_bf16_lds_bytes()
{
    return (size_t)4 * longk_bf16_copy_elems(kLkTileChunk) * 2 + (size_t)kLkRows * kLkTileWinBlocks * kBf16BlockBytes;
}

template <int UNUSED = 0>   // (a template only so that the header can be included by several translation units)
__global__ __launch_bounds__(64 * kLkWaves) void corr_longk_tiled_bf16_kernel(const bf16_t *__restrict__ in,
                                                                               const bf16_t *__restrict__ f,
                                                                               bf16_t *__restrict__ out, const LongKTileGeom g)
{
    extern __shared__ __align__(16) unsigned char lktb_smem[];
    constexpr int CE = longk_bf16_copy_elems(kLkTileChunk);
    constexpr int FW = (kLkTileChunk + 2 * kLkWMargin + 3) & ~3;
    constexpr int XR = kLkTileWinBlocks * kBf16BlockBytes;
    uint16_t *fwc = reinterpret_cast<uint16_t *>(lktb_smem);     // copy s at fwc + s * CE: copy_s[e] = chunk tap e + s - margin
    unsigned char *xr = lktb_smem + (size_t)4 * CE * 2;          // two staged windows

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int t = __builtin_amdgcn_readfirstlane(tid >> 6);      // the wave's tile of the piece
    const int i16 = lane & 15;
    const int kg = lane >> 4;
    const int c = blockIdx.x;
    const int a = g.NP - 1 - (int)(blockIdx.y % (unsigned)g.NP);     // piece (the dear ones of a causal filter first)
    const int b0 = 2 * (int)(blockIdx.y / (unsigned)g.NP);
    const int n0 = (kLkTilePiece / 16) * a + 16 * t;                 // row block of the tile's first output block
    const bf16_t *f_c = f + (size_t)c * (size_t)g.K;

    floatx4 tot0 = floatx4{0.f, 0.f, 0.f, 0.f}, tot1 = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int ck = 0; ck < g.NCK; ++ck) {
        const int klen = min(kLkTileChunk, g.K - ck * kLkTileChunk);
        const int padc = g.pad - ck * kLkTileChunk;
        const int dminc = -((padc + 15) >> 4), dmaxc = (klen - padc + 14) >> 4;     // (arithmetic shifts: floor division)
        const int wlo = (kLkTilePiece / 16) * a + dminc;             // row block of window block 0
        const int nwb = kLkTilePiece / 16 + (dmaxc - dminc);         // window blocks
        if (wlo + nwb - 1 < 0 || wlo >= g.NB) continue;              // the window misses the row (block-uniform)
        __syncthreads();                                             // everyone is done with the previous chunk
        for (int i = tid; i < 4 * FW; i += 64 * kLkWaves) {
            const int s = i / FW, e = i - s * FW;
            const int jj = e + s - kLkWMargin;
            uint16_t v = 0;
            if (jj >= 0 && jj < klen) {
                const int j = ck * kLkTileChunk + jj;
                v = f_c[g.reverse ? (g.K - 1 - j) : j].bits;
            }
            fwc[s * CE + e] = v;
        }
        for (int rb = 0; rb < kLkRows; ++rb) {
            unsigned char *xrow = xr + rb * XR;
            const int b = b0 + rb;
            const bf16_t *in_row = in + ((size_t)(b < g.B ? b : 0) * (size_t)g.C + (size_t)c) * (size_t)g.L;
            for (int gi = tid; gi < nwb * 4; gi += 64 * kLkWaves) {
                const int m = wlo + (gi >> 2);
                const int u = 16 * m + 4 * (gi & 3);
                uint2 v = make_uint2(0u, 0u);
                if (b < g.B && m >= 0 && u + 3 < g.L) v = *reinterpret_cast<const uint2 *>(in_row + u);
                *reinterpret_cast<uint2 *>(xrow + (gi >> 2) * kBf16BlockBytes + (gi & 3) * 8) = v;
            }
        }
        __syncthreads();
        // offsets for which some block n0 + j + d of the tile lies inside the row
        const int dlo = max(dminc, -(n0 + 15));
        const int dhi = min(dmaxc, g.NB - 1 - n0);
        if (dlo <= dhi && b0 < g.B) {
            // A: lane (r = i16, kg) needs chunk taps 16 d + 4 kg + e - r + padc, e = 0..3: copy (a0 & 3) read at a0 - (a0 & 3),
            // a0 = margin + 4 kg - r + padc (16 d keeps a0 & 3);  B: lane (j = i16, kg) reads window block 16 t + j + d - dminc
            const int a0 = kLkWMargin + 4 * kg - i16 + padc;
            const int sh = a0 & 3;
            const uint16_t *ap = fwc + sh * CE + (a0 - sh) + 16 * dlo;
            const unsigned char *bp = xr + (16 * t + i16 + (dlo - dminc)) * kBf16BlockBytes + 8 * kg;
            for (int d0 = dlo; d0 <= dhi; d0 += kLkFold) {
                const int n = min(kLkFold, dhi - d0 + 1);
                floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
                for (int i = 0; i < n; ++i) {
                    const shortx4 av = *reinterpret_cast<const shortx4 *>(ap);
                    const shortx4 x0 = *reinterpret_cast<const shortx4 *>(bp);
                    const shortx4 x1 = *reinterpret_cast<const shortx4 *>(bp + XR);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, x0, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, x1, acc1, 0, 0, 0);
                    ap += 16;
                    bp += kBf16BlockBytes;
                }
                tot0 += acc0;
                tot1 += acc1;
            }
        }
    }
    // lane (block j = i16, row group kg) owns outputs 16 j + 4 kg + 0..3 of the tile
    const int to = 16 * n0 + 16 * i16 + 4 * kg;
    if (b0 < g.B && to + 3 < g.L) {
        bf16_t *o0 = out + ((size_t)b0 * (size_t)g.C + (size_t)c) * (size_t)g.L + to;
        st_elem4(o0, make_float4(tot0[0], tot0[1], tot0[2], tot0[3]));
        if (b0 + 1 < g.B) st_elem4(o0 + (size_t)g.C * (size_t)g.L, make_float4(tot1[0], tot1[1], tot1[2], tot1[3]));
    }
}

// ------------------------------------------------------------------------------------------------
// Stage 1 of the weight gradient for long filters (eq. (dk_def)):
//     G_d[q'][q] = sum_b sum_n X[n + d][q'] dY[n][q],      dw[j] = sum over 16 d + q' - q + pad = j.
// There are hundreds of offsets d, each with a 16x16 accumulator, so the offsets are what is split
// over waves: they are cut into contiguous groups of at most GD offsets and every one of the
// W = 16 * gridDim.y wave slots of a channel owns at most two groups.  An offset far from lag 0 reaches
// the row in few chunks, one near lag 0 in all of them, so the host sizes the groups and pairs heavy with
// light ones until the slots carry about equal work (LongKDwTable).  A workgroup stages two rows of x (256 zero floats on both
// sides) and of dY at a time; a wave walks the 64-position chunks that its groups can touch: one LDS
// dword of dY and, per offset, one of x feed one matrix instruction.  At the end each wave sums the
// diagonals of its accumulators into the taps of its groups and stores them into slice (group & 1)
// of the partial tensor: groups of equal parity own disjoint taps, so nothing is added in memory;
// the slices are zero-filled beforehand by fill_zero_kernel and summed by the ordinary stage 2.
constexpr int kLkDwMargin = 256;        // zero floats on both sides of a staged x row
constexpr int kLkDwMaxGD = 9;           // offsets per group (4 accumulator registers each, two groups per wave)

struct LongKDwGeom {
    int B, C, L, K, pad;
    int dmin, dmax;
    int NCH;        // 64-position chunks per row
    int bper;       // batch entries per batch slice (a multiple of the rows staged together): workgroup (c, y, z) walks
                    // entries z * bper .. and writes the slices 2 z and 2 z + 1, so that few channels or few offsets
                    // still fill the chip
};

// Which offsets a wave slot owns.  The block offsets dmin..dmax are cut into contiguous groups of 1..9 offsets
// (group i: offsets da[i] .. da[i] + n[i] - 1, in increasing order of i); every wave slot owns at most two groups.
// The host balances the work (offsets near the edge of the filter reach the row in few chunks, offsets near lag 0
// in all of them) and passes the table by value with the launch.
constexpr int kLkDwMaxGroups = 128;
constexpr int kLkDwMaxSlots = 64;
constexpr unsigned char kLkDwNoGroup = 255;
struct LongKDwTable {
    short da[kLkDwMaxGroups];
    unsigned char n[kLkDwMaxGroups];
    unsigned char g0[kLkDwMaxSlots], g1[kLkDwMaxSlots];
};

inline size_t longk_dw_lds_bytes(int L, int NCH)
{
    const size_t stage = sizeof(float) * (size_t)kLkRows * ((size_t)((L + 2 * kLkDwMargin + 3) & ~3) + (size_t)NCH * 64);
    const size_t reduce = sizeof(float) * (size_t)kLkWaves * (256 + 16 * kLkDwMaxGD + 32);   // epilogue scratch of every wave
    return stage > reduce ? stage : reduce;
}

__device__ __forceinline__ int floor_div(int a, int b) { return (a >= 0) ? a / b : -((-a + b - 1) / b); }
__device__ __forceinline__ int ceil_div(int a, int b) { return -floor_div(-a, b); }

template <int UNUSED = 0>   // (a template only so that the header can be included by several translation units)
__global__ __launch_bounds__(256) void fill_zero_kernel(float *__restrict__ p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0.f;
}

// The chunks [ch_lo, ch_hi] of one staged row for a group of N offsets.
template <int N, int GD>
__device__ __forceinline__ void lk_dw_chunks(floatx4 (&G)[GD], const float *xp, const float *gp, int ch_lo, int ch_hi)
{
#pragma unroll 2
    for (int ch = ch_lo; ch <= ch_hi; ++ch) {
        const float gq = gp[64 * ch];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const float xa = xp[64 * ch + 16 * i];
            G[i] = mfma16x16x4(xa, gq, G[i]);
        }
    }
}
// ... for a group size known at run time (wave-uniform)
template <int GD, int N = GD>
__device__ __forceinline__ void lk_dw_chunks_n(int n, floatx4 (&G)[GD], const float *xp, const float *gp, int ch_lo, int ch_hi)
{
    if (n == N) lk_dw_chunks<N, GD>(G, xp, gp, ch_lo, ch_hi);
    else if constexpr (N > 1) lk_dw_chunks_n<GD, N - 1>(n, G, xp, gp, ch_lo, ch_hi);
}

template <typename T, int GD>
__global__ __launch_bounds__(64 * kLkWaves, 4) void dw_longk_kernel(const T *__restrict__ x, const T *__restrict__ dy,
                                                                     float *__restrict__ part, const LongKDwGeom g,
                                                                     const LongKDwTable tb)
{
    extern __shared__ __align__(16) float lk_smem[];
    const int XW = (g.L + 2 * kLkDwMargin + 3) & ~3;        // floats of one staged x row
    const int GW = g.NCH * 64;                              // floats of one staged dY row
    float *sx = lk_smem;                                    // sx[rb * XW + kLkDwMargin + u] = x[u]
    float *sg = lk_smem + kLkRows * XW;                     // sg[rb * GW + t] = dy[t]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = blockIdx.x;
    const int slot = (int)blockIdx.y * kLkWaves + wave;

    // the two groups of this wave: offsets [da, db] inclusive, empty if da > db
    int grp[2], da[2], db[2], nn[2], ch_lo[2], ch_hi[2];
    grp[0] = tb.g0[slot];
    grp[1] = tb.g1[slot];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const bool valid = grp[k] != kLkDwNoGroup;
        const int gi = valid ? grp[k] : 0;
        nn[k] = valid ? min((int)tb.n[gi], GD) : 0;
        da[k] = tb.da[gi];
        db[k] = da[k] + nn[k] - 1;
        // chunks in which some offset of the group reaches the row
        ch_lo[k] = max(0, ceil_div(-63 - 16 * db[k], 64));
        ch_hi[k] = valid ? min(g.NCH - 1, floor_div(g.L - 1 - 16 * da[k], 64)) : -1;
    }

    floatx4 G0[GD], G1[GD];
#pragma unroll
    for (int i = 0; i < GD; ++i) {
        G0[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        G1[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    const int b_begin = (int)blockIdx.z * g.bper, b_end = min(g.B, b_begin + g.bper);
    for (int b0 = b_begin; b0 < b_end; b0 += kLkRows) {
        __syncthreads();
        for (int rb = 0; rb < kLkRows; ++rb) {
            const int b = b0 + rb;
            float *xrow = sx + rb * XW;
            float *grow = sg + rb * GW;
            const size_t row = ((size_t)(b < b_end ? b : 0) * (size_t)g.C + (size_t)c) * (size_t)g.L;
            for (int i = tid; i < 2 * kLkDwMargin; i += 64 * kLkWaves)
                xrow[i < kLkDwMargin ? i : g.L + i] = 0.f;
            for (int gi0 = tid; gi0 < g.NCH * 16; gi0 += 64 * kLkWaves) {
                // (addresses recomputed from gi every trip rather than kept as induction variables across the whole
                // kernel, next to the accumulators)
                int gi = gi0;
                asm volatile("" : "+v"(gi));
                const int u = 4 * gi;
                float4 vx = make_float4(0.f, 0.f, 0.f, 0.f), vg = vx;
                if (b < b_end && u + 3 < g.L) {
                    vx = ld_elem4(x + row + u);
                    vg = ld_elem4(dy + row + u);
                }
                if (u + 3 < g.L) *reinterpret_cast<float4 *>(xrow + kLkDwMargin + u) = vx;
                *reinterpret_cast<float4 *>(grow + u) = vg;
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            for (int rb = 0; rb < kLkRows; ++rb) {
                // A operand: X[n0 + kk + d][q'] = sx[64 ch + 16 d + lane];  B operand: dY[n0 + kk][q] = sg[64 ch + lane]
                const float *xp = sx + rb * XW + kLkDwMargin + 16 * da[k] + lane;
                const float *gp = sg + rb * GW + lane;
                if (k == 0) lk_dw_chunks_n<GD>(nn[0], G0, xp, gp, ch_lo[0], ch_hi[0]);
                else lk_dw_chunks_n<GD>(nn[1], G1, xp, gp, ch_lo[1], ch_hi[1]);
            }
        }
    }

    // ---- diagonal sums.  Wave-private scratch in the (now free) x region: 256 floats of one
    // accumulator plus the taps of one group, tap T = 16 i + e + 15 for offset da + i, e = q' - q.
    __syncthreads();
    constexpr int NTAP = 16 * GD + 32;
    float *scr = lk_smem + wave * (256 + NTAP);
    float *tap = scr + 256;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        if (da[k] > db[k]) continue;
        for (int i = lane; i < NTAP; i += 64) tap[i] = 0.f;
        wave_lds_fence();
#pragma unroll
        for (int i = 0; i < GD; ++i) {
            const floatx4 Gi = (k == 0) ? G0[i] : G1[i];
#pragma unroll
            for (int v = 0; v < 4; ++v) scr[(4 * (lane >> 4) + v) * 16 + (lane & 15)] = Gi[v];
            wave_lds_fence();
            if (lane < 31) {
                const int e = lane - 15;
                const int q_lo = e > 0 ? e : 0, q_hi = e > 0 ? 15 : 15 + e;
                float sum = 0.f;
                for (int qp = q_lo; qp <= q_hi; ++qp) sum += scr[qp * 16 + (qp - e)];
                if (da[k] + i <= db[k]) tap[16 * i + lane] += sum;     // a short last group owns fewer offsets
            }
            wave_lds_fence();
        }
        const int ntap = 16 * (db[k] - da[k]) + 31;
        float *dst = part + ((size_t)(2 * (int)blockIdx.z + (grp[k] & 1)) * (size_t)g.C + (size_t)c) * (size_t)g.K;
        for (int i = lane; i < ntap; i += 64) {
            const int j = 16 * da[k] + (i - 15) + g.pad;
            if (j >= 0 && j < g.K) dst[j] = tap[i];
        }
        wave_lds_fence();
    }
}

// ------------------------------------------------------------------------------------------------
// The same stage 1 for bf16 storage on the bf16 matrix instruction (v_mfma_f32_16x16x16_bf16): the contraction of
// one instruction runs over 16 consecutive blocks n, so a chunk is 256 positions and a wave issues a quarter of the
// instructions.  Same groups, same table, same epilogue as dw_longk_kernel (the accumulators have the same lane
// layout).  Lane (i = lane % 16, kg = lane / 16) holds the contraction entries k = 4 kg + v: element i of blocks
// n0 + 4 kg + v (+ d), v = 0..3.  So that these four values are ONE LDS read, the rows are staged transposed:
//     xt[i][m] = x[16 (m - 32) + i]   (16 lines of bf16, one entry per block, 32 zero blocks on both sides),
//     gt[i][n] = dy[16 n + i],
// and the operand of offset d is xt[i][32 + n0 + 4 kg + d .. + 3].  Its alignment is that of d: x is kept twice, the
// second copy shifted by one entry, which makes every operand two aligned dwords (ds_read2_b32); dY needs one copy
// (8-byte aligned).  Lines are 16 bytes modulo 256 apart: the 32 lanes of a half wave then read 64 different banks.
constexpr int kLkDwBf16MarginBlocks = 32;
__host__ __device__ inline int lk_bf16_line_bytes(int entries) { return (2 * entries + 255 - 16) / 256 * 256 + 16; }
inline size_t longk_dw_bf16_lds_bytes(int L)
{
    const int nb = (L + 255) / 256 * 16;                            // blocks per row, whole chunks
    const size_t xcopy = (size_t)16 * lk_bf16_line_bytes(nb + 2 * kLkDwBf16MarginBlocks);
    const size_t stage = (size_t)kLkRows * (2 * xcopy + (size_t)16 * lk_bf16_line_bytes(nb));
    const size_t reduce = sizeof(float) * (size_t)kLkWaves * (256 + 16 * kLkDwMaxGD + 32);
    return stage > reduce ? stage : reduce;
}

typedef __attribute__((address_space(3))) const uint32_t *lds_u32_ptr;
typedef unsigned int lk_uintx2 __attribute__((ext_vector_type(2)));

// The 256-position chunks [ch_lo, ch_hi] of one staged row for a group of N offsets.  The operand of offset da + i is
// the four entries m0 + i .. m0 + i + 3 of this lane's line.  Even i read them from the copy in which m0 is
// dword-aligned (xe: address of entry m0 there), odd i from the other copy (xo: entry m0 + 1): the windows of a copy
// overlap, so a chunk needs (N + 1) / 2 + 1 dwords of one copy and N / 2 + 1 of the other instead of two per
// offset.  ga: the dY operand.  A chunk further is 16 entries = 32 bytes.
template <int N, int GD>
__device__ __forceinline__ void lk_dw_chunks_bf16(floatx4 (&G)[GD], lds_u32_ptr xe, lds_u32_ptr xo, lds_u32_ptr ga,
                                                  int ch_lo, int ch_hi)
{
    constexpr int NE = (N + 1) / 2, NO = N / 2;
#pragma unroll 2
    for (int ch = ch_lo; ch <= ch_hi; ++ch) {
        const lk_uintx2 bw = {ga[8 * ch], ga[8 * ch + 1]};
        const shortx4 bq = __builtin_bit_cast(shortx4, bw);
        unsigned e[NE + 1], o[NO + 1];
#pragma unroll
        for (int t = 0; t <= NE; ++t) e[t] = xe[8 * ch + t];
#pragma unroll
        for (int t = 0; t <= NO; ++t) o[t] = NO > 0 ? xo[8 * ch + t] : 0u;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const lk_uintx2 aw = (i & 1) ? lk_uintx2{o[i / 2], o[i / 2 + 1]} : lk_uintx2{e[i / 2], e[i / 2 + 1]};
            G[i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, aw), bq, G[i], 0, 0, 0);
        }
    }
}
template <int GD, int N = GD>
__device__ __forceinline__ void lk_dw_chunks_bf16_n(int n, floatx4 (&G)[GD], lds_u32_ptr xe, lds_u32_ptr xo, lds_u32_ptr ga,
                                                    int ch_lo, int ch_hi)
{
    if (n == N) lk_dw_chunks_bf16<N, GD>(G, xe, xo, ga, ch_lo, ch_hi);
    else if constexpr (N > 1) lk_dw_chunks_bf16_n<GD, N - 1>(n, G, xe, xo, ga, ch_lo, ch_hi);
}

template <int GD>
__global__ __launch_bounds__(64 * kLkWaves, 4) void dw_longk_bf16_kernel(const bf16_t *__restrict__ x,
                                                                          const bf16_t *__restrict__ dy,
                                                                          float *__restrict__ part, const LongKDwGeom g,
                                                                          const LongKDwTable tb)
{
    extern __shared__ __align__(16) unsigned char lkb_dw_smem[];
    constexpr int MB = kLkDwBf16MarginBlocks;
    const int NB = (g.L + 255) / 256 * 16;                  // blocks per row, whole chunks
    const int NC256 = NB / 16;
    const int XL = lk_bf16_line_bytes(NB + 2 * MB);         // bytes of one line of a transposed x copy
    const int GL = lk_bf16_line_bytes(NB);                  // ... of transposed dY
    const int XC = 16 * XL;                                 // bytes of one x copy
    const int ROWB = 2 * XC + 16 * GL;                      // bytes of one staged row: x copy 0, x copy 1, dY
    // row rb: x copy s at rb * ROWB + s * XC, entry (i, m) at + i * XL + 2 (m - s);  dY at rb * ROWB + 2 XC + i * GL + 2 n

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, kg = lane >> 4;
    const int c = blockIdx.x;
    const int slot = (int)blockIdx.y * kLkWaves + wave;

    // the two groups of this wave: offsets [da, db] inclusive, empty if da > db
    int grp[2], da[2], db[2], nn[2], ch_lo[2], ch_hi[2];
    grp[0] = tb.g0[slot];
    grp[1] = tb.g1[slot];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const bool valid = grp[k] != kLkDwNoGroup;
        const int gi = valid ? grp[k] : 0;
        nn[k] = valid ? min((int)tb.n[gi], GD) : 0;
        da[k] = tb.da[gi];
        db[k] = da[k] + nn[k] - 1;
        // chunks in which some offset of the group reaches the row: x positions 256 ch + 16 da .. 256 ch + 255 + 16 db
        ch_lo[k] = max(0, ceil_div(-255 - 16 * db[k], 256));
        ch_hi[k] = valid ? min(NC256 - 1, floor_div(g.L - 1 - 16 * da[k], 256)) : -1;
    }

    floatx4 G0[GD], G1[GD];
#pragma unroll
    for (int i = 0; i < GD; ++i) {
        G0[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        G1[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // the margins of the x copies stay zero for the whole kernel: clear the staging region once
    for (int i = tid; i < kLkRows * ROWB / 16; i += 64 * kLkWaves)
        *reinterpret_cast<uint4 *>(lkb_dw_smem + 16 * i) = make_uint4(0u, 0u, 0u, 0u);

    const int b_begin = (int)blockIdx.z * g.bper, b_end = min(g.B, b_begin + g.bper);
    for (int b0 = b_begin; b0 < b_end; b0 += kLkRows) {
        __syncthreads();
        for (int rb = 0; rb < kLkRows; ++rb) {
            const int b = b0 + rb;
            unsigned char *x0 = lkb_dw_smem + rb * ROWB, *gt = x0 + 2 * XC;
            const size_t row = ((size_t)(b < b_end ? b : 0) * (size_t)g.C + (size_t)c) * (size_t)g.L;
#pragma unroll 1
            for (int gi0 = tid; gi0 < NB * 4; gi0 += 64 * kLkWaves) {
                // (the addresses below are recomputed from gi every time: kept as induction variables they would
                // occupy two dozen registers for the whole kernel, next to the accumulators)
                int gi = gi0;
                asm volatile("" : "+v"(gi));
                const int u = 4 * gi;
                uint2 vx = make_uint2(0u, 0u), vg = vx;
                if (b < b_end && u + 3 < g.L) {
                    vx = *reinterpret_cast<const uint2 *>(x + row + u);
                    vg = *reinterpret_cast<const uint2 *>(dy + row + u);
                }
                const int blk = u >> 4, i0 = u & 15;
                const uint16_t ex[4] = {(uint16_t)vx.x, (uint16_t)(vx.x >> 16), (uint16_t)vx.y, (uint16_t)(vx.y >> 16)};
                const uint16_t eg[4] = {(uint16_t)vg.x, (uint16_t)(vg.x >> 16), (uint16_t)vg.y, (uint16_t)(vg.y >> 16)};
                unsigned char *px = x0 + i0 * XL + 2 * (MB + blk), *pg = gt + i0 * GL + 2 * blk;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    *reinterpret_cast<uint16_t *>(px) = ex[e];
                    *reinterpret_cast<uint16_t *>(px + XC - 2) = ex[e];          // the copy shifted by one entry
                    *reinterpret_cast<uint16_t *>(pg) = eg[e];
                    px += XL;
                    pg += GL;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            if (nn[k] == 0) continue;
            for (int rb = 0; rb < kLkRows; ++rb) {
                const unsigned char *x0 = lkb_dw_smem + rb * ROWB;
                // operand of offset da + i: entries m0 + i .. m0 + i + 3, m0 = MB + 4 kg + da; copy s holds entry m at m - s
                const int m0 = MB + 4 * kg + da[k];
                const int sh = m0 & 1;                                   // (wave-uniform: the parity of da)
                const lds_u32_ptr xe = (lds_u32_ptr)(x0 + sh * XC + i16 * XL + 2 * (m0 - sh));
                const lds_u32_ptr xo = (lds_u32_ptr)(x0 + (1 - sh) * XC + i16 * XL + 2 * (m0 + sh));
                const lds_u32_ptr ga = (lds_u32_ptr)(x0 + 2 * XC + i16 * GL + 8 * kg);
                if (k == 0) lk_dw_chunks_bf16_n<GD>(nn[0], G0, xe, xo, ga, ch_lo[0], ch_hi[0]);
                else lk_dw_chunks_bf16_n<GD>(nn[1], G1, xe, xo, ga, ch_lo[1], ch_hi[1]);
            }
        }
    }

    // ---- diagonal sums.  Wave-private scratch in the (now free) staging region: 256 floats of one
    // accumulator plus the taps of one group, tap T = 16 i + e + 15 for offset da + i, e = q' - q.
    __syncthreads();
    constexpr int NTAP = 16 * GD + 32;
    float *scr = reinterpret_cast<float *>(lkb_dw_smem) + wave * (256 + NTAP);
    float *tap = scr + 256;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        if (da[k] > db[k]) continue;
        for (int i = lane; i < NTAP; i += 64) tap[i] = 0.f;
        wave_lds_fence();
#pragma unroll
        for (int i = 0; i < GD; ++i) {
            const floatx4 Gi = (k == 0) ? G0[i] : G1[i];
#pragma unroll
            for (int v = 0; v < 4; ++v) scr[(4 * (lane >> 4) + v) * 16 + (lane & 15)] = Gi[v];
            wave_lds_fence();
            if (lane < 31) {
                const int e = lane - 15;
                const int q_lo = e > 0 ? e : 0, q_hi = e > 0 ? 15 : 15 + e;
                float sum = 0.f;
                for (int qp = q_lo; qp <= q_hi; ++qp) sum += scr[qp * 16 + (qp - e)];
                if (da[k] + i <= db[k]) tap[16 * i + lane] += sum;     // a short last group owns fewer offsets
            }
            wave_lds_fence();
        }
        const int ntap = 16 * (db[k] - da[k]) + 31;
        float *dst = part + ((size_t)(2 * (int)blockIdx.z + (grp[k] & 1)) * (size_t)g.C + (size_t)c) * (size_t)g.K;
        for (int i = lane; i < ntap; i += 64) {
            const int j = 16 * da[k] + (i - 15) + g.pad;
            if (j >= 0 && j < g.K) dst[j] = tap[i];
        }
        wave_lds_fence();
    }
}

}  // namespace dwconv
