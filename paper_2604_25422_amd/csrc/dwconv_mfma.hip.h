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
#include <type_traits>

#include "dwconv_common.hip.h"

namespace dwconv {

typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ floatx4 mfma16x16x4(float a, float b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

constexpr int kLdsBlockStride = 24;   // floats per staged 16-block: 16 + 8 pad, measured conflict-free for the strided b128 reads
constexpr int kSegBlocks = 64;        // 16-blocks per segment: one segment = 1024 positions
constexpr int kSegLen = kSegBlocks * 16;
constexpr int kWavesPerBlock = 4;        // weight-gradient kernel (block-level final reduction)
constexpr int kMfmaWavesPerSimd = 4;      // register budget both kernels are compiled for (512 / 4 = 128 per lane)
constexpr int kCorrWavesPerBlock = 4;    // correlate kernel: waves are independent; neighbours share halos

// Orders LDS traffic of one wave: everything before is visible to every lane after.
// The LDS regions below are private to a wave, so no workgroup barrier is needed.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Geometry the host computes once per call for the correlate kernel.
struct CorrGeom {
    int C, L, K;
    int rows;           // B * C
    int pad;            // effective pad of this correlation
    int reverse;        // filter index reversed (input gradient)
    int dmin;           // first block offset
    int segs_per_row;   // segments of kSegLen outputs per row
    int n_waves;        // waves launched; wave w walks segments w, w + n_waves, ... of the memory order (row, seg)
    int step_rows;      // n_main / walk_segs
    int step_seg;       // n_main % walk_segs
    int step_c;         // step_rows % C
    // Kernels that load rows straight into LDS (the others walk all segments: walk_segs = segs_per_row, n_light = 0,
    // n_main = n_waves).  Waves n_light .. n_waves - 1 walk the first walk_segs segments of every row (step_rows, step_seg
    // and step_c are those of n_main over walk_segs); walk_segs is segs_per_row, or segs_per_row - 1 when the last segment
    // holds so few positions that it gets waves of its own: wave w < n_light takes the last segment of rows w, w + n_light, ...
    int walk_segs;
    int n_main;
    int n_light;
    int step_c_light;   // n_light % C
};

// Row access through buffer instructions.  A buffer resource describes (the tail of) ONE row
// (base, num_records in bytes, stride 0); the hardware range check makes a load whose byte offset
// lies outside [0, num_records) return zero, so the zero padding of the operator costs no
// instructions: an offset before the row start is a negative number, i.e. a huge unsigned one.
//
// The prefetch loads are issued through inline assembly on purpose.  They stay in flight across the
// whole matrix phase of a segment, and the compiler's own wait-count bookkeeping, which has to be
// conservative across the loop back edge, otherwise splits a round of loads with waits on its own
// members (a full memory latency per segment).  Untracked loads need exactly one manual wait, where
// their registers are drained into LDS: s_waitcnt vmcnt(0).  The counter retires in order, so any
// wait the compiler inserts for its own loads and stores only becomes stricter, never wrong.
// On this part every vector-ALU instruction also takes issue time away from the matrix instructions of
// the same SIMD (measured: about 5.5 cycles each), so a window that starts inside the row folds its
// start into the resource (scalar work) and uses per-lane offsets that are loop constants.
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
constexpr unsigned kBufferFlags = 0x00020000u;   // raw buffer, 32-bit data format (gfx9 family)
constexpr int kOutOfRow = 0x40000000;            // byte offset no row reaches (rows are shorter than 2^28 elements): load gives 0

// Resource for the bytes [start, L * sizeof(T)) of a row; start >= 0.  All operands are wave-uniform.
template <typename T>
__device__ __forceinline__ uintx4 row_tail_resource(const T *row, int L, int start)
{
    const unsigned long long a = reinterpret_cast<unsigned long long>(row) + (unsigned long long)start;
    // (a start at or past the end of the row gives an EMPTY resource: a negative size would wrap to a huge one, under
    // which even the out-of-row marker offset is in range)
    const int bytes = L * (int)sizeof(T) - start;
    const uintx4 r = {(unsigned)a, (unsigned)(a >> 32) & 0xffffu, (unsigned)(bytes > 0 ? bytes : 0), kBufferFlags};
    return r;
}

__device__ __forceinline__ uintx4 buffer_load_x4_untracked(uintx4 rsrc, int byte_off)
{
    uintx4 v;
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(v) : "v"(byte_off), "s"(rsrc) : "memory");
    return v;
}
// ... with a compile-time byte offset (0 .. 4095) added by the instruction: one offset register serves several loads
template <int IMM>
__device__ __forceinline__ uintx4 buffer_load_x4_untracked_imm(uintx4 rsrc, int byte_off)
{
    static_assert(IMM >= 0 && IMM < 4096, "12-bit immediate offset");
    uintx4 v;
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:%3" : "=v"(v) : "v"(byte_off), "s"(rsrc), "n"(IMM) : "memory");
    return v;
}
__device__ __forceinline__ uintx2 buffer_load_x2_untracked(uintx4 rsrc, int byte_off)
{
    uintx2 v;
    asm volatile("buffer_load_dwordx2 %0, %1, %2, 0 offen" : "=v"(v) : "v"(byte_off), "s"(rsrc) : "memory");
    return v;
}
// Wait for every outstanding vector-memory operation of the wave, then hand the prefetch registers
// back to the compiler (the empty statements keep their uses below the wait).
__device__ __forceinline__ void wait_untracked_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
template <typename V, int N>
__device__ __forceinline__ void release_after_wait(V (&regs)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(regs[i]));
}

// Byte offset for a buffer load (out of range where the virtual row holds a zero).
template <int ES>
__device__ __forceinline__ int rows_byte_offset(const RowsMap &m, int u)
{
    const int e = rows_element(m, u);
    return e >= 0 ? ES * e : kOutOfRow;
}

// The same for a 16-byte granule of eight 2-byte elements that starts at virtual position u (a multiple of 8; pitch a
// multiple of 8, row length even).  A row whose length is not a multiple of 8 ends inside its last granule: the load
// then brings the first elements of the next row in memory where the virtual row holds zeros.  `live` is the number of
// elements of the granule that belong to the row when that is the case (2, 4 or 6), 8 otherwise; the lane clears the
// rest of its LDS slot once the load has landed (zero_slot_tail).
__device__ __forceinline__ int rows_granule8_byte_offset(const RowsMap &m, int u, int &live)
{
    const int b = (int)__umulhi((unsigned)u, m.M);
    const int t = u - b * m.P;
    const bool in = (unsigned)u < (unsigned)m.Lv && t < m.L;
    const int left = m.L - t;
    live = (in && left < 8) ? left : 8;
    return in ? 2 * (b * m.CL + t) : kOutOfRow;
}
// Clear the dwords of a 16-byte LDS slot from element `live` on (live = 2, 4, 6; 8: nothing).  Ordinary LDS stores:
// they stay behind the wait that precedes them and ahead of the operand reads that follow them in program order.
__device__ __forceinline__ void zero_slot_tail(const short *slot, int live)
{
    if (live < 8) {
        unsigned *p = reinterpret_cast<unsigned *>(const_cast<short *>(slot));
        if (live <= 2) p[1] = 0u;
        if (live <= 4) p[2] = 0u;
        p[3] = 0u;
    }
}
// The same for fp32 rows of any length (pitch a multiple of 4): a 16-byte granule of four floats that starts at virtual
// position u (a multiple of 4); `live` = 1, 2 or 3 when a row ends inside it, 4 otherwise.
__device__ __forceinline__ int rows_granule4_byte_offset(const RowsMap &m, int u, int &live)
{
    const int b = (int)__umulhi((unsigned)u, m.M);
    const int t = u - b * m.P;
    const bool in = (unsigned)u < (unsigned)m.Lv && t < m.L;
    const int left = m.L - t;
    live = (in && left < 4) ? left : 4;
    return in ? 4 * (b * m.CL + t) : kOutOfRow;
}
__device__ __forceinline__ void zero_slot_tail(const float *slot, int live)
{
    if (live < 4) {
        float *p = const_cast<float *>(slot);
        if (live <= 1) p[1] = 0.f;
        if (live <= 2) p[2] = 0.f;
        p[3] = 0.f;
    }
}
// Four consecutive outputs of a virtual row, at positions u .. u + 3 (u a multiple of 4): they lie in one row, in one gap,
// or - rows whose length is not a multiple of four - the first n of them end a row.  Element offset of the first (from the
// channel's first row) or -1, and n.
__device__ __forceinline__ int rows_element_group(const RowsMap &m, int u, int &n)
{
    const int b = (int)__umulhi((unsigned)u, m.M);
    const int t = u - b * m.P;
    const bool in = (unsigned)u < (unsigned)m.Lv && t < m.L;
    const int left = m.L - t;
    n = left < 4 ? left : 4;
    return in ? b * m.CL + t : -1;
}
template <typename T>
__device__ __forceinline__ void st_rows_group(T *p, float4 v, int n)
{
    if (n == 4) {
        st_elem4_stream(p, v);
    } else {
        st_elem(p, v.x);
        if (n > 1) st_elem(p + 1, v.y);
        if (n > 2) st_elem(p + 2, v.z);
    }
}

// Raw bits of 4 consecutive elements (a "granule").
template <typename T> struct Raw4;
template <> struct Raw4<float> {
    typedef uintx4 type;
    static __device__ __forceinline__ type load(uintx4 r, int byte_off) { return buffer_load_x4_untracked(r, byte_off); }
    static __device__ __forceinline__ float4 widen(type v)
    {
        return make_float4(__uint_as_float(v[0]), __uint_as_float(v[1]), __uint_as_float(v[2]), __uint_as_float(v[3]));
    }
};
template <> struct Raw4<bf16_t> {
    typedef uintx2 type;
    static __device__ __forceinline__ type load(uintx4 r, int byte_off) { return buffer_load_x2_untracked(r, byte_off); }
    static __device__ __forceinline__ float4 widen(type v)
    {
        return make_float4(__uint_as_float(v[0] << 16), __uint_as_float(v[0] & 0xffff0000u),
                           __uint_as_float(v[1] << 16), __uint_as_float(v[1] & 0xffff0000u));
    }
};

// out[row, t] = sum_j in~[row, t + j - pad] * f_eff[c, j]
//
// Every wave walks segments wave, wave + n_waves, ... of the memory order (b, c, seg) and keeps the
// Toeplitz operands of the current channel in registers (reloaded when the channel changes).
// Per segment it
//   (1) issues the global loads of the NEXT segment plus halo into registers,
//   (2) contracts the 4 D tiles (16 blocks = 256 outputs each) of the current segment out of its
//       private LDS region (16-blocks padded to 24 floats, zeros outside the row),
//   (3) drains the prefetch registers into the same LDS region, and
//   (4) stores 16 bytes per lane per D tile (streaming stores: the outputs are not read again by this
//       operator, and keeping them out of the last-level cache leaves it to the inputs the backward calls re-read),
// so loads are in flight during (2) and the stores of a segment have the whole of the next
// segment's (2) to retire before the next wait on the memory counter.
//
// ROWS (short rows, see RowsMap): the unit of work is a segment of the virtual row of a channel; wave slots are
// ordered (virtual segment, channel), so neighbouring waves read neighbouring channels of the same batches, and
// `row` / `seg` below then hold the virtual segment and the channel.
// RAG: rows that are not whole granules of four (fp32, ordinary rows): the loads need nothing (row resources, per-dword
// range check); the last group of four outputs of a row is stored by element, which costs registers, so these
// variants are compiled apart and run two waves per SIMD from eight block offsets.
template <typename T, int ND, bool ROWS, bool RAG = false>
__global__ __launch_bounds__(64 * kCorrWavesPerBlock, ((ND > 9 || ((RAG || ROWS) && ND > 7)) ? 2 : ND > 6 ? 3 : kMfmaWavesPerSimd)) void corr_mfma_kernel(const T *__restrict__ in,
                                                                         const T *__restrict__ f, T *__restrict__ out,
                                                                         const CorrGeom g, const RowsMap rm)
{
    constexpr int NIB = kSegBlocks + ND - 1;       // input blocks staged per segment
    constexpr int NG = NIB * 4;                    // 16-byte granules staged per segment
    constexpr int NLD = (NG + 63) / 64;            // granules per lane
    constexpr int NDT = kSegBlocks / 16;           // D tiles per segment
    __shared__ __align__(16) float s_in[kCorrWavesPerBlock][NIB * kLdsBlockStride];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i16 = lane & 15;      // A: output position r;  B/D: block j
    const int k4 = lane >> 4;       // contraction sub-index;  D: row group

    // Wave w walks segments w, w + n_waves, ...: at any moment the waves of the chip read one
    // contiguous stretch of memory, which spreads the traffic evenly over the HBM channels.
    // (row, seg, c) are wave-uniform and advanced without divisions.
    // The four waves of a block take four consecutive segments, so three of the four halos a block
    // needs are the tails of segments the same compute unit has just read.
    const int wg = (int)blockIdx.x * kCorrWavesPerBlock + __builtin_amdgcn_readfirstlane(wave);
    // (the divisions run on the vector ALU; the results are wave-uniform and are needed in scalar registers)
    int row = __builtin_amdgcn_readfirstlane(wg / g.segs_per_row);                 // b * C + c
    int seg = __builtin_amdgcn_readfirstlane(wg % g.segs_per_row);
    int c = ROWS ? seg : __builtin_amdgcn_readfirstlane(row % g.C);
    if (wg >= g.n_waves || row >= g.rows) return;      // (the last block may hold spare waves)
    int row_n, seg_n, c_n;                         // the segment after (row, seg)
    auto advance = [&]() {
        seg_n = seg + g.step_seg;
        const int carry = seg_n >= g.segs_per_row ? 1 : 0;
        seg_n -= carry ? g.segs_per_row : 0;
        row_n = row + g.step_rows + carry;
        if constexpr (ROWS) {
            c_n = seg_n;
        } else {
            c_n = c + g.step_c + carry;
            c_n -= c_n >= g.C ? g.C : 0;
            c_n -= c_n >= g.C ? g.C : 0;
        }
    };

    // per-lane constants: byte offset of the lane's i-th granule inside the staged window, and its LDS slot
    constexpr int ES = (int)sizeof(T);
    typename Raw4<T>::type pre[NLD];
    // every round of loads but the last is full: one lane offset plus the instruction's immediate offset (fp32)
    const int off_lane = 4 * ES * lane;
    const int off_tail = (lane + 64 * (NLD - 1) < NG) ? 4 * ES * (lane + 64 * (NLD - 1)) : kOutOfRow;
    auto load_round = [&](uintx4 r, int base, auto ic) {
        constexpr int i = decltype(ic)::value;
        if constexpr (i == NLD - 1) pre[i] = Raw4<T>::load(r, off_tail + base);
        else if constexpr (ES == 4 && 1024 * i < 4096) pre[i] = buffer_load_x4_untracked_imm<(ES == 4 ? 1024 * i : 0)>(r, off_lane + base);
        else pre[i] = Raw4<T>::load(r, off_lane + 4 * ES * 64 * i + base);
    };
    auto prefetch = [&](int prow, int pseg) {
        if constexpr (ROWS) {
            // virtual segment prow of channel pseg: every lane translates the positions of its granules
            const int v0 = prow * kSegLen + 16 * g.dmin;
            const unsigned long long a = reinterpret_cast<unsigned long long>(in + (size_t)pseg * (size_t)g.L);
            const uintx4 r = {(unsigned)a, (unsigned)(a >> 32) & 0xffffu, rm.bytes - (unsigned)(pseg * g.L) * (unsigned)ES,
                              kBufferFlags};
#pragma unroll
            for (int i = 0; i < NLD; ++i)
                pre[i] = Raw4<T>::load(r, lane + 64 * i < NG ? rows_byte_offset<ES>(rm, v0 + 4 * (lane + 64 * i)) : kOutOfRow);
        } else {
            const int u0 = ES * (pseg * kSegLen + 16 * g.dmin);          // may be negative: before the row start
            const int start = u0 > 0 ? u0 : 0;
            const uintx4 r = row_tail_resource(in + (size_t)prow * (size_t)g.L, g.L, start);
            const int base = u0 < 0 ? u0 : 0;          // a window that starts before the row: negative offsets
            load_round(r, base, std::integral_constant<int, 0>{});
            if constexpr (NLD > 1) load_round(r, base, std::integral_constant<int, 1>{});
            if constexpr (NLD > 2) load_round(r, base, std::integral_constant<int, 2>{});
            if constexpr (NLD > 3) load_round(r, base, std::integral_constant<int, 3>{});
            if constexpr (NLD > 4) load_round(r, base, std::integral_constant<int, 4>{});
            static_assert(NLD <= 5, "at most five rounds of loads per segment");
        }
    };
    float *sw = s_in[wave];
    float *sw_lane = sw + (lane >> 2) * kLdsBlockStride + (lane & 3) * 4;
    // LDS block lb holds in~[seg*kSegLen + 16 (dmin + lb) + 0..15]; granule lane + 64 i is block 16 i + lane/4
    auto drain = [&]() {
        wait_untracked_loads();
        release_after_wait(pre);
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (64 * (i + 1) <= NG || lane + 64 * i < NG)       // only the last round is partial
                *reinterpret_cast<float4 *>(sw_lane + 16 * i * kLdsBlockStride) = Raw4<T>::widen(pre[i]);
    };
    // Toeplitz operands: A[d][v] (lane (r, k)) = f_eff[16 (dmin + d) + 4k + v - r + pad]
    float A[ND][4];
    auto load_filter = [&](int ch) {
        const T *f_c = f + (size_t)ch * (size_t)g.K;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int j = 16 * (g.dmin + d) + 4 * k4 + v - i16 + g.pad;
                const bool ok = j >= 0 && j < g.K;
                const int jc = ok ? (g.reverse ? (g.K - 1 - j) : j) : 0;
                const float a = ld_elem(f_c + jc);
                A[d][v] = ok ? a : 0.f;
            }
    };
    // the filter loads of the first channel go out ahead of the first segment's loads: one memory round trip
    // at the start of a wave instead of two
    load_filter(c);
    int cur_c = c;
    prefetch(row, seg);
    drain();
    wave_lds_fence();

    const float *sp = sw + i16 * kLdsBlockStride + 4 * k4;

    for (;;) {
        advance();
        const bool more = row_n < g.rows;
        // (1)
        if (more) prefetch(row_n, seg_n);
        if (c != cur_c) {
            load_filter(c);
            cur_c = c;
        }
        // (2) one dependent chain of 4*ND matrix instructions per D tile.  Group g = (dt, d) is one
        // 16-byte LDS read feeding four matrix instructions; reads run PF groups ahead of their use.
        floatx4 acc[NDT];
        {
            constexpr int NGRP = NDT * ND;
            constexpr int PF = (ND == 6 || ND == 10) ? 2 : 4;     // shorter read-ahead where registers run out
            float4 bv[PF];
#pragma unroll
            for (int q = 0; q < PF; ++q)
                bv[q] = *reinterpret_cast<const float4 *>(sp + (16 * (q / ND) + (q % ND)) * kLdsBlockStride);
#pragma unroll
            for (int q = 0; q < NGRP; ++q) {
                const int dt = q / ND, d = q % ND;
                const float4 cur = bv[q % PF];
                floatx4 a4 = (d == 0) ? floatx4{0.f, 0.f, 0.f, 0.f} : acc[dt];
                a4 = mfma16x16x4(A[d][0], cur.x, a4);
                a4 = mfma16x16x4(A[d][1], cur.y, a4);
                a4 = mfma16x16x4(A[d][2], cur.z, a4);
                a4 = mfma16x16x4(A[d][3], cur.w, a4);
                acc[dt] = a4;
                if (q + PF < NGRP) {
                    const int n = q + PF;
                    bv[q % PF] = *reinterpret_cast<const float4 *>(sp + (16 * (n / ND) + (n % ND)) * kLdsBlockStride);
                }
            }
            // pin the interleaving: PF reads, then (4 matrix instructions, 1 read) per group
#pragma unroll
            for (int q = 0; q < PF; ++q) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
#pragma unroll
            for (int q = 0; q < NGRP; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
                if (q + PF < NGRP) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
        wave_lds_fence();
        // (3)
        if (more) drain();
        // (4) lane (block j = i16, row group k4) owns outputs 16 j + 4 k4 + 0..3 of each D tile;
        // stores past the end of the row are dropped by the range check
        const int lane_t = 16 * i16 + 4 * k4;
        if constexpr (ROWS) {
            T *out_c = out + (size_t)c * (size_t)g.L;                                // wave-uniform
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) {
                const int e = rows_element(rm, row * kSegLen + 256 * dt + lane_t);   // four outputs: one row or one gap
                if (e >= 0) st_elem4_stream(out_c + e, make_float4(acc[dt][0], acc[dt][1], acc[dt][2], acc[dt][3]));
            }
        } else {
            T *out_seg = out + (size_t)row * (size_t)g.L + (size_t)(seg * kSegLen);   // wave-uniform
            if ((seg + 1) * kSegLen <= g.L) {
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt)
                    st_elem4_stream(out_seg + (256 * dt + lane_t), make_float4(acc[dt][0], acc[dt][1], acc[dt][2], acc[dt][3]));
            } else {
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    if constexpr (RAG) {       // (the last group of a row that is not whole granules: by element)
                        st_elem4_stream_upto(out_seg + (256 * dt + lane_t), make_float4(acc[dt][0], acc[dt][1], acc[dt][2], acc[dt][3]),
                                             seg * kSegLen + 256 * dt + lane_t, g.L);
                    } else {
                        if (seg * kSegLen + 256 * dt + lane_t + 3 < g.L)
                            st_elem4_stream(out_seg + (256 * dt + lane_t), make_float4(acc[dt][0], acc[dt][1], acc[dt][2], acc[dt][3]));
                    }
                }
            }
        }
        wave_lds_fence();
        if (!more) break;
        row = row_n; seg = seg_n; c = c_n;
    }
}

// bf16 storage on the bf16 matrix instruction (v_mfma_f32_16x16x16_bf16): the same blocked-Toeplitz
// contraction as corr_mfma_kernel, but the staged tile stays in bf16 (no conversion on the way in),
// one instruction covers a whole 16-block of the contraction (lane (i, kg) holds k = 4 kg + 0..3),
// products of two bf16 are exact in fp32 and the accumulators are fp32; one rounding to bf16 at the
// store.  Needs L % 8 == 0 and 16-byte aligned tensors (16-byte granules of 8 elements).
typedef short shortx4 __attribute__((ext_vector_type(4)));
constexpr int kBf16BlockBytes = 48;      // staged 16-block: 32 bytes + 16 pad

template <int ND>
__global__ __launch_bounds__(64 * kCorrWavesPerBlock, (ND > 9 ? 2 : ND > 8 ? 3 : kMfmaWavesPerSimd)) void corr_mfma_bf16_kernel(
    const bf16_t *__restrict__ in, const bf16_t *__restrict__ f, bf16_t *__restrict__ out, const CorrGeom g,
    const RowsMap /* short rows are an fp32 path */)
{
    constexpr int NIB = kSegBlocks + ND - 1;       // input blocks staged per segment
    constexpr int NG = NIB * 2;                    // 16-byte granules (8 elements) staged per segment
    constexpr int NLD = (NG + 63) / 64;            // granules per lane
    constexpr int NDT = kSegBlocks / 16;           // D tiles per segment
    __shared__ __align__(16) unsigned char s_in[kCorrWavesPerBlock][NIB * kBf16BlockBytes];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i16 = lane & 15;      // A: output position r;  B/D: block j
    const int k4 = lane >> 4;       // contraction group (k = 4 k4 + e);  D: row group

    const int wg = (int)blockIdx.x * kCorrWavesPerBlock + __builtin_amdgcn_readfirstlane(wave);
    // (wave-uniform, needed in scalar registers: the divisions run on the vector ALU)
    int row = __builtin_amdgcn_readfirstlane(wg / g.segs_per_row);                 // b * C + c
    int seg = __builtin_amdgcn_readfirstlane(wg % g.segs_per_row);
    int c = __builtin_amdgcn_readfirstlane(row % g.C);
    if (wg >= g.n_waves || row >= g.rows) return;      // (the last block may hold spare waves)
    int row_n, seg_n, c_n;                         // the segment after (row, seg)
    auto advance = [&]() {
        seg_n = seg + g.step_seg;
        const int carry = seg_n >= g.segs_per_row ? 1 : 0;
        seg_n -= carry ? g.segs_per_row : 0;
        row_n = row + g.step_rows + carry;
        c_n = c + g.step_c + carry;
        c_n -= c_n >= g.C ? g.C : 0;
        c_n -= c_n >= g.C ? g.C : 0;
    };

    uintx4 pre[NLD];
    int ld_off[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) ld_off[i] = (lane + 64 * i < NG) ? 16 * (lane + 64 * i) : kOutOfRow;
    auto prefetch = [&](int prow, int pseg) {
        const int u0 = 2 * (pseg * kSegLen + 16 * g.dmin);           // bytes; may be negative
        const int start = u0 > 0 ? u0 : 0;
        const uintx4 r = row_tail_resource(in + (size_t)prow * (size_t)g.L, g.L, start);
        if (u0 >= 0) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) pre[i] = buffer_load_x4_untracked(r, ld_off[i]);
        } else {
#pragma unroll
            for (int i = 0; i < NLD; ++i) pre[i] = buffer_load_x4_untracked(r, ld_off[i] + u0);
        }
    };
    unsigned char *sw = s_in[wave];
    unsigned char *sw_lane = sw + (lane >> 1) * kBf16BlockBytes + (lane & 1) * 16;
    // LDS block lb holds in~[seg*kSegLen + 16 (dmin + lb) + 0..15] as raw bf16; granule lane + 64 i is block 32 i + lane/2
    auto drain = [&]() {
        wait_untracked_loads();
        release_after_wait(pre);
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (64 * (i + 1) <= NG || lane + 64 * i < NG)       // only the last round is partial
                *reinterpret_cast<uintx4 *>(sw_lane + 32 * i * kBf16BlockBytes) = pre[i];
    };
    prefetch(row, seg);
    drain();
    wave_lds_fence();

    shortx4 A[ND];
    int cur_c = -1;
    const unsigned char *sp = sw + i16 * kBf16BlockBytes + 8 * k4;

    for (;;) {
        advance();
        const bool more = row_n < g.rows;
        if (more) prefetch(row_n, seg_n);
        if (c != cur_c) {
            // Toeplitz operands: A[d][e] (lane (r, kg)) = f_eff[16 (dmin + d) + 4 kg + e - r + pad]
            const bf16_t *f_c = f + (size_t)c * (size_t)g.K;
#pragma unroll
            for (int d = 0; d < ND; ++d)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int j = 16 * (g.dmin + d) + 4 * k4 + e - i16 + g.pad;
                    const bool ok = j >= 0 && j < g.K;
                    const int jc = ok ? (g.reverse ? (g.K - 1 - j) : j) : 0;
                    const uint16_t bits = f_c[jc].bits;
                    A[d][e] = ok ? (short)bits : (short)0;
                }
            cur_c = c;
        }
        floatx4 acc[NDT];
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            shortx4 bv[ND];
#pragma unroll
            for (int d = 0; d < ND; ++d)
                bv[d] = *reinterpret_cast<const shortx4 *>(sp + (16 * dt + d) * kBf16BlockBytes);
            floatx4 a4 = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int d = 0; d < ND; ++d) a4 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(A[d], bv[d], a4, 0, 0, 0);
            acc[dt] = a4;
        }
        wave_lds_fence();
        if (more) drain();
        // lane (block j = i16, row group k4) owns outputs 16 j + 4 k4 + 0..3 of each D tile
        bf16_t *out_seg = out + (size_t)row * (size_t)g.L + (size_t)(seg * kSegLen);   // wave-uniform
        const int lane_t = 16 * i16 + 4 * k4;
        if ((seg + 1) * kSegLen <= g.L) {
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
                st_elem4_stream(out_seg + (256 * dt + lane_t), make_float4(acc[dt][0], acc[dt][1], acc[dt][2], acc[dt][3]));
        } else {
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
                if (seg * kSegLen + 256 * dt + lane_t + 3 < g.L)
                    st_elem4_stream(out_seg + (256 * dt + lane_t), make_float4(acc[dt][0], acc[dt][1], acc[dt][2], acc[dt][3]));
        }
        wave_lds_fence();
        if (!more) break;
        row = row_n; seg = seg_n; c = c_n;
    }
}

// Prefetch of four consecutive elements that may fall outside the row [0, L): the load is always
// issued, from a clamped in-range address, and the value is masked only when it is consumed
// (mask4), so that nothing waits on the load where it is issued.  Needs L >= 4, L % 4 == 0, u % 4 == 0.
template <typename T>
__device__ __forceinline__ float4 ld4_clamped(const T *row, int u, int L)
{
    return ld_elem4(row + min(max(u, 0), L - 4));
}
__device__ __forceinline__ float4 mask4(float4 v, int u, int L)
{
    return (u >= 0 && u + 3 < L) ? v : make_float4(0.f, 0.f, 0.f, 0.f);
}

// Sums the diagonals of one wave's ND accumulators:
//     dw_wave[j] = sum of G_d[q'][q] over 16 (dmin + d) + q' - q + pad = j.
// Lane (q = lane % 16, k = lane / 16) holds G_d[4 k + v][q] in element v.  The accumulators are scattered into
// a skewed LDS image M[jl][q], jl = 16 d + q' - q + 15, rows padded to 17 floats, in which every diagonal is a
// row: cell (jl, q) is written by at most one (d, q'), the cells nothing maps to stay zero, and lane j adds the
// 16 cells of its row in q order (independent reads, conflict-free at stride 17).  sw: the wave's private LDS
// region, at least (16 ND + 15) * 17 floats, 16-byte aligned.
// The taps [j0, j1) only, tap j into dw_wave[j - j0] (a launch over part of the block offsets owns part of the taps).
template <int ND>
__device__ __forceinline__ void dw_wave_diagonal_sums(const floatx4 (&G)[ND], float *sw, float *dw_wave, int lane, int j0,
                                                      int j1, int pad, int dmin)
{
    constexpr int ROWS = 16 * ND + 15, RS = 17;
    constexpr int N4 = (ROWS * RS + 3) / 4;
    for (int i = lane; i < N4; i += 64) *reinterpret_cast<float4 *>(sw + 4 * i) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_fence();
    const int q = lane & 15, k4 = lane >> 4;
#pragma unroll
    for (int d = 0; d < ND; ++d)
#pragma unroll
        for (int v = 0; v < 4; ++v) sw[(16 * d + 4 * k4 + v - q + 15) * RS + q] = G[d][v];
    wave_lds_fence();
    for (int j = j0 + lane; j < j1; j += 64) {
        const int jl = j - pad - 16 * dmin + 15;
        float sum = 0.f;
        if (jl >= 0 && jl < ROWS) {
            float t[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) t[i] = sw[jl * RS + i];
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += t[i];
        }
        dw_wave[j - j0] = sum;
    }
}
// ... all K taps
template <int ND>
__device__ __forceinline__ void dw_wave_diagonal_sums(const floatx4 (&G)[ND], float *sw, float *dw_wave, int lane, int K,
                                                      int pad, int dmin)
{
    dw_wave_diagonal_sums<ND>(G, sw, dw_wave, lane, 0, K, pad, dmin);
}

// Stage 1 of the weight gradient on the matrix cores.
// grid = (C, S).  The segments of a channel are ordered (b, seg); wave w of slice s takes segments
// W s + w, W s + w + W S, ...  A wave keeps ND 16x16
// accumulators G_d for its whole life.  Per segment: the loads of the next segment are issued,
// the current one is contracted out of the wave's private LDS region (x window with halo, then
// dY; both operands of a 64-position chunk are 64 consecutive floats), then the prefetch
// registers are drained into LDS.  At the end every wave sums the diagonals of its own G_d, and
// the W per-wave results are added in wave order.
constexpr int dw_mfma_wave_floats(int ND)
{
    const int stage = kSegLen + 16 * ND + kSegLen, gf = ND * 256;
    return stage > gf ? stage : gf;
}
constexpr size_t dw_mfma_lds_bytes(int ND, int W) { return (size_t)W * (size_t)(dw_mfma_wave_floats(ND) + 16 * ND) * sizeof(float); }

// W waves per block.  dw_out == nullptr: the block's sums go to slice blockIdx.y of part; otherwise (one
// block per channel, gridDim.y == 1) they are the weight gradient itself and go to dw_out.
// ROWS: short rows, the wave walks the virtual row of its channel (see RowsMap); B is then 1 and segs_per_row the
// number of segments of the virtual row.
template <typename T, int ND, int W, bool ROWS>
__global__ __launch_bounds__(64 * W, kMfmaWavesPerSimd) void dw_partial_mfma_kernel(
    const T *__restrict__ x, const T *__restrict__ dy, float *__restrict__ part, T *__restrict__ dw_out, int B, int C,
    int L, int K, int pad, int dmin, int segs_per_row, const RowsMap rm)
{
    constexpr int XW = kSegLen + 16 * ND;          // staged x window (floats)
    constexpr int NGX = XW / 4;
    constexpr int NLX = (NGX + 63) / 64;
    constexpr int NLG = kSegLen / 256;             // dY granules per lane
    constexpr int NCH = kSegLen / 64;              // 64-position chunks per segment
    constexpr int GF = ND * 256;                   // floats of one wave's G
    constexpr int STAGE = XW + kSegLen;
    constexpr int WREG = STAGE > GF ? STAGE : GF;  // per-wave LDS region
    static_assert(WREG == dw_mfma_wave_floats(ND), "host and kernel agree on the LDS layout");
    extern __shared__ __align__(16) float dyn_lds[];
    float (*s_mem)[WREG] = reinterpret_cast<float (*)[WREG]>(dyn_lds);
    float (*s_dw)[16 * ND] = reinterpret_cast<float (*)[16 * ND]>(dyn_lds + W * WREG);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int c = blockIdx.x;
    // wave-slice ws of the channel walks segments ws, ws + stride, ...: at any moment the chip reads
    // whole rows of a few batches, contiguous over the channels.  (b, seg) are wave-uniform and
    // advanced without divisions.
    const int stride = (int)gridDim.y * W;
    const int ws = (int)blockIdx.y * W + __builtin_amdgcn_readfirstlane(wave);
    const int step_b = stride / segs_per_row, step_seg = stride % segs_per_row;
    int b = ws / segs_per_row, seg = ws % segs_per_row;
    int b_n, seg_n;
    auto advance = [&]() {
        seg_n = seg + step_seg;
        const int carry = seg_n >= segs_per_row ? 1 : 0;
        seg_n -= carry ? segs_per_row : 0;
        b_n = b + step_b + carry;
    };
    float *sx = s_mem[wave];            // sx[i] = x~[t0 + 16 dmin + i]
    float *sg = s_mem[wave] + XW;       // sg[i] = dy[t0 + i]

    floatx4 G[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) G[d] = floatx4{0.f, 0.f, 0.f, 0.f};

    float4 pre_x[NLX], pre_g[NLG];
    auto prefetch = [&](int pb, int pseg) {
        if constexpr (ROWS) {
            // virtual segments are walked downwards, like the batches below; every lane translates its positions
            const int t0 = (segs_per_row - 1 - pseg) * kSegLen;
            const int u0 = t0 + 16 * dmin;
            const T *xc = x + (size_t)c * (size_t)L, *gc = dy + (size_t)c * (size_t)L;
            const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int i = 0; i < NLX; ++i) {
                const int e = rows_element(rm, u0 + 4 * (lane + 64 * i));
                pre_x[i] = e >= 0 ? ld_elem4(xc + e) : zero;
            }
#pragma unroll
            for (int i = 0; i < NLG; ++i) {
                const int e = rows_element(rm, t0 + 4 * (lane + 64 * i));
                pre_g[i] = e >= 0 ? ld_elem4(gc + e) : zero;
            }
        } else {
            // batches are walked from the last to the first: the input-gradient call that usually runs just before
            // this one walks them upwards, so its last rows of dY are still in the last-level cache
            const size_t row = ((size_t)(B - 1 - pb) * (size_t)C + (size_t)c) * (size_t)L;
            const int t0 = pseg * kSegLen;
            const int u0 = t0 + 16 * dmin;
#pragma unroll
            for (int i = 0; i < NLX; ++i) pre_x[i] = ld4_clamped(x + row, u0 + 4 * (lane + 64 * i), L);
#pragma unroll
            for (int i = 0; i < NLG; ++i) pre_g[i] = ld4_clamped(dy + row, t0 + 4 * (lane + 64 * i), L);
        }
    };
    auto drain = [&](int pseg) {
        const int t0 = pseg * kSegLen;
        const int u0 = t0 + 16 * dmin;
#pragma unroll
        for (int i = 0; i < NLX; ++i) {
            const int gi = lane + 64 * i;
            if (gi < NGX) *reinterpret_cast<float4 *>(sx + 4 * gi) = ROWS ? pre_x[i] : mask4(pre_x[i], u0 + 4 * gi, L);
        }
#pragma unroll
        for (int i = 0; i < NLG; ++i) {
            const int gi = lane + 64 * i;
            *reinterpret_cast<float4 *>(sg + 4 * gi) = ROWS ? pre_g[i] : mask4(pre_g[i], t0 + 4 * gi, L);
        }
    };
    if (b < B) {
        prefetch(b, seg);
        drain(seg);
    }
    wave_lds_fence();

    while (b < B) {
        advance();
        const bool more = b_n < B;
        if (more) prefetch(b_n, seg_n);
        // 64-position chunk ch, block offset d:  G_d += X[n0 + k + dmin + d][q'] * dY[n0 + k][q]
        //   A operand sx[64 ch + 16 d + lane],  B operand sg[64 ch + lane].
        // LDS reads run ahead of the matrix instructions in two small rings.
        {
            constexpr int NQ = NCH * ND;
            constexpr int PFX = 6, PFG = 2;
            float xr[PFX], gr[PFG];
#pragma unroll
            for (int ch = 0; ch < PFG; ++ch) gr[ch] = sg[64 * ch + lane];
#pragma unroll
            for (int q = 0; q < PFX; ++q) xr[q] = sx[64 * (q / ND) + 16 * (q % ND) + lane];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int ch = q / ND, d = q % ND;
                G[d] = mfma16x16x4(xr[q % PFX], gr[ch % PFG], G[d]);
                if (q + PFX < NQ) {
                    const int n = q + PFX;
                    xr[q % PFX] = sx[64 * (n / ND) + 16 * (n % ND) + lane];
                }
                if (d == ND - 1 && ch + PFG < NCH) gr[ch % PFG] = sg[64 * (ch + PFG) + lane];
            }
#pragma unroll
            for (int q = 0; q < PFX + PFG; ++q) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (q + PFX < NQ) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if (q % ND == ND - 1 && q / ND + PFG < NCH) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
        wave_lds_fence();
        if (more) drain(seg_n);
        wave_lds_fence();
        b = b_n; seg = seg_n;
    }

    // ---- per-wave diagonal sums, then the waves of the block in wave order
    static_assert(WREG >= ((16 * ND + 15) * 17 + 3) / 4 * 4, "diagonal image fits the wave's region");
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
