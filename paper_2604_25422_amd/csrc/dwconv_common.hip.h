// Shared device helpers of the gfx950 depthwise-convolution kernels:
// storage-type load/store (fp32 and bfloat16 with fp32 arithmetic).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dwconv {

// bfloat16 storage element: the upper 16 bits of an IEEE binary32.
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Round-to-nearest-even fp32 -> bf16 (NaN stays a quiet NaN).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float ld_elem(const float *p) { return *p; }
__device__ __forceinline__ float ld_elem(const bf16_t *p) { return bf16_bits_to_f32(p->bits); }
__device__ __forceinline__ void st_elem(float *p, float v) { *p = v; }
__device__ __forceinline__ void st_elem(bf16_t *p, float v) { p->bits = (uint16_t)f32_to_bf16_bits(v); }

// Four consecutive elements, p aligned to 4 elements.
__device__ __forceinline__ float4 ld_elem4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ float4 ld_elem4(const bf16_t *p)
{
    uint2 u = *reinterpret_cast<const uint2 *>(p);
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                       __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u));
}
__device__ __forceinline__ void st_elem4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
// Streaming variants: the line is not kept in the caches on its way to memory.
typedef float nt_floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int nt_uintx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void st_elem4_stream(float *p, float4 v)
{
    nt_floatx4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<nt_floatx4 *>(p));
}
__device__ __forceinline__ void st_elem4(bf16_t *p, float4 v)
{
    uint2 u;
    u.x = f32_to_bf16_bits(v.x) | (f32_to_bf16_bits(v.y) << 16);
    u.y = f32_to_bf16_bits(v.z) | (f32_to_bf16_bits(v.w) << 16);
    *reinterpret_cast<uint2 *>(p) = u;
}
__device__ __forceinline__ void st_elem4_stream(bf16_t *p, float4 v)
{
    nt_uintx2 u;
    u[0] = f32_to_bf16_bits(v.x) | (f32_to_bf16_bits(v.y) << 16);
    u[1] = f32_to_bf16_bits(v.z) | (f32_to_bf16_bits(v.w) << 16);
    __builtin_nontemporal_store(u, reinterpret_cast<nt_uintx2 *>(p));
}

// Four consecutive outputs at positions t .. t + 3 of a row of L positions, the last group of a row possibly
// partial (rows whose length is not a multiple of four): whole groups as one streaming store, the rest by element.
template <typename T>
__device__ __forceinline__ void st_elem4_stream_upto(T *p, float4 v, int t, int L)
{
    if (t + 3 < L) {
        st_elem4_stream(p, v);
    } else {
        if (t < L) st_elem(p, v.x);
        if (t + 1 < L) st_elem(p + 1, v.y);
        if (t + 2 < L) st_elem(p + 2, v.z);
    }
}

// Short rows.  A 1024-position segment of a row much shorter than that is mostly padding, so for short rows the
// kernels work on the VIRTUAL row of a channel instead: its B rows (b, c), b = 0..B-1, laid end to end with pitch
// P = L + gap, gap >= max(pad, K-1-pad) zeros, so that no tap of one row reaches into the next.  That is the same
// operator on a longer signal; only the address of a position changes: virtual position u = b P + t maps to
// element (b C + c) L + t when t < L and to a zero otherwise.  Positions are translated when rows are loaded
// (each lane fetches what belongs in its LDS slot) and when outputs are stored.
struct RowsMap {
    int P;          // pitch of a row inside the virtual row (multiple of 4)
    int L;          // row length
    int CL;         // C * L: elements between row (b, c) and row (b + 1, c)
    int Lv;         // B * P: length of the virtual row
    unsigned M;     // floor(2^32 / P) + 1: u / P == umulhi(u, M) for 0 <= u < 2^32 / P
    unsigned bytes; // bytes from element (0, 0, 0) to the end of the tensor (< 2^30)
};
// Element offset (from the channel's first row) of virtual position u, or -1 where the virtual row holds a zero.
__device__ __forceinline__ int rows_element(const RowsMap &m, int u)
{
    const int b = (int)__umulhi((unsigned)u, m.M);
    const int t = u - b * m.P;
    return ((unsigned)u < (unsigned)m.Lv && t < m.L) ? b * m.CL + t : -1;
}

// Channel of workgroup bx in a grid (C, slices) whose workgroups own one channel each.  Short rows of neighbouring
// channels share the cache line in which one ends and the next begins, and every one of the 8 accelerator dies has an
// L2 of its own; workgroups go to the dies round-robin by linear index, so die k gets the workgroups with bx = k
// (mod 8) of a slice.  Give it a run of consecutive channels (C / 8 of them, one more on the first C % 8 dies): the
// two readers of a shared line then sit behind one L2.
__device__ __forceinline__ int die_run_channel(int bx, int C)
{
    const int q = C >> 3, r = C & 7, k = bx & 7, i = bx >> 3;
    return k * q + (k < r ? k : r) + i;
}
}  // namespace dwconv
