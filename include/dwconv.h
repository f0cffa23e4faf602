/*
 * dwconv.h -- C ABI of the MI355X (gfx950) depthwise 1-D convolution library.
 *
 * The operator is the depthwise convolution of S4ConvD as the paper states it
 * in Sec. IV-A ("Common Problem Definition and Memory Layout"): one length-K
 * filter per channel slid along the time axis of a [B, C, L] tensor (the paper
 * writes H for the channel count C and k for the filter w), with the three
 * execution paths the paper measures separately: forward (eq. (dwconv)),
 * input gradient (eq. (dx_def)) and kernel/weight gradient (eq. (dk_def)).
 *
 * Common conventions for every entry point
 *   - All tensor pointers are DEVICE pointers (HIP global memory on the current
 *     device).  The caller owns every buffer; the library never allocates,
 *     frees or synchronises.  Work is enqueued on `stream` (a hipStream_t passed
 *     as void*; NULL is the default stream) and the call returns at once.
 *   - x, y, dy, dx are dense row-major [B, C, L] with t the stride-1 index;
 *     w, dw are dense row-major [C, K] (Sec. IV-A, last paragraph).  No strides.
 *   - dtype is the STORAGE type of every tensor of the call (DWCONV_F32 as in
 *     the paper, or DWCONV_BF16).  Products and sums are always fp32; bf16
 *     outputs are rounded to nearest-even once, at the final store.
 *   - Padding: the output length is L.  x~ is x extended by zeros; pad_left in
 *     [0, K-1] zeros are implied on the left and K-1-pad_left on the right.
 *     pad_left = K/2 is the paper's p (eq. (padding_width)), pad_left = K-1 is
 *     causal, (K-1)/2 is 'same' for odd K.  pad_left is the FORWARD pad in all
 *     calls; the library derives the gradient offsets itself.
 *   - Inputs are never written.  Outputs are overwritten, never accumulated.
 *     Inputs and outputs must not overlap.  Tensor base pointers must be aligned
 *     to the element size.
 *   - Same inputs give bitwise-identical outputs from run to run: the weight
 *     gradient is reduced in two ordered levels, never with atomics (the
 *     structure the paper describes in Sec. IV-C/D for its second-stage
 *     reduction).
 *   - Arguments are validated before any HIP call is made; a failed validation
 *     launches nothing.  Return value: a DWCONV_* status, DWCONV_OK (0) on
 *     success.  The library never throws and never aborts.
 *   - K = 1 and K > L are legal.  B*C*L must fit 2^40 elements.
 *   - Non-finite inputs.  The zero padding of x~ is a value that gets multiplied, not a term that is skipped, and
 *     the matrix-core kernels also multiply the zero taps that fill their 16 x 16 filter blocks.  An Inf or NaN at
 *     x[b,c,u] (dy[b,c,u] for the input gradient) therefore makes non-finite the outputs the definition gives it
 *     and possibly, as NaN, outputs of the same row up to 63 positions further on either side, the last 63 positions
 *     of row (b-1,c) and the first 63 of row (b+1,c); an Inf or NaN in w[c,:] may reach every output of channel c.
 *     In the weight gradient a non-finite x or dy of channel c may reach every dw[c,:].  No other channel is ever
 *     touched, and finite inputs never produce a NaN that the definition does not produce.
 */
#ifndef DWCONV_H
#define DWCONV_H

#include <stddef.h>

/* The entry points are the only symbols the shared library exports. */
#define DWCONV_API __attribute__((visibility("default")))

#ifdef __cplusplus
extern "C" {
#endif

enum dwconv_dtype {
    DWCONV_F32  = 0,  /* IEEE binary32 storage (the paper's precision) */
    DWCONV_BF16 = 1   /* bfloat16 storage, fp32 accumulate             */
};

enum dwconv_status {
    DWCONV_OK            = 0,
    DWCONV_ERR_NULL      = 1,  /* a required pointer is NULL                       */
    DWCONV_ERR_SHAPE     = 2,  /* B, C, L or K < 1, or B*C*L too large             */
    DWCONV_ERR_PAD       = 3,  /* pad_left < 0 or pad_left > K-1                   */
    DWCONV_ERR_DTYPE     = 4,  /* dtype is not a dwconv_dtype                      */
    DWCONV_ERR_WORKSPACE = 5,  /* workspace NULL, too small or not 16-byte aligned */
    DWCONV_ERR_ALIGN     = 6,  /* a tensor pointer is not element-aligned          */
    DWCONV_ERR_LAUNCH    = 7,  /* HIP reported an error when launching             */
    DWCONV_ERR_SCRATCH   = 8   /* dwconv_bwd_weight_noalloc: shape needs more than the built-in scratch */
};

/*
 * Forward, Sec. IV-A eq. (dwconv):
 *     y[b,c,t] = sum_{j=0}^{K-1} x~[b,c,t+j-pad_left] * w[c,j]
 * (cross-correlation, the filter is not flipped).
 * x [B,C,L] in, w [C,K] in, y [B,C,L] out; all device, all of `dtype`.
 */
DWCONV_API int dwconv_fwd(const void *x, const void *w, void *y,
               int B, int C, int L, int K, int pad_left, int dtype, void *stream);

/*
 * Input gradient, Sec. IV-A eq. (dx_def), computed as the adjoint of
 * eq. (dwconv) with respect to x:
 *     dx[b,c,s] = sum_{j=0}^{K-1} dy~[b,c,s-j+pad_left] * w[c,j]
 * (equal to the printed eq. (dx_def) whenever K = 2*pad_left + 1).
 * dy [B,C,L] in, w [C,K] in, dx [B,C,L] out.
 */
DWCONV_API int dwconv_bwd_input(const void *dy, const void *w, void *dx,
                     int B, int C, int L, int K, int pad_left, int dtype, void *stream);

/*
 * Weight (kernel) gradient, Sec. IV-A eq. (dk_def):
 *     dw[c,j] = sum_b sum_t dy[b,c,t] * x~[b,c,t+j-pad_left]
 * x, dy [B,C,L] in; dw [C,K] out (storage dtype).  Runs the two stages below
 * back to back on `stream`; when a whole channel is reduced inside one
 * workgroup (dwconv_bwd_weight_single_pass(...) == 1) the block-level sums are
 * the gradient and the first stage writes dw itself: one kernel, workspace
 * untouched.  `workspace` is device memory of at least
 * dwconv_bwd_weight_workspace_bytes(...) bytes, 16-byte aligned; its contents
 * on entry are ignored and it may be reused once the call's work has finished.
 */
DWCONV_API int dwconv_bwd_weight(const void *x, const void *dy, void *dw,
                      void *workspace, size_t workspace_bytes,
                      int B, int C, int L, int K, int pad_left, int dtype, void *stream);

/*
 * Stage 1 of the weight gradient (Sec. IV-C/D: per-block partial sums written
 * to an intermediate tensor):
 *     part[s,c,j] = sum over the (b,t) of slice s of dy[b,c,t] * x~[b,c,t+j-pad_left]
 * part is fp32 [S, C, K] in `workspace`, S = dwconv_bwd_weight_slices(...).
 * Within a block the sum runs over wave-level and then LDS-level reductions in
 * a fixed order.
 */
DWCONV_API int dwconv_bwd_weight_partial(const void *x, const void *dy,
                              void *workspace, size_t workspace_bytes,
                              int B, int C, int L, int K, int pad_left, int dtype, void *stream);

/*
 * Stage 2 of the weight gradient (Sec. IV-C/D):
 *     dw[c,j] = sum_{s=0}^{S-1} part[s,c,j], in increasing s.
 * Reads the fp32 partials stage 1 left in `workspace`, writes dw [C,K] in
 * `dtype`.  Shape arguments must equal those given to stage 1.
 */
DWCONV_API int dwconv_bwd_weight_finalize(const void *workspace, size_t workspace_bytes, void *dw,
                               int B, int C, int L, int K, int pad_left, int dtype, void *stream);

/*
 * dwconv_bwd_weight for callers that cannot allocate device memory or carry a workspace around: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace, same
 * kernels, same bits in dw.  The partial sums go to an array inside the library's device code
 * (dwconv_noalloc_scratch_bytes() = 16 MiB per GPU the library runs on, held until the process ends); a shape whose
 * dwconv_bwd_weight_workspace_bytes(...) exceeds that returns DWCONV_ERR_SCRATCH and launches nothing (every
 * benchmark shape fits; C*K*4 bytes per slice is what counts).  The call allocates and frees nothing.  Its first call
 * on a device looks the array's address up (hipGetSymbolAddress), so make that call outside a capture.  All calls on
 * one GPU share the one array: calls that overlap in time on different streams race; on one stream they are ordered.
 * The array keeps the previous call's contents; the kernels overwrite or clear what they read.
 */
DWCONV_API int dwconv_bwd_weight_noalloc(const void *x, const void *dy, void *dw,
                              int B, int C, int L, int K, int pad_left, int dtype, void *stream);

/* Size in bytes of the built-in scratch dwconv_bwd_weight_noalloc uses. */
DWCONV_API size_t dwconv_noalloc_scratch_bytes(void);

/*
 * Both gradients of the backward pass in one call: dx as dwconv_bwd_input, dw as dwconv_bwd_weight.
 * The paper names kernel fusion as the remaining lever for the backward path (Sec. VI): for filters of the
 * register-resident class (dwconv_bwd_is_fused(...) == 1: up to six 16-position block offsets, i.e. K up to about 66, or
 * any K on rows of at most 48 positions; rows that start on a 4-byte boundary; not fp32 rows of 52 to 128 positions,
 * and bf16 rows of 52 to about 800 positions only from 64 positions and of even length) one kernel reads dy once and produces dx and the stage-1 sums of dw (5 tensor passes over memory per
 * forward + backward step instead of 6); every other shape or type runs the two separate paths one after the
 * other.  dy, x [B,C,L] in; w [C,K] in; dx [B,C,L] out; dw [C,K] out; workspace as for dwconv_bwd_weight.
 * dx must not alias dy or x.  Results: dx equals dwconv_bwd_input's bit for bit; dw is a fixed-order sum like
 * dwconv_bwd_weight's (same tolerance, run-to-run identical).
 */
DWCONV_API int dwconv_bwd(const void *dy, const void *x, const void *w, void *dx, void *dw,
               void *workspace, size_t workspace_bytes,
               int B, int C, int L, int K, int pad_left, int dtype, void *stream);

/* 1 when dwconv_bwd runs the fused kernel for this shape (given tensors aligned as it needs: 16 bytes always do); 0 otherwise. */
DWCONV_API int dwconv_bwd_is_fused(int B, int C, int L, int K, int pad_left, int dtype);

/* Number S of partial slices per coefficient stage 1 writes for this shape; 0 on bad arguments. */
DWCONV_API int dwconv_bwd_weight_slices(int B, int C, int L, int K, int pad_left, int dtype);

/*
 * 1 when, for this shape and 16-byte aligned tensors, dwconv_bwd_weight runs as a single kernel
 * (one workgroup per channel, S = 1, no second stage); 0 otherwise or on bad arguments.
 */
DWCONV_API int dwconv_bwd_weight_single_pass(int B, int C, int L, int K, int pad_left, int dtype);

/*
 * Bytes of workspace dwconv_bwd_weight and dwconv_bwd need for this shape (fp32 [S', C, K] rounded up, S' the larger
 * of S and the slice count of the fused kernel, which differs for rows of at most 48 positions); 0 on bad arguments.
 */
DWCONV_API size_t dwconv_bwd_weight_workspace_bytes(int B, int C, int L, int K, int pad_left, int dtype);

/* Static, NUL-terminated description of a status code (never NULL). */
DWCONV_API const char *dwconv_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
DWCONV_API int dwconv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DWCONV_H */
