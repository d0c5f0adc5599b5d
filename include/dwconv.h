/*
 * dwconv.h -- C ABI of the MI355X (gfx950) depthwise-convolution training library.
 *
 * The operation (paper Section II, "depthwise convolution": one K x K filter per input
 * channel; Section III-A: per channel i the filter vector w(i) multiplies the im2col matrix
 * C(i) of the same channel, Eq. 3; the weight gradient keeps only the block-diagonal entries,
 * Eq. 4).  The paper's dense block-diagonal route is prior art and is not what runs here:
 * the three passes are direct per-channel stencils, bound by HBM bandwidth.
 *
 * Conventions (the paper leaves them open; these are the readings this library fixes):
 *   - cross-correlation, no filter flip (the paper computes W . im2col(X));
 *   - symmetric zero padding `pad`; Ho = floor((H + 2*pad - K)/stride) + 1, Wo likewise;
 *   - channel multiplier `mult` = m: O = C*m output channels, output channel o reads input
 *     channel o / m (integer division);
 *   - no bias; bwd_filter sums over the batch without a 1/N factor;
 *   - every output tensor is overwritten (never accumulated into).
 *
 * Tensors are dense, no strides argument:
 *   layout NCHW: x, dx [N,C,H,W];  y, dy [N,O,Ho,Wo];  w, dw [O,K,K]
 *   layout NHWC: x, dx [N,H,W,C];  y, dy [N,Ho,Wo,O];  w, dw [K,K,O]
 * dtype F32: all tensors are IEEE fp32.
 * dtype BF16: x, w, y, dy, dx hold bf16 bit patterns (uint16_t), products are accumulated
 *   in fp32 and results rounded to nearest-even on store; dw is fp32 (it is the result of an
 *   fp32 reduction and feeds an optimizer).
 *
 * Every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned, and no output
 * may alias an input.  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 * The library never allocates, frees, copies or synchronises: all work is enqueued
 * asynchronously on `stream` and the buffers must stay alive until the stream reaches it.
 * Concurrent calls on different streams are safe as long as they use different workspaces.  The
 * only global state is a snapshot of the DWCONV_TUNE_* tuning variables, which is taken once and
 * is empty unless DWCONV_TUNE=1 was set in the environment (see dwconv_tuning_reload below): no
 * call reads the environment, and a workspace query and the launch that follows always agree.
 *
 * Errors: 0 on success, a negative dwconv_status otherwise.  Arguments are validated on the
 * host before the first HIP call, and on a validation failure nothing is enqueued.
 */
#ifndef DWCONV_H
#define DWCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum dwconv_layout { DWCONV_NCHW = 0, DWCONV_NHWC = 1 };
enum dwconv_dtype { DWCONV_F32 = 0, DWCONV_BF16 = 1 };

enum dwconv_status {
    DWCONV_OK = 0,
    DWCONV_ERR_NULL = -1,        /* a required pointer is NULL                                    */
    DWCONV_ERR_BAD_DIM = -2,     /* N,C,H,W,K,stride,mult < 1, pad < 0, or Ho/Wo < 1              */
    DWCONV_ERR_BAD_ENUM = -3,    /* layout or dtype is not one of the enumerators                 */
    DWCONV_ERR_WORKSPACE = -4,   /* bwd_filter workspace is NULL or smaller than required         */
    DWCONV_ERR_ALIGN = -5,       /* a data pointer is not 16-byte aligned                         */
    DWCONV_ERR_UNSUPPORTED = -6, /* K > DWCONV_MAX_K                                              */
    DWCONV_ERR_LAUNCH = -7,      /* HIP reported an error when the kernel was launched            */
    DWCONV_ERR_TOO_LARGE = -8,   /* a tensor has 2^31 or more elements (kernels index in 32 bit)  */
    DWCONV_ERR_SCRATCH = -9      /* dwconv_bwd_filter_noalloc: the shape needs more scratch than   */
                                 /* DWCONV_NOALLOC_SCRATCH_BYTES                                    */
};

#define DWCONV_MAX_K 15

/* Problem description: M-channel F x F input and K x K filters in the paper's notation
 * (Section II, "standard convolutions"), generalised to H != W, a batch, a stride, a padding
 * and a channel multiplier. */
typedef struct dwconv_desc {
    int32_t N, C, H, W; /* input tensor dims, all >= 1                                    */
    int32_t K;          /* square K x K filter, 1 <= K <= DWCONV_MAX_K                    */
    int32_t stride;     /* same in H and W, >= 1                                          */
    int32_t pad;        /* symmetric zero padding, >= 0                                   */
    int32_t mult;       /* channel multiplier m >= 1; O = C*mult                          */
    int32_t layout;     /* enum dwconv_layout, applies to x, y, dx, dy, w, dw             */
    int32_t dtype;      /* enum dwconv_dtype (storage type; accumulation is always fp32)  */
} dwconv_desc;

/* Output spatial size of the layer.  Host-only, no HIP call.
 * Returns DWCONV_OK, or ERR_NULL / ERR_BAD_DIM / ERR_BAD_ENUM / ERR_UNSUPPORTED / ERR_TOO_LARGE;
 * Ho, Wo may be NULL. */
int dwconv_out_dims(const dwconv_desc *desc, int32_t *Ho, int32_t *Wo);

/* Bytes of device scratch that dwconv_bwd_filter needs for `desc` (partial sums of the
 * two-stage reduction).  Host-only.  Returns 0 for an invalid desc.  Never more than
 * max(64 MiB, O*K*K*4): shapes whose partial sums would not fit in 64 MiB run with a single
 * partial, the size of dw itself. */
size_t dwconv_bwd_filter_workspace_bytes(const dwconv_desc *desc);

/* Forward pass (Section III-A: z(i) = w(i) . C(i), Eq. 3):
 *   y[n,o,oh,ow] = sum_{kh,kw} w[o,kh,kw] * x[n, o/m, oh*s-p+kh, ow*s-p+kw], x = 0 outside.
 * x: device, read.  w: device, read.  y: device, written in full. */
int dwconv_fwd(const dwconv_desc *desc, const void *x, const void *w, void *y, void *stream);

/* Backward-data pass (the input gradient of the forward pass; Section III-A, backward
 * propagation through the convolution):
 *   dx[n,c,ih,iw] = sum over q < m and taps (kh,kw) with (ih+p-kh), (iw+p-kw) divisible by s
 *                   and the quotients inside [0,Ho) x [0,Wo)
 *                   of w[c*m+q,kh,kw] * dy[n,c*m+q,(ih+p-kh)/s,(iw+p-kw)/s].
 * dy: device, read.  w: device, read.  dx: device, every element written (zeros where no
 * tap lands). */
int dwconv_bwd_data(const dwconv_desc *desc, const void *dy, const void *w, void *dx, void *stream);

/* Backward-filter pass (Eq. 4: only the diagonal blocks of the dense weight gradient survive):
 *   dw[o,kh,kw] = sum_{n,oh,ow} dy[n,o,oh,ow] * x[n, o/m, oh*s-p+kh, ow*s-p+kw], x = 0 outside.
 * x, dy: device, read.  dw: device, fp32 for both dtypes, written in full.
 * workspace: device scratch of at least dwconv_bwd_filter_workspace_bytes(desc) bytes,
 * 16-byte aligned; contents on entry are ignored and on exit unspecified.
 * The reduction uses no atomics: per-thread fp32 partial sums, a fixed-order reduction inside
 * each workgroup, one partial per workgroup in the workspace, and a second kernel that adds the
 * partials in a fixed order.  The result is bit-identical from run to run. */
int dwconv_bwd_filter(const dwconv_desc *desc, const void *x, const void *dy, void *dw,
                      void *workspace, size_t workspace_bytes, void *stream);

/* dwconv_bwd_filter for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results (bit for bit) and
 * error codes as dwconv_bwd_filter, without the workspace: the partial sums go to an array of
 * DWCONV_NOALLOC_SCRATCH_BYTES that is part of the library's device code (each GPU the library runs
 * on holds one copy until the process ends).  A shape whose partial sums need more (see
 * dwconv_bwd_filter_workspace_bytes; every layer of the benchmark workloads needs less than 9 MB)
 * returns DWCONV_ERR_SCRATCH and enqueues nothing.  The call allocates and frees nothing and
 * does not synchronise.  The device of `stream` must be the current device.  All calls on one
 * GPU share the one array: two calls that may overlap on that GPU (different streams, or
 * different threads) race; calls on one stream are ordered and safe.  Contents left by an earlier
 * call are never read. */
#define DWCONV_NOALLOC_SCRATCH_BYTES (16u << 20)
int dwconv_bwd_filter_noalloc(const dwconv_desc *desc, const void *x, const void *dy, void *dw, void *stream);

/* Whole backward pass of the layer in one call: dx as dwconv_bwd_data, dw as dwconv_bwd_filter
 * (Section III-A, backward propagation: both gradients come from the same dy; the paper's
 * Table III reports them as one "Backward" time).  Where a fused kernel exists (3x3, pad 1,
 * multiplier 1, and multiplier 2 in NHWC at stride 1.  Stride 1: NHWC; NCHW with rows of whole
 * 16-byte vectors; NCHW planes with rows of 4, 7, 8, 14 or 28.  Stride 2: NHWC on even maps;
 * NCHW on even maps with rows of 56 and more in fp32, 112 and more in bf16; NCHW planes with
 * rows of 8, 14 or 28 and an even height) dy and x are read once and the pass moves
 * 2|x| + |y| elements instead of
 * 2(|x| + |y|); every other shape runs the two passes one after the other on `stream`, with
 * results identical to the separate calls.  dwconv_variant_name(desc, 3) tells which.
 * x, dy, w: device, read.  dx: device, every element written.  dw: device, fp32, written in full.
 * workspace: device scratch of at least dwconv_bwd_workspace_bytes(desc) bytes, 16-byte aligned.
 * Same error codes, same determinism (no atomics) as the separate entry points. */
size_t dwconv_bwd_workspace_bytes(const dwconv_desc *desc);
int dwconv_bwd(const dwconv_desc *desc, const void *x, const void *dy, const void *w, void *dx, void *dw,
               void *workspace, size_t workspace_bytes, void *stream);

/* Human-readable name of a status code; never NULL. */
const char *dwconv_status_string(int status);

/* Name of the kernel variant the dispatcher picks for `desc` and `pass` (0 fwd, 1 bwd_data,
 * 2 bwd_filter, 3 the whole backward pass of dwconv_bwd: "separate" when it runs the two passes),
 * e.g. "nhwc_rowwalk_k3s1" or "generic".  Host-only; for reports and
 * tests.  Returns "invalid" for an invalid desc. */
const char *dwconv_variant_name(const dwconv_desc *desc, int pass);

/* Tuning hook, not needed in normal use.  The dispatcher's tile sizes can be overridden through
 * DWCONV_TUNE_* environment variables, but only as a snapshot: it is taken at the first call into
 * the library, and holds nothing unless DWCONV_TUNE=1 is set then.  This call takes a new snapshot
 * (after the caller changed the environment) and returns the number of variables it holds.  It must
 * not overlap any other call into the library, and a workspace size queried before it is stale. */
int dwconv_tuning_reload(void);

/* ---- Group convolution: more than one channel per group ------------------------------------------
 *
 * Section V-B (extensibility): a depthwise convolution is the group convolution whose number of
 * groups equals its number of channels; with fewer groups the 0/1 mask of Eq. 2 keeps, for an output
 * channel, the K x K blocks of every input channel of its own group.  As for the depthwise layer,
 * the dense masked product is not what runs: the passes are direct stencils over the Cg = C/groups
 * input channels of a group, still bound by memory for small Cg; with 4 or 8 channels per group the
 * sum over a group's channels is a small dense contraction and runs on the matrix cores (NHWC: forward
 * and backward-data; NCHW with 28x28 or 56x56 planes, and with 2 channels per group on 112x112 planes:
 * all three passes).
 *
 * The C input and O output channels are split into `groups` runs of Cg = C/groups and Og = O/groups
 * consecutive channels; output channel o reads input channels (o/Og)*Cg .. (o/Og)*Cg + Cg - 1.
 *   layout NCHW: x, dx [N,C,H,W];  y, dy [N,O,Ho,Wo];  w, dw [O,Cg,K,K]
 *   layout NHWC: x, dx [N,H,W,C];  y, dy [N,Ho,Wo,O];  w, dw [K,K,Cg,O]
 * All other conventions (cross-correlation, padding, output size, dtypes, dw in fp32, pointers,
 * alignment, stream, errors, determinism) are those of the depthwise entry points above.
 * groups == C (Cg == 1) is the depthwise layer with multiplier O/C and runs on its kernels.
 *
 *   fwd        y[n,o,oh,ow]   = sum_{ci<Cg,kh,kw} w[o,ci,kh,kw] * x[n,(o/Og)*Cg+ci,oh*s-p+kh,ow*s-p+kw]
 *   bwd_data   dx[n,c,ih,iw]  = sum over the Og output channels o of the group of c and the taps
 *                               (kh,kw) that land on (ih,iw) of w[o,c%Cg,kh,kw] * dy[n,o,oh,ow]
 *   bwd_filter dw[o,ci,kh,kw] = sum_{n,oh,ow} dy[n,o,oh,ow] * x[n,(o/Og)*Cg+ci,oh*s-p+kh,ow*s-p+kw]
 */
typedef struct dwconv_group_desc {
    int32_t N, C, H, W; /* input tensor dims, all >= 1                                    */
    int32_t K;          /* square K x K filter, 1 <= K <= DWCONV_MAX_K                    */
    int32_t stride;     /* >= 1                                                           */
    int32_t pad;        /* >= 0                                                           */
    int32_t groups;     /* >= 1, divides C and O (otherwise DWCONV_ERR_BAD_DIM)           */
    int32_t O;          /* output channels, >= 1                                          */
    int32_t layout;     /* enum dwconv_layout                                             */
    int32_t dtype;      /* enum dwconv_dtype                                              */
} dwconv_group_desc;

/* Output spatial size; host-only.  Ho, Wo may be NULL. */
int gconv_out_dims(const dwconv_group_desc *desc, int32_t *Ho, int32_t *Wo);
/* Device scratch gconv_bwd_filter needs; host-only; 0 for an invalid desc; at most
 * max(64 MiB, O*Cg*K*K*4), as for the depthwise layer. */
size_t gconv_bwd_filter_workspace_bytes(const dwconv_group_desc *desc);
/* x, w: device, read.  y: device, written in full. */
int gconv_fwd(const dwconv_group_desc *desc, const void *x, const void *w, void *y, void *stream);
/* dy, w: device, read.  dx: device, every element written. */
int gconv_bwd_data(const dwconv_group_desc *desc, const void *dy, const void *w, void *dx, void *stream);
/* x, dy: device, read.  dw: device, fp32, written in full.  workspace as for dwconv_bwd_filter;
 * two-stage reduction without atomics, bit-identical from run to run. */
int gconv_bwd_filter(const dwconv_group_desc *desc, const void *x, const void *dy, void *dw,
                     void *workspace, size_t workspace_bytes, void *stream);
/* Name of the kernel variant for `pass` (0 fwd, 1 bwd_data, 2 bwd_filter); "invalid" for a bad desc. */
const char *gconv_variant_name(const dwconv_group_desc *desc, int pass);

#ifdef __cplusplus
}
#endif
#endif /* DWCONV_H */
