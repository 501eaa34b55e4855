/*
 * ngconv.h -- C ABI of the MI355X (gfx950) Convolution op family over two and three spatial axes
 * (and Softmax).
 *
 * The library stands where a backend's kernels stand in the paper's stack: the
 * per-backend translation step (Sec. 4, "Transformers") decides how tensor
 * elements are laid out and which backend kernel runs each node, with
 * convolution among the kernels it names, and the framework side only
 * allocates tensors and asks for execution (Sec. 1).  Here the caller
 * allocates and the library executes.  An op is a stateless node whose output
 * shape and element type follow from its inputs and constant attributes
 * (Sec. 2, "Intermediate Representation").  The attributes here are those of
 * the Convolution op: window movement strides, padding below / above, window
 * dilation, plus the element type and the element layout of each tensor (per
 * Sec. 2 the layout of a tensor the user never sees is the backend's choice,
 * whatever its axis order).
 *
 * Definitions (cross-correlation, no filter flip; floor output size):
 *   P = floor((H + pad_below_h + pad_above_h - dil_h*(R-1) - 1) / stride_h) + 1, Q likewise
 *   forward         y[n,k,p,q]  = sum_{c,r,s} X(n,c, p*stride_h - pad_below_h + r*dil_h,
 *                                                   q*stride_w - pad_below_w + s*dil_w) * w[k,c,r,s]
 *                   X = x inside the image, 0 outside
 *   epilogue        z = y (+ bias[k]) ; z = max(z,0)     (ops compounded for the hardware,
 *                   one of the backend optimisations the Abstract lists), applied on the
 *                   fp32 accumulator before the single rounding to the output type
 *   backprop-data   dx = adjoint of forward w.r.t. x applied to dy  (Sec. 3: derivative
 *                   ops come from autodiff of the forward op); elements of dx that no
 *                   window touches are written as 0
 *   backprop-filt.  dw = adjoint of forward w.r.t. w applied to dy; always fp32, [K,C,R,S]
 *
 * Conventions common to every call
 *   - All data / filter / bias / workspace pointers are DEVICE pointers on the current
 *     HIP device.  `hip_stream` is a hipStream_t (NULL = the default stream).
 *   - The caller owns every buffer.  The library never allocates or frees device
 *     memory, never synchronises, never changes the current device.  All work is
 *     enqueued on `hip_stream`; calls return once enqueued.
 *   - Outputs are fully overwritten (never accumulated into).  Inputs and outputs must
 *     not overlap.
 *   - Every call validates its arguments on the host first and returns a negative
 *     ngc_status without launching anything if they are invalid.  A descriptor for
 *     which no kernel exists returns NGC_UNSUPPORTED; there is no CPU fallback.
 *   - Accumulation is always fp32.  bf16 results are rounded once, to nearest even.
 *   - Results are run-to-run identical (no floating-point atomics).
 *   - Each tensor must hold fewer than 2^31 elements.  A bf16 node with blocked tensors whose x or y
 *     reaches 2 GiB runs as several launches over groups of images (ngc_conv_variant: "sliced:...").
 *
 * Every op accepts every combination of data layouts; which combinations run on the MFMA kernels
 * (bf16) and which on the slow direct kernels is a property of the build: blocked x and y for all
 * shapes with C and K multiples of 16, NCHW x of the 3-channel stem, and NCHW x and / or y of 1x1
 * layers with stride 1, no padding and H*W a multiple of 8 are read and written in place; any other
 * bf16 node with NCHW tensors whose blocked form has an MFMA kernel runs on blocked copies that the
 * library keeps at the front of the workspace (ngc_conv_workspace_bytes counts them; the variant is
 * then named "staged:<kernel>").  ngc_conv_variant names the choice.
 *
 * Element layouts
 *   NGC_NCHW      x[n][c][h][w]
 *   NGC_NCHW16C   x[n][cb][h][w][ci], c = 16*cb + ci, cb < ceil(C/16); lanes with
 *                 c >= C hold +0 (writers store +0 there, readers may rely on it)
 *   NGC_KCRS          w[k][c][r][s]
 *   NGC_BLOCKED_FWD   w[r][s][cb][k][ci]   (c = 16*cb+ci; C padded to 16 with +0)
 *   NGC_BLOCKED_BWD   w[r][s][kb][c][ki]   (k = 16*kb+ki; K padded to 16 with +0)
 *                 The two blocked filter layouts put the reduction axis of forward /
 *                 backprop-data innermost; they are produced by ngc_filter_convert.
 */
#ifndef NGCONV_H
#define NGCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NGC_OK = 0,
    NGC_BAD_ARG = -1,             /* null pointer, bad enum value, bias missing with NGC_EPI_BIAS */
    NGC_BAD_SHAPE = -2,           /* non-positive dim, stride/dilation < 1, negative pad, P or Q <= 0,
                                     tensor with >= 2^31 elements */
    NGC_UNSUPPORTED = -3,         /* valid descriptor, but no kernel for this dtype/layout combination */
    NGC_WORKSPACE_TOO_SMALL = -4, /* ws_bytes < ngc_conv_workspace_bytes(...) or ws null when needed */
    NGC_LAUNCH_FAILED = -5,       /* the HIP runtime refused a launch (hipGetLastError != success) */
    NGC_SCRATCH_EXCEEDED = -6     /* ngc_conv_bwd_filters_noalloc: the node needs more than NGC_STATIC_SCRATCH_BYTES */
} ngc_status;

typedef enum { NGC_F32 = 0, NGC_BF16 = 1 } ngc_dtype;
typedef enum { NGC_NCHW = 0, NGC_NCHW16C = 1 } ngc_data_layout;
typedef enum { NGC_KCRS = 0, NGC_BLOCKED_FWD = 1, NGC_BLOCKED_BWD = 2 } ngc_filter_layout;
enum { NGC_EPI_NONE = 0, NGC_EPI_BIAS = 1, NGC_EPI_RELU = 2 };   /* bit flags, forward only */
enum { NGC_OP_FWD = 0, NGC_OP_BWD_DATA = 1, NGC_OP_BWD_FILTERS = 2, NGC_OP_BIAS_GRAD = 3, NGC_OP_BWD_DATA_DB = 4,
       NGC_OP_BWD_DATA_FILTERS = 5 };

/* Constant attributes of one Convolution node and of its two derivative nodes. */
typedef struct {
    int32_t n, c, h, w;            /* data batch shape, logical axes N,C,H,W whatever the layout    */
    int32_t k, r, s;               /* filters: K x C x R x S                                        */
    int32_t stride_h, stride_w;    /* window movement strides, >= 1                                 */
    int32_t dil_h, dil_w;          /* window dilation, >= 1                                         */
    int32_t pad_below_h, pad_below_w;   /* zero padding on the low-index side (top, left), >= 0     */
    int32_t pad_above_h, pad_above_w;   /* zero padding on the high-index side (bottom, right), >= 0*/
    int32_t dtype;                 /* ngc_dtype of x, w, y, dy, dx (bias and dw are always fp32)    */
    int32_t x_layout;              /* ngc_data_layout of x and dx                                   */
    int32_t y_layout;              /* ngc_data_layout of y and dy                                   */
    int32_t w_layout;              /* ngc_filter_layout of the filter argument of fwd / bwd_data    */
    int32_t epilogue;              /* NGC_EPI_* flags, used by ngc_conv_fwd only                    */
} ngc_conv_desc;

/* Output extents P, Q of the node (Sec. 2: attributes determine the output shape).
 * Host only.  Returns NGC_OK, NGC_BAD_ARG (null) or NGC_BAD_SHAPE. */
int ngc_conv_out_shape(const ngc_conv_desc *desc, int32_t *p, int32_t *q);

/* Bytes of device workspace `op` (NGC_OP_*) needs for this descriptor; 0 if none or if the
 * descriptor is invalid / unsupported (the op call itself reports the error).  Host only. */
size_t ngc_conv_workspace_bytes(const ngc_conv_desc *desc, int op);

/* Convolution forward with the compounded bias / ReLU epilogue (Sec. 4 kernel; Abstract,
 * compounding).  x: [N,C,H,W] in x_layout; w: [K,C,R,S] in w_layout (KCRS or BLOCKED_FWD);
 * bias: fp32 [K], may be NULL unless NGC_EPI_BIAS is set; y: [N,K,P,Q] in y_layout, overwritten. */
int ngc_conv_fwd(const ngc_conv_desc *desc, const void *x, const void *w, const float *bias,
                 void *y, void *ws, size_t ws_bytes, void *hip_stream);

/* ConvolutionBackpropData (Sec. 3, derivative of the forward node w.r.t. its data input).
 * dy: [N,K,P,Q] in y_layout; w: in w_layout (KCRS or BLOCKED_BWD); dx: [N,C,H,W] in x_layout,
 * every element overwritten (0 where no window reaches).  No epilogue. */
int ngc_conv_bwd_data(const ngc_conv_desc *desc, const void *dy, const void *w,
                      void *dx, void *ws, size_t ws_bytes, void *hip_stream);

/* ConvolutionBackpropData compounded with the backprop of the ReLU that produced the convolution's
 * data input (Abstract: compounding of operations; Sec. 3: the derivative graph of a ReLU-convolution
 * chain has exactly this pair of nodes): dx = ConvolutionBackpropData(dy, w) where x_in > 0, +0
 * elsewhere (x_in <= 0, -0 and NaN block the gradient).  x_in: the forward data input of the node,
 * same shape, layout and element type as dx; it must not alias dx.  Other arguments, workspace
 * (NGC_OP_BWD_DATA) and errors as ngc_conv_bwd_data; NGC_BAD_ARG if x_in is NULL or misaligned. */
int ngc_conv_bwd_data_relu(const ngc_conv_desc *desc, const void *dy, const void *w, const void *x_in,
                           void *dx, void *ws, size_t ws_bytes, void *hip_stream);

/* ngc_conv_bwd_data_relu that also returns the bias gradient of the layer that produced x_in (three
 * nodes of the derivative graph of a conv -> bias -> ReLU -> conv chain in one call, Sec. 3 and the
 * Abstract's compounding): db[c] = sum over n, h, w of the dx written (the stored, rounded values),
 * fp32, [C] device floats, overwritten.  Where the backprop-data kernel can (blocked dx on the strip
 * and 1x1 GEMM kernels) its workgroups emit the partial sums themselves, otherwise a second pass
 * reads dx; either way the result is a fixed-order reduction.  Workspace:
 * ngc_conv_workspace_bytes(desc, NGC_OP_BWD_DATA_DB).  Errors as ngc_conv_bwd_data_relu; NGC_BAD_ARG
 * also for a NULL or misaligned db. */
int ngc_conv_bwd_data_relu_db(const ngc_conv_desc *desc, const void *dy, const void *w, const void *x_in,
                              void *dx, float *db, void *ws, size_t ws_bytes, void *hip_stream);

/* Bias gradient of the compounded bias epilogue (Sec. 3: adjoint of broadcasting the bias):
 * db[k] = sum over n, p, q of dy[n,k,p,q], accumulated and written in fp32, db: [K] device floats,
 * overwritten.  dy: [N,K,P,Q] in y_layout.  Two-stage fixed-order reduction through `ws`
 * (ngc_conv_workspace_bytes(desc, NGC_OP_BIAS_GRAD) bytes; NGC_WORKSPACE_TOO_SMALL otherwise):
 * the result does not depend on timing. */
int ngc_bias_grad(const ngc_conv_desc *desc, const void *dy, float *db, void *ws, size_t ws_bytes,
                  void *hip_stream);

/* Softmax over the last axis of a dense [rows, cols] tensor of `dtype` (the other kernel the paper
 * names as supplied by a backend library, Sec. 4): y[i][j] = exp(x[i][j]) / sum_k exp(x[i][k]),
 * evaluated with the row maximum subtracted, fp32 arithmetic, one rounding.  x, y: device pointers,
 * element aligned (16-byte aligned tensors with cols a multiple of 16 bytes take the one-pass
 * kernel); y may be x.  Inputs must be finite.  1 <= rows < 2^31, rows * cols < 2^40.
 * NGC_BAD_ARG: bad dtype, NULL or misaligned pointer; NGC_BAD_SHAPE: bad sizes. */
int ngc_softmax(int32_t dtype, int64_t rows, int32_t cols, const void *x, void *y, void *hip_stream);

/* Backprop of ngc_softmax (Sec. 3: derivative graph of the forward op): dx[i][j] = y[i][j] *
 * (dy[i][j] - sum_k dy[i][k] y[i][k]), y the forward result.  dx may be y or dy.  Same conditions. */
int ngc_softmax_bwd(int32_t dtype, int64_t rows, int32_t cols, const void *y, const void *dy, void *dx,
                    void *hip_stream);

/* Name of the kernel ngc_softmax (bwd = 0) / ngc_softmax_bwd (bwd = 1) runs for 16-byte aligned
 * tensors of this row length ("invalid" for bad arguments). */
const char *ngc_softmax_variant(int32_t dtype, int32_t cols, int32_t bwd);

/* ConvolutionBackpropFilters (Sec. 3, derivative w.r.t. the filters input).
 * x in x_layout, dy in y_layout; dw: fp32 [K][C][R][S], overwritten.  The cross-workgroup
 * reduction goes through `ws` (partials) and a fixed-order second stage. */
int ngc_conv_bwd_filters(const ngc_conv_desc *desc, const void *x, const void *dy,
                         float *dw, void *ws, size_t ws_bytes, void *hip_stream);

/* ngc_conv_bwd_filters for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving / training loops, harnesses that forbid hipMalloc.  Same result (bit for bit), same
 * kernels, same argument rules; the split-reduction partials go to an array of NGC_STATIC_SCRATCH_BYTES that is
 * part of the library's device image (each GPU the library runs on holds one copy until the process ends).  The
 * call allocates and frees nothing.  A node whose ngc_conv_workspace_bytes(desc, NGC_OP_BWD_FILTERS) exceeds the
 * array is refused with NGC_SCRATCH_EXCEEDED before anything is launched.  All calls on one GPU share that GPU's
 * array: calls that overlap in time on one GPU (two streams, two threads) race on it; calls on one stream are safe. */
#define NGC_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int ngc_conv_bwd_filters_noalloc(const ngc_conv_desc *desc, const void *x, const void *dy, float *dw,
                                 void *hip_stream);
size_t ngc_static_scratch_bytes(void);

/* ConvolutionBackpropData and ConvolutionBackpropFilters of one node in a single pass (Sec. 3: the
 * derivative graph holds one op per input of the forward op, and both consume the same adjoint dy;
 * Sec. 4 leaves it to the backend to run several ops of the graph as one kernel).  dx and dw are what
 * ngc_conv_bwd_data and ngc_conv_bwd_filters produce (dx rounded once from fp32; dw fp32, [K,C,R,S],
 * run-to-run identical), dy is read from memory once instead of twice.
 * Built for: bf16, x / dx and dy blocked (NGC_NCHW16C), w_layout NGC_BLOCKED_BWD, 1x1 window, stride 1,
 * no padding, C a multiple of 64, K = 64, 128, 256 or 512, tensors below 2 GiB; any other descriptor returns
 * NGC_UNSUPPORTED (the caller then makes the two calls).  ngc_conv_variant(desc, NGC_OP_BWD_DATA_FILTERS)
 * names the kernel or says "unsupported".  ws: ngc_conv_workspace_bytes(desc, NGC_OP_BWD_DATA_FILTERS) bytes
 * (0 for unsupported descriptors; NGC_WORKSPACE_TOO_SMALL otherwise).  Errors as ngc_conv_bwd_data. */
int ngc_conv_bwd_data_filters(const ngc_conv_desc *desc, const void *x, const void *dy, const void *w,
                              void *dx, float *dw, void *ws, size_t ws_bytes, void *hip_stream);

/* The same with the backprop of the ReLU that produced the node's data input compounded into the dx store, as in
 * ngc_conv_bwd_data_relu with x_in = x: dx[i] = x[i] > 0 ? dx[i] : +0 (dw is unchanged: it uses x as it is). */
int ngc_conv_bwd_data_filters_relu(const ngc_conv_desc *desc, const void *x, const void *dy, const void *w,
                                   void *dx, float *dw, void *ws, size_t ws_bytes, void *hip_stream);

/* Data layout conversion (Abstract / Sec. 2: data layout abstraction): copies bit patterns
 * between NGC_NCHW and NGC_NCHW16C for an [n,c,h,w] tensor of `dtype`; tail lanes of a blocked
 * destination are written as +0.  src_layout == dst_layout is a plain copy.  Bit exact. */
int ngc_layout_convert(int32_t dtype, int32_t n, int32_t c, int32_t h, int32_t w,
                       const void *src, int32_t src_layout, void *dst, int32_t dst_layout,
                       void *hip_stream);

/* Filter re-layout (done once per weight update): w_kcrs [K][C][R][S] of desc->dtype ->
 * dst_layout (NGC_BLOCKED_FWD or NGC_BLOCKED_BWD), padded lanes +0.  Bit exact.
 * Destination sizes: ngc_filter_elems(desc, dst_layout) elements. */
int ngc_filter_convert(const ngc_conv_desc *desc, const void *w_kcrs, void *w_blocked,
                       int32_t dst_layout, void *hip_stream);

/* Element counts of the tensors of a node in their layouts (blocked layouts pad the blocked
 * axis to a multiple of 16).  which: 0 = x/dx, 1 = y/dy.  Host only; 0 on invalid input. */
size_t ngc_data_elems(const ngc_conv_desc *desc, int which);
size_t ngc_filter_elems(const ngc_conv_desc *desc, int32_t layout);

/* Name of the kernel variant the dispatcher picks for (desc, op): a static string such as
 * "igemm_bf16_128x128" or "direct"; "unsupported" / "invalid" otherwise.  Host only. */
const char *ngc_conv_variant(const ngc_conv_desc *desc, int op);

/* ---- Convolution over three spatial axes (N, C, D, H, W) --------------------------------------
 * The IR is rank-general (Sec. 2: tensors of any rank, an op is its inputs plus constant
 * attributes); this is the same op with one more window axis:
 *   O = floor((D + pad_below_d + pad_above_d - dil_d*(T-1) - 1) / stride_d) + 1, P, Q likewise
 *   y[n,k,o,p,q] = sum_{c,t,r,s} X(n,c, o*stride_d - pad_below_d + t*dil_d, p*stride_h - ...,
 *                                        q*stride_w - ...) * w[k,c,t,r,s],  X = 0 outside the volume
 * with the epilogue, the two adjoints (Sec. 3), the element types, the error behaviour and the
 * calling conventions of the rank-2 entry points above.
 * Layouts: NGC_NCHW = x[n][c][d][h][w]; NGC_NCHW16C = x[n][cb][d][h][w][ci]; filters NGC_KCRS =
 * w[k][c][t][r][s], NGC_BLOCKED_FWD = w[t][r][s][cb][k][ci], NGC_BLOCKED_BWD = w[t][r][s][kb][c][ki]
 * (ngc_conv3d_filter_convert).  Data tensors convert with ngc_layout_convert(dtype, n, c, d*h, w, ...):
 * both layouts keep (d, h, w) contiguous in that order.
 * Kernels: a window that moves over at most one group of adjacent axes ((T,1,1), (1,1,S), 1x1x1)
 * is the rank-2 op on a reshaped tensor and runs on the rank-2 kernels; other bf16 blocked shapes
 * with C and K multiples of 16 run on the MFMA kernels with a depth axis (forward / backprop-data:
 * windows of 2..25 taps in (h, w) and up to 7 depth taps, else C and K multiples of 32 / 64);
 * everything else on direct kernels (KCRS filters only).
 */
typedef struct {
    int32_t n, c, d, h, w;         /* data batch shape, logical axes N,C,D,H,W                      */
    int32_t k, t, r, s;            /* filters: K x C x T x R x S                                    */
    int32_t stride_d, stride_h, stride_w;
    int32_t dil_d, dil_h, dil_w;
    int32_t pad_below_d, pad_below_h, pad_below_w;
    int32_t pad_above_d, pad_above_h, pad_above_w;
    int32_t dtype;                 /* ngc_dtype of x, w, y, dy, dx (bias and dw are always fp32)    */
    int32_t x_layout, y_layout;    /* ngc_data_layout                                               */
    int32_t w_layout;              /* ngc_filter_layout of the filter argument of fwd / bwd_data    */
    int32_t epilogue;              /* NGC_EPI_* flags, forward only                                 */
} ngc_conv3d_desc;

/* Output extents O, P, Q.  Host only.  NGC_OK, NGC_BAD_ARG (null) or NGC_BAD_SHAPE. */
int ngc_conv3d_out_shape(const ngc_conv3d_desc *desc, int32_t *o, int32_t *p, int32_t *q);

/* Workspace bytes of op NGC_OP_*; 0 if none or invalid. */
size_t ngc_conv3d_workspace_bytes(const ngc_conv3d_desc *desc, int op);

/* Forward with the compounded bias / ReLU epilogue.  x: [N,C,D,H,W] in x_layout; w in w_layout
 * (KCRS or BLOCKED_FWD); bias fp32 [K] or NULL; y: [N,K,O,P,Q] in y_layout, overwritten. */
int ngc_conv3d_fwd(const ngc_conv3d_desc *desc, const void *x, const void *w, const float *bias,
                   void *y, void *ws, size_t ws_bytes, void *hip_stream);

/* Backprop-data.  dy: [N,K,O,P,Q] in y_layout; w in w_layout (KCRS or BLOCKED_BWD); dx in x_layout,
 * every element overwritten (0 where no window reaches). */
int ngc_conv3d_bwd_data(const ngc_conv3d_desc *desc, const void *dy, const void *w,
                        void *dx, void *ws, size_t ws_bytes, void *hip_stream);

/* The backward compounds of the rank-2 family (ngc_conv_bwd_data_relu, ngc_conv_bwd_data_relu_db,
 * ngc_bias_grad) for rank-3 tensors, same definitions, arguments and errors: dx = backprop-data where
 * x_in > 0, +0 elsewhere; db[c] = sum over n, d, h, w of the dx written (fp32, a second pass over dx);
 * ngc_conv3d_bias_grad: db[k] = sum over n, o, p, q of dy.  Workspaces:
 * ngc_conv3d_workspace_bytes(desc, NGC_OP_BWD_DATA / NGC_OP_BWD_DATA_DB / NGC_OP_BIAS_GRAD). */
int ngc_conv3d_bwd_data_relu(const ngc_conv3d_desc *desc, const void *dy, const void *w, const void *x_in,
                             void *dx, void *ws, size_t ws_bytes, void *hip_stream);
int ngc_conv3d_bwd_data_relu_db(const ngc_conv3d_desc *desc, const void *dy, const void *w, const void *x_in,
                                void *dx, float *db, void *ws, size_t ws_bytes, void *hip_stream);
int ngc_conv3d_bias_grad(const ngc_conv3d_desc *desc, const void *dy, float *db, void *ws, size_t ws_bytes,
                         void *hip_stream);

/* Backprop-filters.  dw: fp32 [K][C][T][R][S], overwritten; fixed-order reduction through `ws`. */
int ngc_conv3d_bwd_filters(const ngc_conv3d_desc *desc, const void *x, const void *dy,
                           float *dw, void *ws, size_t ws_bytes, void *hip_stream);

/* Filter re-layout: w [K][C][T][R][S] of desc->dtype -> NGC_BLOCKED_FWD / NGC_BLOCKED_BWD
 * (ngc_conv3d_filter_elems elements, padded lanes +0).  Bit exact. */
int ngc_conv3d_filter_convert(const ngc_conv3d_desc *desc, const void *w_kctrs, void *w_blocked,
                              int32_t dst_layout, void *hip_stream);
size_t ngc_conv3d_filter_elems(const ngc_conv3d_desc *desc, int32_t layout);

/* Element counts of x/dx (which = 0) and y/dy (which = 1) in their layouts.  Host only. */
size_t ngc_conv3d_data_elems(const ngc_conv3d_desc *desc, int which);

/* Name of the kernel variant picked for (desc, op): "rank2:<rank-2 variant>" for windows that
 * reduce to the rank-2 op, "igemm3_bf16_*", "wgrad_gemm3_bf16", "direct3", "unsupported", "invalid". */
const char *ngc_conv3d_variant(const ngc_conv3d_desc *desc, int op);

/* Test hook.  The library reads its NGC_* environment switches (kernel-variant overrides for tests and
 * experiments; NGC_DRY_RUN=1 skips every launch after the host-side planning) once per process, at first use,
 * and caches the launch plan of every descriptor it has seen per thread.  This call reads the switches again and
 * drops the cached plans.  Not meant for production code; not thread safe against calls in flight. */
void ngc_reload_switches(void);

/* Static description of a status code. */
const char *ngc_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* NGCONV_H */
