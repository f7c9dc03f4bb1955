/*
 * igconv - implicit-GEMM convolution (forward, backward data, backward filter) for AMD
 * MI355X (gfx950).
 *
 * C ABI of the library.  It follows the problem statement of the paper
 * "cuDNN: Efficient Primitives for Deep Learning" (arXiv 1410.0759): a host-callable
 * C interface whose data lives on the GPU in user-controlled buffers (Section 2,
 * 2.1), opaque tensor / filter descriptors with arbitrary per-dimension strides for
 * tensors (Section 2.1), one convolution descriptor holding pad and stride
 * (Section 2.1.1, Table 1), and a forward convolution computed as a lowered matrix
 * product whose lowered data matrix only ever exists in on-chip memory, so that no
 * auxiliary memory is needed (Section 3.1, 3.2).
 *
 * Conventions that hold for every entry point
 *  - Every call returns an igcStatus; nothing throws across the ABI.  Output
 *    arguments are written only when the call returns IGC_STATUS_SUCCESS.
 *  - Handles and descriptors are HOST objects created and destroyed by the caller.
 *    Descriptors are read at call time only: they may be changed or destroyed as
 *    soon as a call returns.
 *  - x, w and y are DEVICE pointers owned by the caller.  The library never
 *    allocates, frees or copies device memory; where a workspace helps, the caller
 *    provides it.
 *  - alpha and beta are HOST pointers, read before the call returns: to float for float
 *    and bfloat16 data (computed in fp32), to double for double data (Section 2: single
 *    and double precision; double problems are computed in fp64 throughout).
 *  - igcConvolutionForward only enqueues work on the handle's stream and returns.
 *  - All argument validation happens before the first GPU call, so every
 *    BAD_PARAM / NOT_SUPPORTED path can be exercised on a machine without a GPU.
 *  - No global mutable state: use one handle per host thread; descriptors may be
 *    shared between threads while nobody is setting them (Section 2.1).
 */
#ifndef IGCONV_H_
#define IGCONV_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    IGC_STATUS_SUCCESS = 0,
    IGC_STATUS_BAD_PARAM = 1,        /* null pointer, non-positive size, inconsistent descriptors */
    IGC_STATUS_NOT_SUPPORTED = 2,    /* valid problem outside what the kernels cover */
    IGC_STATUS_NOT_INITIALIZED = 3,  /* descriptor used before it was set */
    IGC_STATUS_ALLOC_FAILED = 4,     /* host allocation of a handle/descriptor failed */
    IGC_STATUS_EXECUTION_FAILED = 5  /* the GPU runtime reported an error at launch */
} igcStatus;

typedef enum {
    IGC_DATA_FLOAT = 0,   /* IEEE binary32 */
    IGC_DATA_BFLOAT16 = 1, /* upper 16 bits of a binary32 */
    IGC_DATA_DOUBLE = 2    /* IEEE binary64 (Section 2: single and double precision) */
} igcDataType;

typedef enum {
    IGC_CONVOLUTION = 0,      /* eq. 2: tap r reads row p*u + R-1-r - pad_h (filter inverted) */
    IGC_CROSS_CORRELATION = 1 /* tap r reads row p*u + r - pad_h (Section 2.1.1, last paragraph) */
} igcConvolutionMode;

typedef enum {
    IGC_ACTIVATION_SIGMOID = 0, /* 1 / (1 + exp(-x)) */
    IGC_ACTIVATION_RELU = 1,    /* max(x, 0) */
    IGC_ACTIVATION_TANH = 2
} igcActivationMode;

typedef enum {
    IGC_SOFTMAX_MODE_INSTANCE = 0, /* per image over (c,h,w) */
    IGC_SOFTMAX_MODE_CHANNEL = 1   /* per (n,h,w) over c */
} igcSoftmaxMode;

typedef enum {
    IGC_POOLING_MAX = 0,
    IGC_POOLING_AVERAGE = 1 /* mean of the window's elements that lie inside the image */
} igcPoolingMode;

typedef struct igcContext *igcHandle_t;
typedef struct igcTensorStruct *igcTensorDescriptor_t;
typedef struct igcFilterStruct *igcFilterDescriptor_t;
typedef struct igcConvolutionStruct *igcConvolutionDescriptor_t;
typedef struct igcPoolingStruct *igcPoolingDescriptor_t;

/* Human-readable name of a status; never NULL; static storage. */
const char *igcGetErrorString(igcStatus status);

/* ---- handle (Section 2.1: "Overview and Handles") --------------------------------
 * igcCreate allocates a host context bound to the default stream (NULL).  It makes
 * no GPU call.  igcSetStream stores a hipStream_t (passed as void*) on which later
 * igcConvolutionForward calls are enqueued; the caller keeps ownership of it. */
igcStatus igcCreate(igcHandle_t *handle);
igcStatus igcDestroy(igcHandle_t handle);
igcStatus igcSetStream(igcHandle_t handle, void *hipStream);
igcStatus igcGetStream(igcHandle_t handle, void **hipStream);

/* ---- tensor descriptor (Section 2.1; strides: Section 2.1.1) ----------------------
 * A 4-D tensor with logical dimensions n, c, h, w and one element stride per
 * dimension.  Strides are in ELEMENTS, not bytes, and must be >= 0.  NCHW packed is
 * (c*h*w, h*w, w, 1); NHWC ("interleaved feature maps") is (h*w*c, 1, w*c, c);
 * pitched rows, channel slices and other views are expressed the same way. */
igcStatus igcCreateTensorDescriptor(igcTensorDescriptor_t *desc);
igcStatus igcDestroyTensorDescriptor(igcTensorDescriptor_t desc);
igcStatus igcSetTensor4dDescriptor(igcTensorDescriptor_t desc, igcDataType dataType,
                                   int n, int c, int h, int w,
                                   long long nStride, long long cStride,
                                   long long hStride, long long wStride);
igcStatus igcGetTensor4dDescriptor(igcTensorDescriptor_t desc, igcDataType *dataType,
                                   int *n, int *c, int *h, int *w,
                                   long long *nStride, long long *cStride,
                                   long long *hStride, long long *wStride);

/* ---- filter descriptor (Section 2.1.1: F in R^{KCRS}) -----------------------------
 * k output feature maps, c input feature maps, r rows, s columns; the buffer is
 * packed in that order, s fastest. */
igcStatus igcCreateFilterDescriptor(igcFilterDescriptor_t *desc);
igcStatus igcDestroyFilterDescriptor(igcFilterDescriptor_t desc);
igcStatus igcSetFilter4dDescriptor(igcFilterDescriptor_t desc, igcDataType dataType,
                                   int k, int c, int r, int s);
igcStatus igcGetFilter4dDescriptor(igcFilterDescriptor_t desc, igcDataType *dataType,
                                   int *k, int *c, int *r, int *s);

/* ---- convolution descriptor (Table 1: pad_h, pad_w, u, v) -------------------------
 * pad_h / pad_w rows / columns of zeros on EACH side; u / v vertical / horizontal
 * stride; mode picks eq. 2 or its cross-correlation variant.  pad >= 0, u,v >= 1. */
igcStatus igcCreateConvolutionDescriptor(igcConvolutionDescriptor_t *desc);
igcStatus igcDestroyConvolutionDescriptor(igcConvolutionDescriptor_t desc);
igcStatus igcSetConvolution2dDescriptor(igcConvolutionDescriptor_t desc,
                                        int pad_h, int pad_w, int u, int v,
                                        igcConvolutionMode mode);
igcStatus igcGetConvolution2dDescriptor(igcConvolutionDescriptor_t desc,
                                        int *pad_h, int *pad_w, int *u, int *v,
                                        igcConvolutionMode *mode);

/* ---- output size (eq. 1) ----------------------------------------------------------
 * n = x.n, k = w.k, p = ceil((H - R + 1 + 2 pad_h)/u), q likewise with W, S, v,
 * pad_w.  BAD_PARAM if x.c != w.c or if p or q would be < 1. */
igcStatus igcGetConvolution2dForwardOutputDim(igcConvolutionDescriptor_t convDesc,
                                              igcTensorDescriptor_t xDesc,
                                              igcFilterDescriptor_t wDesc,
                                              int *n, int *k, int *p, int *q);

/* ---- workspace query (Section 3: "no auxiliary memory") ---------------------------
 * Validates the problem exactly as igcConvolutionForward does and always reports
 * *sizeInBytes = 0. */
igcStatus igcGetConvolutionForwardWorkspaceSize(igcHandle_t handle,
                                                igcTensorDescriptor_t xDesc,
                                                igcFilterDescriptor_t wDesc,
                                                igcConvolutionDescriptor_t convDesc,
                                                igcTensorDescriptor_t yDesc,
                                                size_t *sizeInBytes);

/* ---- optional workspace of the forward pass ------------------------------------------
 * igcConvolutionForward never needs a workspace.  A problem with so few output tiles that
 * most of the chip would idle (small mini-batches: Section 4 discusses them) can however be
 * run faster when the caller lends one: the reduction over (c,r,s) is then cut into ranges
 * computed side by side, each leaving a partial copy of y in the workspace, and a second
 * kernel adds the parts in a fixed order (deterministic) and applies alpha and beta.  This
 * query reports the size that allows the finest cut the library would choose, 0 when
 * cutting would not help or does not apply (y with gaps between its elements, the bf16
 * channel-vector kernels).  Any smaller size passed to igcConvolutionForward is fine
 * (fewer ranges, or none).
 * A second use, for float or bfloat16 problems the library runs in tap-major order (zero borders, a
 * filter other than 1x1 or nine taps, enough channels) when no cut is chosen: the query reports the
 * filter's size in bytes, and with a workspace of that size (16-byte aligned) the
 * filter is first rewritten there with the channel index innermost, which makes a step's
 * filter reads contiguous; the sums and their order, hence the result's bits, are the same as
 * without the workspace (a smaller one is ignored).
 * A third use, for float problems with a zero border and so few channels that the library would test
 * every gathered element against the window (the generic gather): the query reports the size of x
 * with its border written out, N*C*(H+2*pad_h)*(W+2*pad_w)*4 bytes; with such a workspace (16-byte
 * aligned) that copy is made first and the pass runs over it as a problem without a border. */
igcStatus igcGetConvolutionForwardOptionalWorkspaceSize(igcHandle_t handle,
                                                        igcTensorDescriptor_t xDesc,
                                                        igcFilterDescriptor_t wDesc,
                                                        igcConvolutionDescriptor_t convDesc,
                                                        igcTensorDescriptor_t yDesc,
                                                        size_t *sizeInBytes);

/* ---- forward convolution (eq. 3, Section 2.1.1; algorithm of Section 3.1) ---------
 *
 *   y[n,k,p,q] = alpha * sum_{c,r,s} w[k,c,r,s] * x0[n,c,hh,ww] + beta * y[n,k,p,q]
 *
 * with x0 = x extended by zeros, (hh, ww) given by the descriptor's mode, pad and
 * stride.  Data types: (x, w, y) = (float, float, float) or (bfloat16, bfloat16,
 * float), products accumulated in fp32; or (double, double, double), accumulated in fp64
 * (no fused bias / activation in double: NOT_SUPPORTED).
 *
 *  - x (device, read): laid out by xDesc.  w (device, read): packed K,C,R,S.
 *    y (device, written; read only when *beta != 0): laid out by yDesc, whose
 *    dimensions must equal igcGetConvolution2dForwardOutputDim's result.
 *  - *beta == 0 makes y write-only: NaN or Inf already in y does not propagate.
 *  - y must not overlap x or w.  x may have zero or overlapping strides; y's strides
 *    must address every output element at a distinct location (else BAD_PARAM).
 *  - workSpace / workSpaceSizeInBytes: NULL / 0 is always fine.  A workspace (device,
 *    4-byte aligned, owned by the caller, not overlapping x, w or y) is used only as
 *    igcGetConvolutionForwardOptionalWorkspaceSize describes.
 *  - NOT_SUPPORTED: any other data-type combination, or a tensor whose largest byte
 *    offset reaches 2^31.
 *  - EXECUTION_FAILED: the kernel launch was rejected by the runtime.
 *  - Results are deterministic run to run (fixed summation order, no atomics).
 */
igcStatus igcConvolutionForward(igcHandle_t handle, const void *alpha,
                                igcTensorDescriptor_t xDesc, const void *x,
                                igcFilterDescriptor_t wDesc, const void *w,
                                igcConvolutionDescriptor_t convDesc,
                                void *workSpace, size_t workSpaceSizeInBytes,
                                const void *beta,
                                igcTensorDescriptor_t yDesc, void *y);

/* ---- backward data (Section 2.1.1: the forms needed for back-propagation are closely
 * related to the forward one; Section 2.1: the same convolution descriptor serves the
 * forward and the backward passes; results are returned raw or accumulated) -----------
 *
 *   dx[n,c,h,w] = alpha * sum over all (k,p,q,r,s) whose forward read lands on (h,w)
 *                           of w[k,c,r,s] * dy[n,k,p,q]      + beta * dx[n,c,h,w]
 *
 * i.e. the transpose of igcConvolutionForward with respect to x, for the same filter and
 * convolution descriptors.  It runs as an implicit GEMM as well (rows c, columns (n,h,w),
 * reduction (k,r,s)): the gathered operand is dy, no lowered matrix is stored; with strides
 * u, v above 1 one launch is made per residue class of (h mod u, w mod v), each reducing
 * over exactly the taps that reach it.
 *
 * Workspace (device, may be null / smaller: then the general route runs, same result up to
 * rounding order): igcGetConvolutionBackwardDataWorkspaceSize returns 0 except for bfloat16
 * problems with u = v = 1, R*S = 9 (K a multiple of 16) or R = S = 1 (K a multiple of 8),
 * pad <= filter size - 1 and dy's channel stride 1, where it returns K*C*R*S*2 bytes: the pass is then the forward pass
 * over dy with the filter's k and c exchanged (written to the workspace, 16-byte aligned,
 * by a small kernel on the same stream) and uses the forward pass's fastest kernels.
 * For float problems with a stride above 1 and few channels (u*v*C <= 128) it returns room for one
 * forward pass that serves all residue classes together: the filter of that pass
 * (u*v*C x K x ceil(R/u) x ceil(S/v) floats, rounded up to 256 bytes) followed by its result
 * (N x u*v*C x (P + ceil(R/u) - 1) x (Q + ceil(S/v) - 1) floats); a first layer's three channels then
 * fill the tiles of one launch instead of a sliver of the tiles of u*v launches.
 * For other float or bfloat16 problems whose launches all run in tap-major order (filters other than nine
 * taps or 1x1 with enough channels) it returns the filter's size in bytes: the filter is then first
 * rewritten with the reduction index innermost (wt[c][r][s][k]), which makes the filter reads of a
 * step contiguous; same sums in the same order, hence the same bits as without the workspace.
 *
 *  - w (device, read): packed K,C,R,S.  dy (device, read): laid out by dyDesc, dimensions
 *    (N, K, P, Q) with P, Q = eq. 1 of dxDesc's H, W.  dx (device, written; read only when
 *    *beta != 0): laid out by dxDesc, dimensions (N, C, H, W); input rows or columns the
 *    forward pass never reads receive beta * dx.
 *  - Data types: (w, dy, dx) = (float, float, float), (bfloat16, bfloat16, float) or
 *    (double, double, double).
 *  - dx must not overlap w or dy and its strides must not alias (else BAD_PARAM).
 *  - Errors as for igcConvolutionForward; all validation precedes the first launch.
 *  - igcSetKernelOverride does not apply; results are deterministic. */
igcStatus igcGetConvolutionBackwardDataWorkspaceSize(igcHandle_t handle,
                                                     igcFilterDescriptor_t wDesc,
                                                     igcTensorDescriptor_t dyDesc,
                                                     igcConvolutionDescriptor_t convDesc,
                                                     igcTensorDescriptor_t dxDesc,
                                                     size_t *sizeInBytes);
igcStatus igcConvolutionBackwardData(igcHandle_t handle, const void *alpha,
                                     igcFilterDescriptor_t wDesc, const void *w,
                                     igcTensorDescriptor_t dyDesc, const void *dy,
                                     igcConvolutionDescriptor_t convDesc,
                                     void *workSpace, size_t workSpaceSizeInBytes,
                                     const void *beta,
                                     igcTensorDescriptor_t dxDesc, void *dx);

/* ---- backward filter (same passages as backward data) ------------------------------
 *
 *   dw[k,c,r,s] = alpha * sum_{n,p,q} dy[n,k,p,q] * x0[n,c,hh,ww] + beta * dw[k,c,r,s]
 *
 * with x0, hh, ww as in igcConvolutionForward: the transpose of the forward pass with
 * respect to w.  An implicit GEMM as well (rows k, columns (c,r,s), reduction (n,p,q));
 * the lowered matrix is never stored.  The output is small and the reduction long, so the
 * reduction is cut into ranges computed side by side, each leaving a partial K*C*R*S
 * result in the workspace, which a second kernel adds up in a fixed order (results are
 * deterministic) while applying alpha and beta.
 *
 *  - x (device, read): laid out by xDesc.  dy (device, read): laid out by dyDesc,
 *    dimensions (N, K, P, Q) from eq. 1.  dw (device, written; read only when *beta != 0):
 *    packed K,C,R,S floats, described by dwDesc (data type float).
 *  - Data types: (x, dy, dw) = (float, float, float), (bfloat16, bfloat16, float) or
 *    (double, double, double; workspace parts are then doubles).
 *  - workSpace (device, scratch, 4-byte aligned, owned by the caller, may be reused as
 *    soon as the stream has run the call): igcGetConvolutionBackwardFilterWorkspaceSize
 *    reports the size that lets the reduction be cut as finely as the library would like.
 *    Any smaller size is accepted, NULL / 0 included: the reduction is then cut into as
 *    many ranges as fit (a part is K*C*R*S results; for bfloat16 x and dy with unit channel
 *    strides K and C are rounded up to the kernel's tiles, and the workspace is used even for
 *    a single range, because that kernel keeps its results in another order than dw's),
 *    down to a single range that writes dw directly - same result up to summation order,
 *    less parallelism.
 *  - dw and workSpace must not overlap x, dy or each other.
 *  - NOT_SUPPORTED also when H + 2*pad_h or W + 2*pad_w exceeds 2^14.
 *  - Other errors as for igcConvolutionForward; igcSetKernelOverride does not apply. */
igcStatus igcGetConvolutionBackwardFilterWorkspaceSize(igcHandle_t handle,
                                                       igcTensorDescriptor_t xDesc,
                                                       igcTensorDescriptor_t dyDesc,
                                                       igcConvolutionDescriptor_t convDesc,
                                                       igcFilterDescriptor_t dwDesc,
                                                       size_t *sizeInBytes);
igcStatus igcConvolutionBackwardFilter(igcHandle_t handle, const void *alpha,
                                       igcTensorDescriptor_t xDesc, const void *x,
                                       igcTensorDescriptor_t dyDesc, const void *dy,
                                       igcConvolutionDescriptor_t convDesc,
                                       void *workSpace, size_t workSpaceSizeInBytes,
                                       const void *beta,
                                       igcFilterDescriptor_t dwDesc, void *dw);

/* ---- forward convolution with the bias addition and the activation fused into its
 * epilogue (Section 2.2 lists both as separate functions; run separately they would each
 * read and write y once more) ---------------------------------------------------------
 *
 *   y[n,k,p,q] = f( alpha * conv(x,w)[n,k,p,q] + beta * y[n,k,p,q] + bias[k] )
 *
 * Everything as for igcConvolutionForward, plus: bias (device, read) is K packed floats or
 * NULL for none; activation is an igcActivationMode or IGC_ACTIVATION_IDENTITY (-1) for
 * none.  BAD_PARAM for any other activation value or a misaligned bias pointer. */
#define IGC_ACTIVATION_IDENTITY (-1)
igcStatus igcConvolutionBiasActivationForward(igcHandle_t handle, const void *alpha,
                                              igcTensorDescriptor_t xDesc, const void *x,
                                              igcFilterDescriptor_t wDesc, const void *w,
                                              igcConvolutionDescriptor_t convDesc,
                                              void *workSpace, size_t workSpaceSizeInBytes,
                                              const void *beta, const void *bias, int activation,
                                              igcTensorDescriptor_t yDesc, void *y);

/* ---- other functions (Section 2.2: activations, softmax, pooling, tensor addition) ----
 * Bandwidth-bound kernels on float tensors, or on double tensors (Section 2: every routine in
 * single and double precision; all tensors of a call share one type), laid out by their
 * descriptors (any non-negative strides for inputs; outputs non-aliasing).  All of them blend
 * like the convolutions: out = alpha * value + beta * out, alpha and beta HOST floats (HOST
 * doubles for double tensors), out read only when *beta != 0.  Common errors: BAD_PARAM for null pointers, mismatched dimensions, aliasing
 * output strides or misaligned pointers; NOT_INITIALIZED for unset descriptors;
 * NOT_SUPPORTED for bfloat16 or mixed data types, byte offsets of 2^31 or more;
 * EXECUTION_FAILED when the runtime rejects the launch.  Validation precedes any GPU call.
 * An input may be the output buffer itself (same descriptor, same pointer: in-place) but
 * must not overlap it otherwise. */

/* y = alpha * f(x) + beta * y, f per igcActivationMode; x and y have equal dimensions. */
igcStatus igcActivationForward(igcHandle_t handle, igcActivationMode mode, const void *alpha,
                               igcTensorDescriptor_t xDesc, const void *x,
                               const void *beta, igcTensorDescriptor_t yDesc, void *y);

/* dx = alpha * dy * f'(.) + beta * dx, with f' taken from the forward OUTPUT y for the
 * sigmoid (y(1-y)) and tanh (1-y^2) and from the forward INPUT x for the rectifier (1 where
 * x > 0).  All four tensors have equal dimensions. */
igcStatus igcActivationBackward(igcHandle_t handle, igcActivationMode mode, const void *alpha,
                                igcTensorDescriptor_t yDesc, const void *y,
                                igcTensorDescriptor_t dyDesc, const void *dy,
                                igcTensorDescriptor_t xDesc, const void *x,
                                const void *beta, igcTensorDescriptor_t dxDesc, void *dx);

/* y = alpha * b + beta * y with b broadcast along each dimension in which it has size 1
 * (its other dimensions equal y's): a bias (1,C,1,1) added to every pixel, a full tensor
 * added element by element, and everything in between. */
igcStatus igcAddTensor(igcHandle_t handle, const void *alpha,
                       igcTensorDescriptor_t bDesc, const void *b,
                       const void *beta, igcTensorDescriptor_t yDesc, void *y);

/* Gradient with respect to the bias of a convolution layer (Section 4: the backward pass of a
 * convolution layer computes the gradients with respect to the bias, the filter weights and
 * the bottom data): db[c] = alpha * (sum over n, h, w of dy[n,c,h,w]) + beta * db[c], the
 * transpose of igcAddTensor's broadcast of a (1,C,1,1) tensor.
 * dyDesc: float, bfloat16 or double, any non-negative strides; dbDesc: dimensions (1,C,1,1),
 * float (double for double dy), its feature-map stride at least 1; alpha and beta: float
 * (double for double dy), host pointers.  dy and db are device pointers owned by the caller;
 * every sum is accumulated in double and the order of the additions is fixed (bitwise
 * repeatable).  workSpace may be NULL: with igcGetConvolutionBackwardBiasWorkspaceSize bytes
 * of device memory (8-byte aligned) the positions are cut into ranges across the chip, whose
 * sums a second kernel adds in order; without, one workgroup per (group of) feature map(s)
 * adds everything - same result to rounding, slower on large tensors.  The workspace's
 * contents before and after the call mean nothing.  Nothing is allocated.
 * BAD_PARAM: null pointer, db's dimensions not (1,C,1,1), negative stride, misaligned
 * pointer; NOT_INITIALIZED: descriptor not set; NOT_SUPPORTED: other type combinations,
 * tensors of 2 GiB or more; EXECUTION_FAILED: the runtime refused a launch. */
igcStatus igcGetConvolutionBackwardBiasWorkspaceSize(igcHandle_t handle, igcTensorDescriptor_t dyDesc,
                                                     igcTensorDescriptor_t dbDesc, size_t *sizeInBytes);
igcStatus igcConvolutionBackwardBias(igcHandle_t handle, const void *alpha,
                                     igcTensorDescriptor_t dyDesc, const void *dy,
                                     void *workSpace, size_t workSpaceSizeInBytes,
                                     const void *beta, igcTensorDescriptor_t dbDesc, void *db);

/* Tensor transformation (Section 2: auxiliary routines for the manipulation of 4-d tensors):
 * y = alpha * x + beta * y for two tensors of equal dimensions and any strides, i.e. a change
 * of layout (NCHW <-> NHWC, pitched <-> packed, a slice into a tensor of its own).  Where x
 * and y are contiguous along different dimensions, 64 x 64 tiles go through LDS so that both
 * sides are accessed in contiguous runs.  x and y must not overlap unless their descriptors
 * are identical. */
igcStatus igcTransformTensor(igcHandle_t handle, const void *alpha,
                             igcTensorDescriptor_t xDesc, const void *x,
                             const void *beta, igcTensorDescriptor_t yDesc, void *y);

/* y = alpha * softmax(x) + beta * y over the groups igcSoftmaxMode names, computed the
 * numerically stable way: exp(x - max of the group) / sum of those. */
igcStatus igcSoftmaxForward(igcHandle_t handle, igcSoftmaxMode mode, const void *alpha,
                            igcTensorDescriptor_t xDesc, const void *x,
                            const void *beta, igcTensorDescriptor_t yDesc, void *y);

/* Softmax backward (Section 2: every routine has a backward form): with y the forward
 * result and dy the gradient with respect to it,
 *   dx_i = alpha * y_i * (dy_i - sum over the group of dy_j * y_j) + beta * dx_i,
 * the groups as in igcSoftmaxForward.  y, dy, dx have equal dimensions. */
igcStatus igcSoftmaxBackward(igcHandle_t handle, igcSoftmaxMode mode, const void *alpha,
                             igcTensorDescriptor_t yDesc, const void *y,
                             igcTensorDescriptor_t dyDesc, const void *dy,
                             const void *beta, igcTensorDescriptor_t dxDesc, void *dx);

/* Pooling descriptor: window size, zero border on each side (pad < window), stride. */
igcStatus igcCreatePoolingDescriptor(igcPoolingDescriptor_t *desc);
igcStatus igcDestroyPoolingDescriptor(igcPoolingDescriptor_t desc);
igcStatus igcSetPooling2dDescriptor(igcPoolingDescriptor_t desc, igcPoolingMode mode,
                                    int windowHeight, int windowWidth,
                                    int pad_h, int pad_w, int u, int v);
igcStatus igcGetPooling2dDescriptor(igcPoolingDescriptor_t desc, igcPoolingMode *mode,
                                    int *windowHeight, int *windowWidth,
                                    int *pad_h, int *pad_w, int *u, int *v);
/* n = x.n, c = x.c, p = floor((H + 2 pad_h - windowHeight)/u) + 1, q likewise (eq. 1 with
 * the window in place of the filter).  BAD_PARAM if p or q would be < 1. */
igcStatus igcGetPooling2dForwardOutputDim(igcPoolingDescriptor_t poolDesc,
                                          igcTensorDescriptor_t xDesc,
                                          int *n, int *c, int *p, int *q);
/* y[n,c,p,q] = alpha * (max or mean over the window starting at (p*u - pad_h, q*v - pad_w),
 * elements outside the image taking no part) + beta * y. */
igcStatus igcPoolingForward(igcHandle_t handle, igcPoolingDescriptor_t poolDesc, const void *alpha,
                            igcTensorDescriptor_t xDesc, const void *x,
                            const void *beta, igcTensorDescriptor_t yDesc, void *y);

/* Pooling backward: dx = alpha * (sum over the windows covering an input element of that
 * window's share of dy) + beta * dx.  Average: every in-image element of a window receives
 * dy / (number of in-image elements).  Maximum: the in-image element holding the window's
 * maximum receives dy, the first in scan order (rows, then columns) among equal ones; the
 * maximum is found again from the forward INPUT x, so the forward result is not needed.
 * dy has the dimensions igcGetPooling2dForwardOutputDim gives for xDesc; dx those of x.
 * Input elements no window reaches receive beta * dx.  Deterministic (no atomics). */
igcStatus igcPoolingBackward(igcHandle_t handle, igcPoolingDescriptor_t poolDesc, const void *alpha,
                             igcTensorDescriptor_t dyDesc, const void *dy,
                             igcTensorDescriptor_t xDesc, const void *x,
                             const void *beta, igcTensorDescriptor_t dxDesc, void *dx);

/* ---- introspection and tuning (host only; no GPU call) ----------------------------
 * The launch plan the library derives for a problem: the tile of the lowered
 * product O_m (K x NPQ) = F_m (K x CRS) . D_m (CRS x NPQ) each workgroup computes,
 * the grid, and the number of reduction steps (Section 3.1: fixed-size sub-matrices
 * read successively into on-chip memory). */
typedef struct {
    int kernelId;    /* index into the library's kernel table */
    int tileM;       /* rows of O_m (output feature maps) per workgroup */
    int tileN;       /* columns of O_m (output pixels n,p,q) per workgroup */
    int tileK;       /* reduction elements (c,r,s) per step */
    int gridX;       /* workgroups launched, a multiple of 8 (XCDs): at most as many as the chip holds at
                        once, each then computing several tiles one after the other */
    int kSteps;      /* reduction steps: ceil(CRS / tileK); R*S*ceil(C / tileK) in tap-major order */
    int threads;     /* threads per workgroup */
    int ldsBytes;    /* LDS per workgroup */
    int swapOperands;/* 1 when lanes run along k in the epilogue (y's c-stride is 1) */
    int vecFilterLoads; /* 1 when filter rows are fetched with 16-byte loads */
    int gatherMode;  /* 0 generic window test, 1 tap-major reduction order, 2 unpadded, 3 nine-tap table,
                        4 bf16 channel vectors, 5 bf16 channel vectors from a staged image patch,
                        7 unpadded with tap offsets tabulated in LDS (short reductions) */
} igcConvolutionForwardPlan;

igcStatus igcGetConvolutionForwardPlan(igcHandle_t handle,
                                       igcTensorDescriptor_t xDesc,
                                       igcFilterDescriptor_t wDesc,
                                       igcConvolutionDescriptor_t convDesc,
                                       igcTensorDescriptor_t yDesc,
                                       igcConvolutionForwardPlan *plan);

/* Number of kernels in the table and a short description ("f32 128x128x32 ...") of
 * one of them; NULL for an id out of range. */
int igcGetKernelCount(void);
const char *igcGetKernelName(int kernelId);

/* Force a kernel for later calls on this handle (-1 restores the heuristic).  A
 * kernel that cannot run the problem (wrong data type) makes the forward call
 * return NOT_SUPPORTED. */
igcStatus igcSetKernelOverride(igcHandle_t handle, int kernelId);

/* Division by a launch-time constant as multiply + shift (Section 3.1, last
 * paragraph).  igcMagicDivisor computes (mul, shift) for a divisor 1 <= d < 2^31;
 * igcMagicDivide evaluates floor(n / d) for 0 <= n < 2^31 exactly the way the
 * kernels do: (umulhi(n, mul) + n) >> shift. */
igcStatus igcMagicDivisor(unsigned int d, unsigned int *mul, unsigned int *shift);
unsigned int igcMagicDivide(unsigned int n, unsigned int mul, unsigned int shift);

/* ---- for callers that cannot allocate ----------------------------------------------
 * igcConvolutionBackwardFilterNoAlloc is igcConvolutionBackwardFilter for callers that can
 * neither allocate device memory nor lend a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same arguments without the workspace, same
 * results (bit for bit those of igcConvolutionBackwardFilter with the workspace its size query
 * reports).  The partial results of the cut reduction go to a scratch array of
 * IGC_NOALLOC_SCRATCH_BYTES that is part of the library's code object (every GPU the library
 * runs on holds one copy until the process ends); the call allocates and frees nothing.
 * NOT_SUPPORTED (and a line on stderr) when the problem's workspace size exceeds the array:
 * use igcConvolutionBackwardFilter with a workspace then.  All calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU (two streams, two threads) race; calls
 * on one stream are ordered and safe.  Nothing is kept in the array between calls. */
#define IGC_NOALLOC_SCRATCH_BYTES (64u << 20)
igcStatus igcConvolutionBackwardFilterNoAlloc(igcHandle_t handle, const void *alpha,
                                              igcTensorDescriptor_t xDesc, const void *x,
                                              igcTensorDescriptor_t dyDesc, const void *dy,
                                              igcConvolutionDescriptor_t convDesc,
                                              const void *beta,
                                              igcFilterDescriptor_t dwDesc, void *dw);

/* ---- measurement aids (bench and test tier; nothing on the hot path calls them) -----
 * igcGetDeviceProperties: compute units and engine clock (kHz) of the current device as
 * the runtime reports them (EXECUTION_FAILED without a GPU).
 * igcMeasureMatrixRate: runs a register-only loop of the matrix instruction the kernels of
 * that data type use (fp32 32x32x2, bf16 32x32x16, fp64 16x16x4; no memory traffic, two
 * wavefronts per SIMD on every compute unit) for about `milliseconds` on the handle's
 * stream, WAITS for it, and returns the rate in TFLOP/s: the arithmetic ceiling at the
 * clocks the chip sustains, to be read beside the datasheet peak.  Allocates nothing on
 * the device.  BAD_PARAM: null pointer, unknown type, milliseconds outside 1..2000.
 * igcMeasureMatrixRateOperands: the same loop with a choice of operand values.  randomOperands
 * = 0: one value per lane, the same in every instruction (igcMeasureMatrixRate: the matrix
 * pipes switch few bits and the chip holds its highest clocks).  randomOperands = 1: finite
 * pseudo-random values of mixed sign, another set of registers with every instruction, as
 * the operands of a real product change: the pipes draw more power, the chip sustains lower
 * clocks, and the rate is the ceiling a kernel fed with real data can reach.  BAD_PARAM also
 * for any other value of randomOperands. */
igcStatus igcGetDeviceProperties(igcHandle_t handle, int *computeUnits, int *clockKHz);
igcStatus igcMeasureMatrixRate(igcHandle_t handle, igcDataType dataType, int milliseconds, double *tflops);
igcStatus igcMeasureMatrixRateOperands(igcHandle_t handle, igcDataType dataType, int milliseconds, int randomOperands, double *tflops);

/* ---- checks of the host logic (test tier; host only, no GPU call) --------------------
 * igcCreate reads the number of compute units of the current device into the handle (256,
 * MI355X's, when the runtime finds no device); the launch plans size their grids and balance
 * their tiles by it.  igcSetComputeUnits replaces that number (8..4096, else BAD_PARAM), so
 * that the planning can be exercised for other sizes without such a device;
 * igcGetComputeUnits reads it back.
 *
 * igcGetConvolutionForwardAddressReach / igcGetConvolutionBackwardDataAddressReach: for a
 * problem the pass accepts, with the kernel and launch parameters the pass would use,
 * reachBytes[i] = one past the largest byte offset the kernels' address arithmetic forms
 * for an element that exists, evaluated in 64 bits from the launch parameters (strides,
 * tap offsets, phase offsets) at the extreme indices; extentBytes[i] = the size the
 * buffer descriptor of that argument is given.  i = 0: the gathered tensor (x, resp. dy),
 * 1: the filter, 2: the output (y, resp. dx; backward data: the maximum over its stride
 * phases, each relative to dx).  A correct plan has 0 < reach <= extent < 2^31 for all
 * three; a reach beyond the extent would be an access the hardware's range check has to
 * absorb - or, for a kernel that addressed memory directly, a fault.  Same validation and
 * status codes as the pass itself; BAD_PARAM for null pointers. */
igcStatus igcSetComputeUnits(igcHandle_t handle, int computeUnits);
igcStatus igcGetComputeUnits(igcHandle_t handle, int *computeUnits);
igcStatus igcGetConvolutionForwardAddressReach(igcHandle_t handle, igcTensorDescriptor_t xDesc,
                                               igcFilterDescriptor_t wDesc, igcConvolutionDescriptor_t convDesc,
                                               igcTensorDescriptor_t yDesc, long long reachBytes[3],
                                               long long extentBytes[3]);
igcStatus igcGetConvolutionBackwardDataAddressReach(igcHandle_t handle, igcFilterDescriptor_t wDesc,
                                                    igcTensorDescriptor_t dyDesc,
                                                    igcConvolutionDescriptor_t convDesc,
                                                    igcTensorDescriptor_t dxDesc, long long reachBytes[3],
                                                    long long extentBytes[3]);

#ifdef __cplusplus
}
#endif
#endif /* IGCONV_H_ */
