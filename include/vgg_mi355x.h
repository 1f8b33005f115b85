/*
 * vgg_mi355x.h -- C ABI of libvgg_mi355x.so: the VGG19 forward pass and
 * training step as hand-written HIP kernels for gfx950 (MI355X).
 *
 * The operations are those of the paper's showcase workload (section "VGG19
 * forward pass", section "VGG19 backward pass", the listing that defines
 * dense and softmax, and the appendix table of HLO instruction counts):
 * sixteen 3x3 stride-1 pad-1 convolutions with bias and ReLU, five 2x2
 * window maxima, three dense layers, softmax; then the reverse sweep.
 *
 * Conventions common to every entry point
 * ---------------------------------------
 *  - Every function returns VGG_OK (0) or a negative vgg_status.  Arguments
 *    are validated on the host BEFORE anything is enqueued, so an error
 *    return means no kernel was launched and no buffer was touched.  No
 *    exceptions, no abort().
 *  - All tensor pointers are DEVICE pointers unless the name ends in
 *    `_host`.  The library never allocates or frees device memory and never
 *    synchronises: every call only enqueues kernels on `stream` (a
 *    hipStream_t passed as void*; NULL is the default stream).  Buffers are
 *    owned by the caller and must stay alive until the stream has drained.
 *    One exception: the first launch of a convolution or weight-gradient
 *    kernel in a process raises that kernel's dynamic-LDS limit
 *    (hipFuncSetAttribute), which is a host-side call and not a stream
 *    operation.  It is serialised inside the library, so entry points may be
 *    called from several host threads; but run every call once before
 *    recording it into a HIP graph.
 *  - Tensor pointers must be 16-byte aligned (VGG_ERR_ALIGN otherwise).
 *  - dtype: VGG_F32 = activations and weights fp32, fp32 MFMA.
 *           VGG_BF16 = activations and weights bf16 (round-to-nearest-even
 *           from fp32), fp32 MFMA accumulation, bias and logits fp32.
 *  - Activation layout at the per-op level is NHWC ([N][H][W][C], C
 *    fastest).  The model-level calls take the canonical NCHW fp32 image
 *    batch and canonical parameters (convolution weights [Cout][Cin][3][3],
 *    dense weights [Out][In], the first dense layer's columns in C,H,W
 *    flatten order) and convert once.
 *  - Packed convolution weights, CinP = vgg_padded_channels(dtype, Cin), zeros
 *    in ci >= Cin, 9*Cout*CinP elements: VGG_F32 keeps element (tap t =
 *    3*kh+kw, co, ci) at index (t*Cout + co)*CinP + ci.  VGG_BF16 blocks the
 *    input channels by 16 -- index ((t*(CinP/16) + ci/16)*Cout + co)*16 + ci%16
 *    -- so that the 32 channels x 16 contraction indices of one matrix
 *    instruction's operand are 1 KB of contiguous memory.  Gradients and fp32
 *    master copies are always in the VGG_F32 layout.
 *  - `ws`/`ws_bytes`: caller-owned scratch; the matching *_workspace_bytes
 *    query gives the size required (VGG_ERR_WORKSPACE if smaller).
 */
#ifndef VGG_MI355X_H
#define VGG_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum vgg_status {
    VGG_OK = 0,
    VGG_ERR_NULL = -1,        /* a required pointer is NULL */
    VGG_ERR_SHAPE = -2,       /* non-positive size, odd H/W into a pool, label out of range ... */
    VGG_ERR_DTYPE = -3,       /* dtype is neither VGG_F32 nor VGG_BF16 */
    VGG_ERR_ALIGN = -4,       /* a tensor pointer is not 16-byte aligned */
    VGG_ERR_WORKSPACE = -5,   /* ws is NULL or ws_bytes too small */
    VGG_ERR_LAUNCH = -6,      /* HIP reported an error when a kernel was enqueued */
    VGG_ERR_UNSUPPORTED = -7, /* valid request the library does not implement (e.g. bf16 training without master copy) */
    VGG_ERR_TOO_LARGE = -8    /* vgg_fc_static: the problem needs more scratch than the built-in buffer holds */
} vgg_status;

typedef enum vgg_dtype { VGG_F32 = 0, VGG_BF16 = 1 } vgg_dtype;

#define VGG19_NUM_CONV 16
#define VGG19_NUM_FC 3

/* Whole-network configuration.  The convolution stack is the fixed VGG19
 * pattern 3-64-64 | 128-128 | 256x4 | 512x4 | 512x4 with a 2x2 max-pool
 * after each group; the classifier is flat -> fc_hidden -> fc_hidden ->
 * classes with flat = 512*(H/32)*(W/32).  H and W must be multiples of 32. */
typedef struct vgg_config {
    int dtype;      /* vgg_dtype */
    int N;          /* batch */
    int H, W;       /* input image size */
    int fc_hidden;  /* 4096 for the full model, 512 for the tiny one */
    int classes;    /* 1000 / 10 */
    float lr;       /* SGD step size used by vgg19_train_step */
    int flags;      /* 0 or VGG_FLAG_FP32_MASTER */
} vgg_config;

/* dtype VGG_BF16 only: the packed parameter block carries, behind the bf16
 * parameters that the kernels read, an fp32 master copy of every tensor.
 * vgg19_train_step needs it for bf16 (the update is applied to the master and
 * the bf16 copy refreshed from it); vgg19_unpack_params reads it back;
 * vgg19_forward ignores it. */
#define VGG_FLAG_FP32_MASTER 1

/* Canonical fp32 parameter (or gradient) set: device pointers. */
typedef struct vgg19_params {
    float *conv_w[VGG19_NUM_CONV]; /* [Cout][Cin][3][3] */
    float *conv_b[VGG19_NUM_CONV]; /* [Cout] */
    float *fc_w[VGG19_NUM_FC];     /* [Out][In] */
    float *fc_b[VGG19_NUM_FC];     /* [Out] */
} vgg19_params;

const char *vgg_strerror(int status);

/* Channel count rounded up to the granularity the convolution kernels read:
 * one 64-byte row, i.e. a multiple of 16 for VGG_F32 and of 32 for VGG_BF16.
 * Returns 0 for a bad dtype or C <= 0. */
int vgg_padded_channels(int dtype, int C);

/* ------------------------------------------------------------------ layout */

/* Packs canonical fp32 weights [Cout][Cin][3][3] into the layout described
 * above, converting to `dtype`.  With transpose_flip != 0 it instead writes
 * the operand the data-gradient convolution consumes: element (t, ci, co) of
 * a [Cin][CoutP] matrix per tap, in the same layout with the roles of the
 * channel counts exchanged, holding w[co][ci][8-t] (taps rotated by 180
 * degrees; cf. the "reverse" ops of the backward column of the appendix
 * table), CoutP = vgg_padded_channels(dtype, Cout). */
int vgg_conv_pack_weights(int dtype, int Cin, int Cout, const float *w_oihw, void *w_packed,
                          int transpose_flip, void *stream);
/* Inverse of the forward packing for fp32 data (used for gradients and
 * updated parameters): [9][Cout][CinP] fp32 -> [Cout][Cin][3][3] fp32. */
int vgg_conv_unpack_weights(int Cin, int Cout, const float *w_packed, float *w_oihw, void *stream);

/* fp32 NCHW -> `dtype` NHWC with the channel count padded with zeros to
 * Cpad (Cpad >= C).  And back: `dtype` NHWC (channel stride Cpad) -> fp32
 * NCHW keeping the first C channels. */
int vgg_nchw_to_nhwc(int dtype, int N, int C, int H, int W, int Cpad, const float *x_nchw,
                     void *y_nhwc, void *stream);
int vgg_nhwc_to_nchw(int dtype, int N, int C, int H, int W, int Cpad, const void *x_nhwc,
                     float *y_nchw, void *stream);
/* Element-wise fp32 <-> dtype conversion of n elements (RNE for bf16). */
int vgg_convert(int src_dtype, int dst_dtype, size_t n, const void *src, void *dst, void *stream);

/* ------------------------------------------------------------- convolution */

/* y[n,h,w,co] = f(bias[co] + sum_{kh,kw,ci} x[n,h+kh-1,w+kw-1,ci] * w[co,ci,kh,kw]),
 * x = 0 outside the image, f = max(0,.) if relu else identity (appendix
 * table rows "convolution", "add", "maximum": a cross-correlation, no kernel
 * flip).  x is NHWC with exactly Cin channels, y NHWC with Cout channels,
 * w_packed as produced by vgg_conv_pack_weights(transpose_flip = 0), bias
 * fp32 [Cout] or NULL.  Workspace is needed when Cin differs from
 * vgg_padded_channels(dtype, Cin) (a zero-padded copy of x is made there)
 * and for small problems (fewer pixel-by-channel tiles than half the chip's
 * compute units and a long contraction): several workgroups then share a
 * tile, each summing a range of input channels into fp32 partial results in
 * the workspace, and a second kernel adds them in a fixed order and applies
 * bias and f.  The query returns 0 when neither applies. */
size_t vgg_conv3x3_fwd_workspace_bytes(int dtype, int N, int H, int W, int Cin, int Cout);
int vgg_conv3x3_fwd(int dtype, int N, int H, int W, int Cin, int Cout, const void *x_nhwc,
                    const void *w_packed, const float *bias, void *y_nhwc, int relu, void *ws,
                    size_t ws_bytes, void *stream);

/* vgg_conv3x3_fwd with the following 2x2 max-pool (vgg_maxpool2x2) fused
 * into its epilogue: pooled is NHWC [N][H/2][W/2][Cout]; argmax (may be NULL)
 * gets one byte per pooled element as in vgg_maxpool2x2; y may be NULL, in
 * which case the un-pooled tensor is never written.  Only for
 * H and W multiples of 16 and Cout a multiple of 16 bytes worth of elements
 * (VGG_ERR_UNSUPPORTED otherwise).  The contraction is never split here: the
 * workspace only has to hold the zero-padded copy of x, if one is needed. */
int vgg_conv3x3_fwd_pool(int dtype, int N, int H, int W, int Cin, int Cout, const void *x_nhwc,
                         const void *w_packed, const float *bias, void *y_nhwc_or_null, void *pooled_nhwc,
                         uint8_t *argmax_or_null, int relu, void *ws, size_t ws_bytes, void *stream);

/* The network's first convolution (3 -> 64 channels), same definition as
 * vgg_conv3x3_fwd, but x is the canonical NCHW fp32 image batch [N][3][H][W]
 * and is read directly; y is NHWC [N][H][W][64] in `dtype`; w_packed is the
 * forward packing for Cin = 3, Cout = 64 in `dtype`. */
int vgg_conv3x3_fwd_first(int dtype, int N, int H, int W, const float *x_nchw, const void *w_packed,
                          const float *bias, void *y_nhwc, int relu, void *stream);

/* The network's first two convolutions and first pool as one call
 * (appendix table, forward column: the first two "convolution" rows and the
 * first "reduce-window"; section on XLA: fused operations keep their
 * intermediates on chip):
 *   y2 = relu(conv3x3(relu(conv3x3(x, w1) + bias1), w2) + bias2),
 *   pooled = maxpool2x2(y2),
 * each convolution and the pool as defined for vgg_conv3x3_fwd /
 * vgg_maxpool2x2, the first layer's output rounded to `dtype` before it
 * enters the second, as when the two are called one after the other (the
 * first layer adds its 27 products in another order than
 * vgg_conv3x3_fwd_first, so a few values differ from that sequence by a
 * rounding step).  x is the NCHW fp32 batch [N][3][H][W]; w1 / w2
 * are the forward packings for 3 -> 64 and 64 -> 64 channels; y2
 * [N][H][W][64] and pooled [N][H/2][W/2][64] are NHWC in `dtype`, either may
 * be NULL (not both) and is then never written; no pooling positions are
 * produced.  The first layer's output is not written at all.  bf16 only, H a
 * multiple of 16 and W of 32 (VGG_ERR_UNSUPPORTED otherwise). */
int vgg_conv3x3_fwd_first_pair(int dtype, int N, int H, int W, const float *x_nchw, const void *w1_packed,
                               const float *bias1, const void *w2_packed, const float *bias2, void *y2_nhwc_or_null,
                               void *pooled_nhwc_or_null, void *stream);

/* dx[n,h,w,ci] = sum_{kh,kw,co} g[n,h-kh+1,w-kw+1,co] * w[co,ci,kh,kw]
 * (gradient with respect to the convolution's input; g is the gradient with
 * respect to its pre-activation output, zero outside the image).  w_tf is
 * the transpose_flip != 0 packing.  If relu_src is non-NULL it must be an
 * NHWC tensor shaped like dx and dx is multiplied by (relu_src > 0), i.e.
 * the ReLU backward of the layer that produced this convolution's input is
 * fused in.  Workspace as for vgg_conv3x3_fwd with the roles of Cin and Cout
 * exchanged (padded copy of g; partial sums of a split contraction). */
size_t vgg_conv3x3_bwd_data_workspace_bytes(int dtype, int N, int H, int W, int Cin, int Cout);
int vgg_conv3x3_bwd_data(int dtype, int N, int H, int W, int Cin, int Cout, const void *g_nhwc,
                         const void *w_tf, const void *relu_src, void *dx_nhwc, void *ws,
                         size_t ws_bytes, void *stream);

/* dw[t,co,ci] = sum_{n,h,w} g[n,h,w,co] * x[n,h+kh-1,w+kw-1,ci],
 * db[co] = sum_{n,h,w} g[n,h,w,co].  x and g are NHWC in `dtype`; dw and db
 * are always fp32 (VGG_BF16: bf16 products, fp32 sums, as on the paper's
 * accelerator).  dw is written in the packed layout [9][Cout][CinP] with
 * CinP = vgg_padded_channels(dtype, Cin) (padding entries zero), db is
 * [Cout] or NULL; Cout must be a multiple of 4 (VGG_F32) or 8 (VGG_BF16),
 * VGG_ERR_UNSUPPORTED otherwise.  The
 * pixel sum is split over workgroups; partial sums go to ws and a second
 * kernel adds them in a fixed order, so results are reproducible run to run. */
size_t vgg_conv3x3_bwd_weight_workspace_bytes(int dtype, int N, int H, int W, int Cin, int Cout);
int vgg_conv3x3_bwd_weight(int dtype, int N, int H, int W, int Cin, int Cout, const void *x_nhwc,
                           const void *g_nhwc, float *dw_packed, float *db, void *ws,
                           size_t ws_bytes, void *stream);

/* -------------------------------------------------------------------- pool */

/* y[n,i,j,c] = max_{dh,dw in {0,1}} x[n,2i+dh,2j+dw,c] (appendix table row
 * "reduce-window").  argmax (may be NULL) gets one byte per output element,
 * 2*dh+dw of the first maximum in the order (0,0),(0,1),(1,0),(1,1).  H, W
 * are the input sizes and must be even; C must be a multiple of 8. */
int vgg_maxpool2x2(int dtype, int N, int H, int W, int C, const void *x_nhwc, void *y_nhwc,
                   uint8_t *argmax, void *stream);
/* Scatter backward (row "select-and-scatter"): dx gets dy at the argmax
 * position of each window and zero at the other three.  H, W = size of dx. */
int vgg_maxpool2x2_bwd(int dtype, int N, int H, int W, int C, const void *dy_nhwc,
                       const uint8_t *argmax, void *dx_nhwc, void *stream);

/* ------------------------------------------------------------------- dense */

/* z[n,o] = f(bias[o] + sum_i w[o,i] * a[n,i])  -- the paper's
 * dense(W, x, b) = W*x + b applied to each image (listing "dense"; HLO
 * "dot").  a [N][In] and w [Out][In] in `dtype`, rows densely packed; z
 * [N][Out] in z_dtype.  Any N, In, Out > 0 (the paper's own example is
 * 10 x 10 times a 10-vector); row lengths that are whole 64-byte units (In a
 * multiple of 16 for VGG_F32, 32 for VGG_BF16, as in the network) take the
 * fast path, others are completed with zeros in registers.  The contraction
 * is split over workgroups; partial sums go to ws and are added in a fixed
 * order. */
size_t vgg_fc_workspace_bytes(int dtype, int N, int In, int Out);
int vgg_fc(int dtype, int N, int In, int Out, const void *a, const void *w, const float *bias,
           void *z, int z_dtype, int relu, void *ws, size_t ws_bytes, void *stream);

/* vgg_fc for callers that cannot allocate device memory or carry a workspace
 * around: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and bit-identical results
 * as vgg_fc, but no ws: the partial sums of the split contraction go to a
 * buffer of VGG_FC_STATIC_SCRATCH_BYTES that is part of the library's device
 * image (every GPU the library is used on holds its own copy until the
 * process ends).  Calls no hipMalloc / hipFree and no allocating routine.
 * Returns VGG_ERR_TOO_LARGE, before touching the device, when
 * vgg_fc_workspace_bytes(dtype, N, In, Out) exceeds the buffer (the network's
 * three dense layers at batch 100 fit: 26.2 MB for 25088 -> 4096).
 * All calls on one GPU share that GPU's buffer: calls that may overlap on one
 * GPU (different streams, different host threads) race; calls on one stream
 * are ordered and safe.  The buffer keeps the previous call's partial sums;
 * every value a call reads it has written first, so nothing needs clearing.
 * The first call on a device looks the buffer's address up
 * (hipGetSymbolAddress), which is not a stream operation: make one call
 * before starting a graph capture. */
#define VGG_FC_STATIC_SCRATCH_BYTES (32u << 20)
int vgg_fc_static(int dtype, int N, int In, int Out, const void *a, const void *w, const float *bias,
                  void *z, int z_dtype, int relu, void *stream);

/* dw[o,i] = sum_n dz[n,o] a[n,i]; db[o] = sum_n dz[n,o] (db may be NULL); if
 * da is non-NULL, da[n,i] = sum_o dz[n,o] w[o,i], multiplied by (a[n,i] > 0)
 * when relu_mask != 0 (ReLU backward of the producer of a).  a and w are in
 * `dtype`; dz, dw, db and da are always fp32.  VGG_BF16: dz is rounded to
 * bf16 where it enters a product (not for db), sums are fp32.  Any N, In, Out
 * > 0 for VGG_F32; VGG_BF16 needs In to be a multiple of 8
 * (VGG_ERR_UNSUPPORTED otherwise).  The workspace
 * is needed when da is requested and, for VGG_BF16, always. */
size_t vgg_fc_bwd_workspace_bytes(int dtype, int N, int In, int Out);
int vgg_fc_bwd(int dtype, int N, int In, int Out, const void *a, const void *w, const void *dz,
               float *dw, float *db, void *da, int relu_mask, void *ws, size_t ws_bytes,
               void *stream);

/* ------------------------------------------------------ softmax, loss, SGD */

/* p[n,k] = exp(z[n,k]) / sum_j exp(z[n,j]) per row (listing "softmax"),
 * evaluated with the row maximum subtracted from the exponents. */
int vgg_softmax(int N, int K, const float *z, float *p, void *stream);
/* loss[0] = -(1/N) sum_n log p[n,labels[n]];  dz = (p - onehot(labels))/N.
 * loss and dz may each be NULL.  Labels outside [0,K) contribute nothing
 * (labels live on the device and cannot be validated on the host).  ws needs
 * N floats when loss is requested (per-row terms, summed in a fixed order). */
int vgg_softmax_xent_bwd(int N, int K, const float *p, const int32_t *labels, float *loss,
                         float *dz, void *ws, size_t ws_bytes, void *stream);
/* theta[i] -= lr * grad[i], i < n. */
int vgg_sgd_update(size_t n, float *theta, const float *grad, float lr, void *stream);

/* ------------------------------------------------------------- whole model */

/* Size in bytes of the packed parameter block for cfg, and of the
 * workspaces of the two model-level calls.  0 if cfg is invalid. */
size_t vgg19_packed_bytes(const vgg_config *cfg);
size_t vgg19_forward_workspace_bytes(const vgg_config *cfg);
size_t vgg19_train_workspace_bytes(const vgg_config *cfg);

/* canonical fp32 -> packed block (convolution weights packed and converted,
 * the first dense layer's columns permuted from C,H,W to H,W,C order, biases
 * fp32; with VGG_FLAG_FP32_MASTER the fp32 master copy as well), and back
 * (fp32 configs, or bf16 with VGG_FLAG_FP32_MASTER: the master copy). */
int vgg19_pack_params(const vgg_config *cfg, const vgg19_params *canonical, void *packed,
                      size_t packed_bytes, void *stream);
int vgg19_unpack_params(const vgg_config *cfg, const void *packed, size_t packed_bytes,
                        const vgg19_params *canonical_out, void *stream);

/* Batch of images in, class scores and probabilities out (section "VGG19
 * forward pass").  x_nchw fp32 [N][3][H][W]; logits and probs fp32
 * [N][classes] (either may be NULL). */
int vgg19_forward(const vgg_config *cfg, const float *x_nchw, const void *packed, float *logits,
                  float *probs, void *ws, size_t ws_bytes, void *stream);

/* One training step (section "VGG19 backward pass", with mean softmax
 * cross-entropy in place of the paper's stand-in sum, whose gradient through
 * softmax is identically zero): forward, loss, full backward, then
 * theta <- theta - cfg->lr * grad on the packed block in place.  VGG_F32,
 * or VGG_BF16 with VGG_FLAG_FP32_MASTER: activations, their gradients and
 * the weights the convolutions read are bf16, all sums fp32 (the matrix
 * unit's bf16 x bf16 -> fp32 of the paper's accelerator); gradients with
 * respect to the dense layers' pre-activations are kept in fp32 and rounded
 * where they enter a product; the update goes to the fp32 master copy and
 * the bf16 copy is refreshed from it.  labels int32 [N].  grads_or_null, when given, receives the
 * 38 gradient tensors in canonical layout.  loss (1 float) and logits
 * ([N][classes]) may be NULL.  The fp32 update streams over the whole packed
 * block: the alignment gaps between its tensors (never read by any kernel)
 * take whatever the workspace holds at the matching positions, so zero the
 * workspace once if the block is to be compared byte for byte. */
int vgg19_train_step(const vgg_config *cfg, const float *x_nchw, const int32_t *labels,
                     void *packed_inout, size_t packed_bytes, const vgg19_params *grads_or_null,
                     float *loss, float *logits, void *ws, size_t ws_bytes, void *stream);

/* Launch plan of the two model-level calls, for inspection: writes up to
 * `cap` kernel-kind codes into kinds_host (host memory) and returns how many
 * launches the call makes (negative vgg_status on a bad cfg).  Codes:
 * 1 conv fwd, 2 conv data-grad, 3 conv weight-grad, 4 pool, 5 pool bwd,
 * 6 dense fwd, 7 dense bwd (dW), 8 dense bwd (dA), 9 other. */
int vgg19_plan(const vgg_config *cfg, int training, int *kinds_host, int cap);

/* Launch plan of one convolution call, for inspection (which kernel a shape
 * gets decides the order of its sums, hence which results are bit-identical):
 * op selects vgg_conv3x3_fwd, vgg_conv3x3_fwd_pool, vgg_conv3x3_bwd_data or
 * vgg_conv3x3_bwd_weight with the same dtype and sizes (first call of the
 * network, vgg_conv3x3_fwd_first, excluded).  Writes VGG_PLAN_INFO_LEN ints to
 * info_host (host memory, cap >= VGG_PLAN_INFO_LEN else VGG_ERR_SHAPE):
 *   [0] kernel: 0 register-staged implicit GEMM, 1 / 2 / 3 direct-to-LDS
 *       implicit GEMM with room for 384 / 448 / 192 halo rows, 4 / 5 the
 *       bf16 implicit GEMM with its weights in registers and room for
 *       384 / 448 halo rows, 6 / 7 the same with 320-pixel tiles and one
 *       workgroup per compute unit; weight
 *       gradient: 100 linear tiles, 114 / 116 patches 14 / 16 pixels wide,
 *       103 the kernel for at most three input channels (fp32); 116 / 117
 *       the bf16 kernel and its variant for at most 32 input channels, 118
 *       the bf16 kernel for at most three input channels on image widths
 *       that are multiples of 16 ([4]..[6] then describe 117's plan, which
 *       is what the workspace is sized for)
 *   [1] pixels per tile   [2] output channels per tile
 *   [3] 0: a tile is consecutive pixels, 1: a patch of one image
 *   [4] pixel tiles
 *   [5] workgroups that share one tile's contraction (forward, data gradient)
 *       or partial results that the fixed-order reduction adds (weight gradient)
 *   [6] workgroups of the main launch */
#define VGG_PLAN_FWD 0
#define VGG_PLAN_FWD_POOL 1
#define VGG_PLAN_BWD_DATA 2
#define VGG_PLAN_BWD_WEIGHT 3
#define VGG_PLAN_INFO_LEN 7
int vgg_conv3x3_plan(int op, int dtype, int N, int H, int W, int Cin, int Cout, int *info_host, int cap);

/* Profiling variant of the two model-level calls: runs one forward pass
 * (training == 0) or one training step (training != 0) with a HIP event
 * recorded on `stream` before every step of the launch plan, WAITS for the
 * stream to drain, and writes the kind code (as in vgg19_plan) and the
 * elapsed milliseconds of every step to kinds_host / ms_host (host memory,
 * `cap` entries each, cap >= the plan length else VGG_ERR_WORKSPACE).
 * Returns the number of steps or a negative vgg_status.  Unlike every other
 * entry point it creates and destroys HIP events and synchronises; it exists
 * for measurement only.  Steps that issue two kernels (a dense layer and its
 * split reduction) are timed as one. */
int vgg19_timed(const vgg_config *cfg, int training, const float *x_nchw, const int32_t *labels,
                void *packed, size_t packed_bytes, float *logits, void *ws, size_t ws_bytes,
                int *kinds_host, float *ms_host, int cap, void *stream);

/* Measurement aid, not a step of the path: a loop of nothing but MFMA
 * instructions (register operands, 2x2 accumulator blocks, four waves per
 * SIMD on every CU), bf16 (v_mfma_f32_32x32x16_bf16) or fp32
 * (v_mfma_f32_32x32x2_f32), with all operands 1.0 (bit 0 of random_operands
 * clear) or with random mantissas and signs (set); bit 1 (bf16 only, else
 * VGG_ERR_UNSUPPORTED) selects v_mfma_f32_16x16x32_bf16, twice as many
 * instructions of half the size on the same operands and accumulator
 * registers.  Timing it gives the matrix rate this chip
 * sustains at the clock it holds under that load, against which the
 * convolution kernels' rate can be read next to the data-sheet peak.
 * sink: device buffer of vgg_mfma_probe_sink_bytes() bytes (results are
 * written there so that the loop is not optimised away); *flops_host (host,
 * may be null) receives the number of floating-point operations of the launch.
 * Asynchronous on `stream`; iters > 0 and random_operands in 0..3 else
 * VGG_ERR_SHAPE. */
size_t vgg_mfma_probe_sink_bytes(void);
int vgg_mfma_probe(int dtype, int random_operands, int iters, float *sink, size_t sink_bytes,
                   double *flops_host, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* VGG_MI355X_H */
