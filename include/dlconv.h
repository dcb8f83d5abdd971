/*
 * dlconv.h -- C boundary of the MI355X (gfx950) convolution + loss library.
 *
 * One GPU's per-step work of the paper's DeepLabv3+-style segmentation
 * network: dense 2-D convolution with stride, zero padding and dilation
 * (forward, data gradient, filter gradient) on NHWC fp16/bf16 tensors with
 * fp32 accumulation, and the class-weighted per-pixel softmax cross-entropy
 * for the 3-class mask.
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, densely
 *     packed, base address 16-byte aligned.  Descriptor pointers are HOST
 *     pointers.  The library allocates nothing, keeps no state and never
 *     synchronises: work is enqueued on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the call returns at once.
 *   - Outputs are fully overwritten (never accumulated into).
 *   - Arguments are validated on the host before anything is launched; a
 *     failed validation returns an error code and touches no device memory.
 *   - Activations are NHWC, filters KRSC (output channel, filter row, filter
 *     column, input channel).  Convolution is cross-correlation (no filter
 *     flip), one group, no bias.
 *   - Results are deterministic run to run (no floating-point atomics).
 */
#ifndef DLCONV_H
#define DLCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DL_OK = 0,
    DL_ERR_NULL = 1,         /* a required pointer is NULL                        */
    DL_ERR_SHAPE = 2,        /* non-positive extent, empty output, size overflow  */
    DL_ERR_DTYPE = 3,        /* dtype outside what the entry point accepts        */
    DL_ERR_ALIGN = 4,        /* a tensor base is not 16-byte aligned              */
    DL_ERR_WORKSPACE = 5,    /* workspace NULL or smaller than the query says     */
    DL_ERR_UNSUPPORTED = 6,  /* valid request the kernels cannot serve            */
    DL_ERR_LAUNCH = 7        /* the HIP runtime refused a launch                  */
} dl_status;

typedef enum { DL_F16 = 0, DL_BF16 = 1, DL_F32 = 2 } dl_dtype;

enum { DL_PASS_FWD = 0, DL_PASS_BWD_DATA = 1, DL_PASS_BWD_FILTER = 2 };

/* Geometry of one convolution, in the paper's naming of a convolution's
 * dimensions (Sec. "Performance Measurement": filter R x S, image H x W,
 * C input channels, K output channels, batch N).  Plain data, caller-owned. */
typedef struct {
    int32_t N, H, W, C;                 /* input  x : [N, H, W, C]                 */
    int32_t K, R, S;                    /* filter w : [K, R, S, C]                 */
    int32_t stride_h, stride_w;         /* >= 1                                    */
    int32_t pad_h, pad_w;               /* >= 0, zeros on both sides of each axis  */
    int32_t dil_h, dil_w;               /* >= 1, atrous sampling step              */
    int32_t dtype;                      /* dl_dtype of x, w, y, dy, dx: F16 | BF16 */
    int32_t dw_dtype;                   /* dl_dtype of dw: same as dtype, or F32   */
} dl_conv_desc;

/* Output extent  P = floor((H + 2*pad_h - dil_h*(R-1) - 1) / stride_h) + 1,
 * Q likewise along W.  DL_ERR_SHAPE if the descriptor is invalid or P, Q < 1. */
dl_status dl_conv_out_shape(const dl_conv_desc *desc, int32_t *P, int32_t *Q);

/* Bytes of device scratch the given pass (DL_PASS_*) needs; may be 0. */
dl_status dl_conv_workspace_bytes(const dl_conv_desc *desc, int pass, size_t *bytes);

/* Which kernels the given pass of this convolution launches, in order, each with
 * its grid, as text ("name<tile>[workgroups]; ..."), NUL-terminated and cut to
 * buf_bytes.  The answer comes from the entry point's own dispatch code run
 * with launches turned into log lines, so it needs no GPU, touches no device
 * memory and cannot disagree with what a real call does.  For measurement
 * reports and dispatch tests. */
dl_status dl_conv_describe(const dl_conv_desc *desc, int pass, char *buf, size_t buf_bytes);

/* Forward convolution, incl. atrous convolution with a dilation factor
 * (paper, Sec. "Segmentation Architecture"):
 *   y[n,p,q,k] = sum_{r,s,c} x[n, p*stride_h - pad_h + r*dil_h,
 *                               q*stride_w - pad_w + s*dil_w, c] * w[k,r,s,c],
 * out-of-image terms are zero.  x: [N,H,W,C], w: [K,R,S,C], y: [N,P,Q,K],
 * all `dtype`; products are accumulated in fp32 and rounded once (nearest
 * even) on store. */
dl_status conv2d_fwd(const dl_conv_desc *desc, const void *x, const void *w, void *y,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* conv2d_fwd with the point-wise tail fused into the store (paper, Sec.
 * "Single GPU Performance": bias layers are among the point-wise operations
 * around the convolutions, and fusing point-wise operations so that tensors
 * are read and written fewer times is the optimisation being pursued):
 *   y[n,p,q,k] = act(conv2d_fwd(x, w)[n,p,q,k] + bias[k]),
 * act = max(., 0) if relu != 0, identity otherwise.  bias: device float[K]
 * (4-byte aligned) or NULL for none; it is added to the fp32 sum, which is then
 * cut and rounded once.  Everything else as for conv2d_fwd (same workspace). */
dl_status conv2d_fwd_bias_relu(const dl_conv_desc *desc, const void *x, const void *w, const float *bias,
                               int32_t relu, void *y, void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same with a residual input added before the activation (the tail of a
 * ResNet block: the skip connection joins the block's last convolution):
 *   y = act(conv(x, w) + bias[k] + residual)
 * residual: [N,P,Q,K] in the descriptor's dtype, 16-byte aligned, or null
 * (then this is conv2d_fwd_bias_relu).  The sum is formed in fp32 and rounded
 * once.  With a residual the launch takes the kernels that can reach the
 * residual before rounding (the 3x3 halo-tile kernel and the two 5x5 kernels,
 * which store through an LDS staging area, are not among them); workspace as
 * reported by dl_conv_workspace_bytes for the forward pass. */
dl_status conv2d_fwd_bias_add_relu(const dl_conv_desc *d, const void *x, const void *w, const float *bias,
                                   const void *residual, int32_t relu, void *y, void *workspace, size_t workspace_bytes,
                                   void *hip_stream);

/* Data gradient (paper, Sec. "Deep learning ...": each layer is
 * differentiable; backward convolutions in the kernel breakdown): the adjoint
 * of conv2d_fwd with respect to x applied to dy.
 *   dx[n,h,w,c] = sum over (p,r),(q,s),k with p*stride_h - pad_h + r*dil_h == h
 *                 and q*stride_w - pad_w + s*dil_w == w of dy[n,p,q,k]*w[k,r,s,c].
 * dy: [N,P,Q,K], w: [K,R,S,C], dx: [N,H,W,C].  Every element of dx is
 * written, including those no output pixel reaches (zeros). */
dl_status conv2d_bwd_data(const dl_conv_desc *desc, const void *dy, const void *w, void *dx,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* Filter gradient:
 *   dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride_h - pad_h + r*dil_h,
 *                                             q*stride_w - pad_w + s*dil_w, c].
 * x: [N,H,W,C], dy: [N,P,Q,K], dw: [K,R,S,C] in `dw_dtype`.  The reduction
 * over N*P*Q is split across workgroups into fp32 partials held in the
 * workspace and summed in a fixed order. */
dl_status conv2d_bwd_filter(const dl_conv_desc *desc, const void *x, const void *dy, void *dw,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/* Transposed convolution ("deconvolutional" layer; paper, caption of the
 * network schematic in Sec. "Segmentation Architecture": the full-resolution
 * decoder up-samples with such layers).  `desc` names the UNDERLYING
 * convolution, the one this layer is the adjoint of: the layer maps
 * x: [N,P,Q,K] to y: [N,H,W,C] with the filter w: [K,R,S,C] (K = the layer's
 * input channels, C = its output channels),
 *   y[n,h,w,c] = sum over (p,r),(q,s),k with p*stride_h - pad_h + r*dil_h == h
 *                and q*stride_w - pad_w + s*dil_w == w of x[n,p,q,k]*w[k,r,s,c],
 * i.e. every input pixel stamps its filter, scaled, at stride-spaced positions.
 * The output size (H, W) is part of `desc`, so any size whose forward extent
 * (dl_conv_out_shape) is (P, Q) can be produced; no separate output padding.
 * Every element of y is written.  Workspace: dl_conv_workspace_bytes(desc,
 * DL_PASS_BWD_DATA).  Same dtype, alignment, ownership and error rules as
 * conv2d_bwd_data, whose arithmetic this is. */
dl_status conv2d_transpose_fwd(const dl_conv_desc *desc, const void *x, const void *w, void *y,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/* Gradient of conv2d_transpose_fwd with respect to its input:
 *   dx[n,p,q,k] = sum_{r,s,c} dy[n, p*stride_h - pad_h + r*dil_h,
 *                                 q*stride_w - pad_w + s*dil_w, c] * w[k,r,s,c].
 * dy: [N,H,W,C], dx: [N,P,Q,K].  Workspace: dl_conv_workspace_bytes(desc, DL_PASS_FWD). */
dl_status conv2d_transpose_bwd_data(const dl_conv_desc *desc, const void *dy, const void *w, void *dx,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* Gradient of conv2d_transpose_fwd with respect to its filter:
 *   dw[k,r,s,c] = sum_{n,p,q} x[n,p,q,k] * dy[n, p*stride_h - pad_h + r*dil_h,
 *                                              q*stride_w - pad_w + s*dil_w, c].
 * x: [N,P,Q,K], dy: [N,H,W,C], dw: [K,R,S,C] in `dw_dtype`.  Workspace:
 * dl_conv_workspace_bytes(desc, DL_PASS_BWD_FILTER). */
dl_status conv2d_transpose_bwd_filter(const dl_conv_desc *desc, const void *x, const void *dy, void *dw,
                                      void *workspace, size_t workspace_bytes, void *hip_stream);

/* Backward of the point-wise tail of conv2d_fwd_bias_relu in one pass (paper, Sec.
 * "Single GPU Performance": fewer reads and writes of the tensors by fusing
 * point-wise operations): given dy = dL/dy and the forward output y, both
 * [n_pixels, K] in `dtype`,
 *   dz[i,k]  = dy[i,k] if y[i,k] > 0 else 0      (relu != 0; the tensor the
 *              convolution's data- and filter-gradient entry points take as dy)
 *   dbias[k] = sum_i dz[i,k]                      (device float[K], fp32 sums in a fixed order)
 * With relu == 0 only dbias is computed (dz = dy; y and dz may be NULL).  dz may
 * alias dy.  Workspace: dl_bias_relu_bwd_workspace_bytes(n_pixels, K). */
dl_status dl_bias_relu_bwd_workspace_bytes(int64_t n_pixels, int32_t K, size_t *bytes);
dl_status bias_relu_bwd(const void *dy, const void *y, int32_t dtype, int64_t n_pixels, int32_t K, int32_t relu,
                        void *dz, float *dbias, void *workspace, size_t workspace_bytes, void *hip_stream);

/* LARC weight update for a list of layers (paper, Sec. "LARC": a separate learning
 * rate for every layer, the size of the update defined relative to the norm of
 * the layer's weights; the paper does not print the formula: this is the published
 * layer-wise rate with LARC's clipping on SGD with momentum and weight decay).
 * Per tensor, norms over the whole tensor in fp32:
 *   local = trust * ||w|| / (||g|| + weight_decay * ||w|| + eps)   (lr if either norm is 0)
 *   rate  = clip ? min(local, lr) : local * lr
 *   v <- momentum * v + rate * (g + weight_decay * w);   w <- w - v
 * tensors: HOST array of n_tensors entries; w, v: device fp32 (v may be NULL when
 * momentum == 0 and is then not kept), g: device tensor of grad_dtype (F16, BF16 or
 * F32: what conv2d_bwd_filter wrote), count elements each.  rates: device float[n_tensors]
 * receiving each tensor's rate, or NULL.  Two launches per 64 tensors; results do not
 * depend on timing.  Workspace: dl_larc_workspace_bytes(n_tensors). */
typedef struct {
    void *w;
    const void *g;
    void *v;
    int64_t count;
} dl_larc_tensor;
dl_status dl_larc_workspace_bytes(int32_t n_tensors, size_t *bytes);
dl_status larc_sgd_step(const dl_larc_tensor *tensors, int32_t n_tensors, int32_t grad_dtype, float lr, float trust,
                        float weight_decay, float momentum, float eps, int32_t clip, float *rates,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/* Scratch bytes for weighted_pixel_ce_fwd_bwd on n_pixels pixels. */
dl_status dl_ce_workspace_bytes(int64_t n_pixels, size_t *bytes);

/* Class-weighted per-pixel softmax cross-entropy over 3 classes (paper,
 * Sec. "Weighted loss": each pixel's loss is scaled by the weight of its
 * labelled class), value and gradient in one pass:
 *   l_i  = -log softmax(z_i)[label_i]
 *   loss = scale * sum_i class_weights[label_i] * l_i
 *   dlogits_i[c] = scale * class_weights[label_i] * (softmax(z_i)[c] - [c == label_i])
 * logits, dlogits: [n_pixels, 3] in `dtype` (F16 | BF16); labels: [n_pixels]
 * uint8 in {0,1,2} (a pixel with any other value has weight 0: it adds nothing to
 * the loss and its gradient is zero; also in the weight-map and the fused
 * variants below); class_weights:
 * device float[3]; loss: device float[1].  Math is fp32 with the row maximum
 * subtracted.  n_pixels == 0 writes loss = 0. */
dl_status weighted_pixel_ce_fwd_bwd(const void *logits, int32_t dtype, const uint8_t *labels,
                                    const float *class_weights, float scale, int64_t n_pixels,
                                    float *loss, void *dlogits,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* weighted_pixel_ce_fwd_bwd for callers that cannot allocate device memory or
 * carry a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments without the workspace, same
 * kernels, same bits; the per-workgroup partial sums live in a 4 KB array that
 * the library itself holds on every GPU it runs on (resolved on the first call
 * on a device; the call allocates and frees nothing).  Limit: n_pixels <=
 * DL_CE_STATIC_MAX_PIXELS, DL_ERR_SHAPE beyond.  All calls on one GPU share
 * that array: calls that may overlap on one GPU (different streams without an
 * ordering between them, several host threads) race on it and must be ordered
 * by the caller; nothing in it has to survive from one call to the next. */
#define DL_CE_STATIC_MAX_PIXELS 1073741824LL   /* 2^30 */
dl_status weighted_pixel_ce_fwd_bwd_static(const void *logits, int32_t dtype, const uint8_t *labels,
                                           const float *class_weights, float scale, int64_t n_pixels,
                                           float *loss, void *dlogits, void *hip_stream);

/* The same loss with the weight given per pixel (paper, Sec. "Weighted loss":
 * the per-pixel weight map is computed by the input pipeline and handed to the
 * GPU with the image): weight_map[i] stands where class_weights[label_i]
 * stands above.  weight_map: device float[n_pixels], 16-byte aligned, any
 * values (0 masks a pixel out).  17 bytes of traffic per pixel instead of 13.
 * Everything else as for weighted_pixel_ce_fwd_bwd. */
dl_status weighted_pixel_ce_map_fwd_bwd(const void *logits, int32_t dtype, const uint8_t *labels,
                                        const float *weight_map, float scale, int64_t n_pixels,
                                        float *loss, void *dlogits,
                                        void *workspace, size_t workspace_bytes, void *hip_stream);

/* The logits layer fused with the loss (the paper's stated next optimisation,
 * Sec. "Single GPU performance": fuse point-wise work into neighbouring layers
 * so that tensors cross DRAM fewer times; the loss of Sec. "Weighted loss"):
 * the 1x1 convolution from C channels to the 3 classes, the class-weighted
 * softmax cross-entropy and both gradients of that convolution in one pass
 * over x,
 *   z_i = W x_i;   loss = scale * sum_i class_weights[label_i] * (-log softmax(z_i)[label_i])
 *   dz_i = scale * class_weights[label_i] * (softmax(z_i) - onehot(label_i))
 *   dx_i = W^T dz_i;   dW = sum_i dz_i x_i^T
 * x, dx: [n_pixels, C] in `dtype` (F16 | BF16), C % 8 == 0, 32 <= C <= 2048;
 * w: [3, C] in `dtype` (a [3,1,1,C] filter); labels, class_weights, loss as for
 * weighted_pixel_ce_fwd_bwd; logits, dlogits: [n_pixels, 3] in `dtype`, each
 * optional (null: not written; they are copies rounded on store: the loss and
 * the gradients are formed from the unrounded fp32 values); dw: [3, C] in
 * dw_dtype (`dtype` or F32).  All device memory, caller-owned, 16-byte aligned
 * bases; outputs are overwritten.  Sums over pixels are added in a fixed order
 * (run-to-run identical).  Traffic: 4*C + 1 bytes per pixel against 6*C + 13
 * for the four separate calls.  Workspace: dl_logits_ce_workspace_bytes.
 * Errors as for the other entry points, before any launch. */
dl_status dl_logits_ce_workspace_bytes(int64_t n_pixels, int32_t C, size_t *bytes);
dl_status logits_ce_fused_fwd_bwd(const void *x, const void *w, int32_t dtype, const uint8_t *labels,
                                  const float *class_weights, float scale, int64_t n_pixels, int32_t C, void *logits,
                                  float *loss, void *dlogits, void *dx, void *dw, int32_t dw_dtype, void *workspace,
                                  size_t workspace_bytes, void *hip_stream);

const char *dl_status_string(dl_status s);

#ifdef __cplusplus
}
#endif
#endif /* DLCONV_H */
