/*
 * mi3d — C ABI of the MI355X (gfx950) hot path for full-resolution 3D U-Net
 * training with data swapping.
 *
 * Two groups of entry points:
 *   1. mi3d_conv3d_{fwd,dgrad,wgrad}: the 3-D convolution layers whose
 *      forward output ("feature map A^l") is produced in the forward pass and
 *      needed again by the same layer in the backward pass (paper, Section
 *      3.1 and Fig. 1).  The paper gives no formula (its convolutions ran in
 *      a closed vendor library, Section 4.1); the definitions below are the
 *      textbook ones.
 *   2. mi3d_swap_*: the data-swapping engine (Sections 3.1-3.3): feature maps
 *      are copied to host memory after the forward pass has used them and
 *      copied back before the layer's backward pass, on side streams so that
 *      the copies overlap GPU computation.
 *
 * General rules
 *   - Plain C, no C++ or framework types.  `stream` arguments are a
 *     hipStream_t passed as void* (NULL = the null stream).
 *   - Pointers named x, w, y, dy, dx, dw, ws and every `dev_*` pointer are
 *     DEVICE pointers, 16-byte aligned, owned by the caller.  Descriptor,
 *     config, stats and out-parameters are HOST pointers.
 *   - Every call returns an int status: MI3D_OK (0) or a negative error.
 *     No call aborts or throws.  Convolution calls only enqueue work on the
 *     given stream: they never allocate device memory and never synchronise.
 *   - Convolution calls are re-entrant.  A swap engine must be used from one
 *     host thread at a time.
 */
#ifndef MI3D_H
#define MI3D_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MI3D_OK = 0,
    MI3D_ERR_INVALID_ARG = -1,      /* null pointer, non-positive size, misaligned pointer, kernel larger than padded input */
    MI3D_ERR_UNSUPPORTED = -2,      /* no kernel for this dtype / shape */
    MI3D_ERR_WORKSPACE = -3,        /* ws_bytes smaller than mi3d_conv3d_workspace_bytes() */
    MI3D_ERR_HIP = -4,              /* a HIP runtime call failed; see mi3d_last_hip_error() */
    MI3D_ERR_HOST_POOL = -5,        /* pinned host pool exhausted */
    MI3D_ERR_OVER_BUDGET = -6,      /* no swap plan fits the device budget / arena exhausted */
    MI3D_ERR_BAD_STATE = -7         /* unknown id, double swap-out, swap-in of a tensor that is not on the host, ... */
};

const char *mi3d_status_string(int status);
/* hipError_t value of the most recent failing HIP call on this host thread (0 if none). */
int mi3d_last_hip_error(void);

/* ------------------------------------------------------------------------ */
/* Convolution                                                              */
/* ------------------------------------------------------------------------ */

typedef enum { MI3D_F32 = 0, MI3D_BF16 = 1 } mi3d_dtype;
typedef enum { MI3D_PASS_FWD = 0, MI3D_PASS_DGRAD = 1, MI3D_PASS_WGRAD = 2 } mi3d_pass;

/*
 * Geometry of one layer.
 *   activations  NDHWC, channel fastest:        x[n][d][h][w][ci]
 *   weights      [Cout][kD][kH][kW][Cin]:       w[co][kd][kh][kw][ci]
 *   explicit symmetric zero padding p per side, stride s, cross-correlation
 *   Do = floor((D + 2 pD - kD) / sD) + 1, same for Ho, Wo.
 * dtype is the element type of x, w, y, dy and dx.  Products are accumulated
 * in fp32 in every case; with MI3D_BF16 the results y and dx are rounded to
 * bf16 (nearest even) once at the end.  dw is always fp32.
 */
typedef struct {
    int N, D, H, W, Cin;
    int Cout, kD, kH, kW;
    int sD, sH, sW, pD, pH, pW;
    int dtype; /* mi3d_dtype */
} mi3d_conv_desc;

int mi3d_conv3d_out_dims(const mi3d_conv_desc *desc, int *Do, int *Ho, int *Wo);

/* Bytes of device scratch the given pass needs for this geometry (may be 0).
 * Returns 0 for an invalid descriptor as well; the pass itself reports it. */
size_t mi3d_conv3d_workspace_bytes(const mi3d_conv_desc *desc, int pass);

/* y[n,o,co] = sum_{t,ci} x[n, o*s - p + t, ci] * w[co,t,ci]     (feature map of Section 3.1)
 * x: N*D*H*W*Cin elements, w: Cout*kD*kH*kW*Cin, y: N*Do*Ho*Wo*Cout (fully overwritten). */
int mi3d_conv3d_fwd(const mi3d_conv_desc *desc, const void *x, const void *w, void *y,
                    void *ws, size_t ws_bytes, void *stream);

/* dx = adjoint of the forward map with respect to x:
 * dx[n,i,ci] = sum over (o,t,co) with o*s - p + t == i of dy[n,o,co] * w[co,t,ci].
 * dx is fully overwritten; positions no output read receive 0. */
int mi3d_conv3d_dgrad(const mi3d_conv_desc *desc, const void *dy, const void *w, void *dx,
                      void *ws, size_t ws_bytes, void *stream);

/* dw[co,t,ci] = sum_{n,o} dy[n,o,co] * x[n, o*s - p + t, ci]; needs the saved
 * input x of the layer, which is why feature maps are kept (or swapped).
 * dw (fp32, Cout*kD*kH*kW*Cin elements) is overwritten, not accumulated.
 * The reduction order is fixed, so repeated calls give identical bits. */
int mi3d_conv3d_wgrad(const mi3d_conv_desc *desc, const void *x, const void *dy, float *dw,
                      void *ws, size_t ws_bytes, void *stream);

/* mi3d_conv3d_wgrad for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same result as mi3d_conv3d_wgrad, bit
 * for bit (same kernels); the scratch the kernels need (per-workgroup partial sums, packed operands) is a static
 * device array of MI3D_STATIC_SCRATCH_BYTES inside the library, which every GPU the library runs on holds from the
 * first call until the process ends.  The call allocates nothing and frees nothing.  A geometry whose weight gradient
 * needs more scratch than that (mi3d_conv3d_workspace_bytes(desc, MI3D_PASS_WGRAD) > MI3D_STATIC_SCRATCH_BYTES)
 * returns MI3D_ERR_WORKSPACE and launches nothing; every layer of the 5-level U-Net at 192^3 and 208^3 fits.  All
 * calls on one GPU share the one array: calls that overlap in time on the same GPU (two streams, two threads) race
 * on it and must be serialised by the caller.  x, dy, dw: device pointers as for mi3d_conv3d_wgrad. */
#define MI3D_STATIC_SCRATCH_BYTES (64u << 20)
size_t mi3d_static_scratch_bytes(void);
int mi3d_conv3d_wgrad_static(const mi3d_conv_desc *desc, const void *x, const void *dy, float *dw, void *stream);

/* Channel-range operands for the decoder's 2x2x2 stride-2 up-sampling layers (Section 4.1: up-sampling,
 * then concatenation with the skip connection).  The tensor of x's shape (x of the forward pass and of the weight
 * gradient, dx of the data gradient) may be `Cin` channels starting at channel `offset` of a tensor that holds
 * `pitch` channels per voxel (both multiples of 8; pitch 0 or a null view = dense).  With it the transposed
 * convolution (run as mi3d_conv3d_dgrad with roles swapped) writes straight into its half of the concatenated
 * tensor, leaving the other channels untouched, and its backward passes read their half of that tensor's
 * gradient in place.  Only the k = 2, s = 2, p = 0 MFMA kernels take views (even extents, Cin % 32 == 0,
 * Cout % 64 == 0); any other geometry returns MI3D_ERR_UNSUPPORTED.  The pointer is that of the wide tensor. */
typedef struct {
    int pitch;   /* channels per voxel of the tensor in memory */
    int offset;  /* first channel of the operand */
} mi3d_view;
int mi3d_conv3d_fwd_view(const mi3d_conv_desc *desc, const void *x, const mi3d_view *xv, const void *w, void *y,
                         void *ws, size_t ws_bytes, void *stream);
int mi3d_conv3d_dgrad_view(const mi3d_conv_desc *desc, const void *dy, const void *w, void *dx, const mi3d_view *dxv,
                           void *ws, size_t ws_bytes, void *stream);
int mi3d_conv3d_wgrad_view(const mi3d_conv_desc *desc, const void *x, const mi3d_view *xv, const void *dy, float *dw,
                           void *ws, size_t ws_bytes, void *stream);

/* Virtual concatenation for the decoder's first convolution of a level (Section 4.1: the up-sampled map is
 * concatenated with the skip connection and convolved).  The tensor of x's shape is given as two tensors of
 * Cin / 2 channels each, [x_lo | x_hi] along the channels, and is never materialised: the forward pass and the
 * weight gradient read the two halves, the data gradient writes the two halves of dx (both fully overwritten).
 * The results are those of the plain calls on the concatenated tensor, bit for bit.  `slope` of the forward call:
 * LeakyReLU applied to y as in mi3d_conv3d_fwd_lrelu, 1 = none.  Only the bf16 3x3x3 stride-1 MFMA kernels take
 * halves (Cin % 64 == 0, Cout % 32 == 0, pads <= 2); any other geometry returns MI3D_ERR_UNSUPPORTED, and
 * mi3d_conv3d_pair_supported tells beforehand (1 / 0).  Workspace as for the plain call of the same pass; all
 * pointers device, 16-byte aligned. */
int mi3d_conv3d_pair_supported(const mi3d_conv_desc *desc, int pass);
int mi3d_conv3d_fwd_pair(const mi3d_conv_desc *desc, const void *x_lo, const void *x_hi, const void *w, void *y,
                         float slope, void *ws, size_t ws_bytes, void *stream);
int mi3d_conv3d_dgrad_pair(const mi3d_conv_desc *desc, const void *dy, const void *w, void *dx_lo, void *dx_hi,
                           void *ws, size_t ws_bytes, void *stream);
int mi3d_conv3d_wgrad_pair(const mi3d_conv_desc *desc, const void *x_lo, const void *x_hi, const void *dy, float *dw,
                           void *ws, size_t ws_bytes, void *stream);

/* Data gradient of the convolution that reads a skip connection (the stride-2 convolution that leaves a U-Net level,
 * Section 4.1), finished in one call: the skip tensor has a second reader, the decoder, whose gradient `add` (the skip
 * half of the decoder convolution's data gradient, of dx's shape) is added, and the LeakyReLU derivative of the layer
 * that produced the skip tensor a_in is applied:
 *   dx = (bf16(dgrad(dy, w)) + add) * (a_in > 0 ? 1 : slope),
 * fp32 arithmetic on the bf16-rounded data gradient, one more rounding: the bits of mi3d_conv3d_dgrad followed by
 * mi3d_skip_grad.  0 <= slope <= 1 (1: the sum alone).  bf16 descriptors, and fp32 descriptors that run on the fp32
 * matrix-core kernels (kernel extent <= 3, stride <= 2; all in fp32, no intermediate rounding); other fp32
 * descriptors: MI3D_ERR_INVALID_ARG.  The stride-2 MFMA data-gradient kernels do it in
 * their store path or while they add their fp32 partial gradients; other geometries run the two passes.  Same
 * workspace as mi3d_conv3d_dgrad; add and a_in must not overlap dx. */
int mi3d_conv3d_dgrad_skip(const mi3d_conv_desc *desc, const void *dy, const void *w, const void *add, const void *a_in,
                           float slope, void *dx, void *ws, size_t ws_bytes, void *stream);

/* Convolution whose kernel also produces the statistics of its output for the instance normalisation that follows it
 * (Section 4.1: convolution, instance normalisation, LeakyReLU): y as mi3d_conv3d_fwd (or mi3d_conv3d_fwd_pair when
 * x_hi is not null: x then is the low half), and stats[n][c] = (mean, 1 / sqrt(var + eps)) of the stored bf16 values of
 * y over the voxels of sample n, biased variance, as mi3d_instnorm_stats computes them in a pass of its own (same
 * values up to the order of the fp32 partial sums; the order is fixed, so repeated calls give identical bits).
 * stats: N * Cout * 2 floats, device.  Only the unchunked bf16 3x3x3 stride-1 MFMA forward kernels (and the 4-channel
 * first-layer kernel with 32 output channels) do this
 * (mi3d_conv3d_fwd_stats_supported tells, 1 / 0); other geometries return MI3D_ERR_UNSUPPORTED and the caller runs
 * the two passes.  Workspace as for mi3d_conv3d_fwd. */
int mi3d_conv3d_fwd_stats_supported(const mi3d_conv_desc *desc);
int mi3d_conv3d_fwd_stats(const mi3d_conv_desc *desc, const void *x, const void *x_hi, const void *w, void *y,
                          float eps, float *stats, void *ws, size_t ws_bytes, void *stream);

/* Data gradient whose kernel also produces the two means the backward pass of the instance normalisation of the layer
 * below needs (Section 4.1: that layer is convolution, instance normalisation, LeakyReLU, and a_in is its activated
 * output, the input of this convolution): dx = dgrad(dy, w) as mi3d_conv3d_dgrad computes it, plus add where add is
 * not NULL (the second gradient of a skip connection, of dx's shape: the bits of mi3d_conv3d_dgrad_skip with slope 1),
 * and with g = dx * lrelu'(a_in) (of the stored bf16 values of dx) and xhat = a_in > 0 ? a_in : a_in / slope,
 *   sums[n][c] = (mean over the voxels of g, mean over the voxels of g * xhat),
 * which is what mi3d_instnorm_lrelu_bwd computes in a reduction pass of its own (same values up to the order of the
 * fp32 partial sums; the order is fixed).  mi3d_instnorm_lrelu_bwd_sums then finishes the backward pass without that
 * reduction.  sums: N * Cin * 2 floats, device; 0 < slope <= 1.  Without add: the unchunked bf16 3x3x3 stride-1 MFMA
 * data-gradient kernels and the 1x1x1 head kernel do this; with add: the unchunked 3x3x3 stride-2 kernel (Cout = 64)
 * (mi3d_conv3d_dgrad_insums_supported tells, 1 / 0); other geometries return MI3D_ERR_UNSUPPORTED and the caller runs
 * mi3d_conv3d_dgrad or mi3d_conv3d_dgrad_skip and mi3d_instnorm_lrelu_bwd.  Workspace as for mi3d_conv3d_dgrad; add and
 * a_in must not overlap dx. */
int mi3d_conv3d_dgrad_insums_supported(const mi3d_conv_desc *desc, int with_add);
int mi3d_conv3d_dgrad_insums(const mi3d_conv_desc *desc, const void *dy, const void *w, const void *add,
                             const void *a_in, float slope, void *dx, float *sums, void *ws, size_t ws_bytes,
                             void *stream);

/* Convolution followed by the network's LeakyReLU (Section 4.1) in one call:
 * y = lrelu(conv(x, w)), lrelu(v) = v > 0 ? v : slope * v, applied to the fp32
 * accumulator before the single rounding to bf16.  0 <= slope < 1; bf16
 * descriptors, and fp32 descriptors that run on the fp32 matrix-core kernels
 * (else MI3D_ERR_INVALID_ARG).  The MFMA forward kernels apply it in their
 * epilogue; other geometries run the convolution and one elementwise pass.
 * Same workspace as mi3d_conv3d_fwd. */
int mi3d_conv3d_fwd_lrelu(const mi3d_conv_desc *desc, const void *x, const void *w, void *y, float slope,
                          void *ws, size_t ws_bytes, void *stream);

/* Data gradient through a convolution AND through the LeakyReLU that produced
 * its input: dz_in = dgrad(dy, w) * (a_in > 0 ? 1 : slope), where a_in (device,
 * bf16, shape of x) is the activated input of the layer, whose sign is that of
 * the pre-activation.  Kernels that sum fp32 partial gradients apply the factor
 * before the single rounding to bf16; other geometries run mi3d_conv3d_dgrad
 * and mi3d_leaky_relu_bwd (two roundings).  0 <= slope < 1; bf16 descriptors,
 * and fp32 descriptors that run on the fp32 matrix-core kernels (a_in fp32).  dz_in
 * must not alias a_in.  Same workspace as mi3d_conv3d_dgrad. */
int mi3d_conv3d_dgrad_lrelu(const mi3d_conv_desc *desc, const void *dy, const void *w, const void *a_in, float slope,
                            void *dx, void *ws, size_t ws_bytes, void *stream);

/* Writes the name of the kernel family the dispatcher routes this geometry and pass to (for reports and tests). */
int mi3d_conv3d_kernel_name(const mi3d_conv_desc *desc, int pass, char *buf, size_t buf_len);

/* ------------------------------------------------------------------------
 * Steps of the training step around the convolutions (the network of
 * Section 4.1: LeakyReLU after each 3x3x3 convolution, skip concatenation in
 * the decoder, sigmoid + soft Dice loss on the Dice coefficient of Section
 * 4.3, SGD).  Every pointer is a device pointer, 16-byte aligned unless said
 * otherwise, caller-owned; calls only enqueue work on `stream`.  Element
 * counts n must be multiples of 8.  Status codes as above.
 * ---------------------------------------------------------------------- */

/* a[i] <- a[i] > 0 ? a[i] : slope * a[i]  (bf16, in place). */
int mi3d_leaky_relu_fwd(void *a, size_t n, float slope, void *stream);
/* da[i] <- da[i] * (a[i] > 0 ? 1 : slope), in place on da; a is the OUTPUT of
 * the activation (it has the sign of its input, so the input is not kept). */
int mi3d_leaky_relu_bwd(void *da, const void *a, size_t n, float slope, void *stream);
/* The same on fp32 tensors (the fp32 training step). */
int mi3d_leaky_relu_bwd_f32(float *da, const float *a, size_t n, float slope, void *stream);
/* out[v][0:Ca] = a[v][:], out[v][Ca:Ca+Cb] = b[v][:] over `voxels` voxels
 * (bf16; Ca, Cb multiples of 8).  The decoder's [upsampled, skip] input. */
int mi3d_concat_channels(const void *a, int Ca, const void *b, int Cb, void *out, size_t voxels, void *stream);
/* Inverse of the above: a[v] = in[v][0:Ca], b[v] = in[v][Ca:Ca+Cb]. */
int mi3d_split_channels(const void *in, int Ca, int Cb, void *a, void *b, size_t voxels, void *stream);
/* a[i] <- a[i] + b[i]  (bf16 operands, fp32 add, one rounding). */
int mi3d_add_inplace(void *a, const void *b, size_t n, void *stream);
/* out[v][0:C] = in[v][c_off : c_off + C] for a tensor of C_total channels per voxel (bf16; channel counts and the
 * offset in multiples of 8): one half of a concatenated tensor's gradient without writing the other. */
int mi3d_slice_channels(const void *in, int C_total, int c_off, int C, void *out, size_t voxels, void *stream);
/* out[v][c_off : c_off + C] = in[v][0:C] for a tensor `out` of C_total channels per voxel; the other channels
 * of out are left as they are (the skip connection's half of a concatenated tensor). */
int mi3d_place_channels(const void *in, int C, void *out, int C_total, int c_off, size_t voxels, void *stream);
/* Gradient that reaches a skip connection's source layer, in one pass:
 * da[v][c] <- (da[v][c] + dcat[v][c_off + c]) * (a[v][c] > 0 ? 1 : slope).  da (C channels, in place) is the
 * gradient from the encoder path, dcat (C_total channels) the gradient of the concatenated decoder input whose
 * channels c_off.. belong to the skip tensor, a the skip tensor itself (LeakyReLU output).  fp32 arithmetic, one
 * rounding to bf16. */
int mi3d_skip_grad(void *da, const void *dcat, int C_total, int c_off, const void *a, int C, size_t voxels, float slope,
                   void *stream);

/* Sigmoid + soft Dice over `voxels` voxels (all samples) of `classes` = 3
 * channels: p = sigmoid(logit), per class I = sum p t, P = sum p, T = sum t,
 * loss = 1 - mean_c (2 I + eps) / (P + T + eps).  logits bf16 [voxels][3],
 * labels uint8 [voxels][3] (8-byte aligned), voxels a multiple of 8.
 * Writes sums[9] = {I_c, P_c, T_c} and the loss (device fp32); the partial
 * sums go through ws (mi3d_dice_workspace_bytes) in a fixed order. */
size_t mi3d_dice_workspace_bytes(int classes);
int mi3d_dice_loss(const void *logits, const uint8_t *labels, size_t voxels, int classes, float eps,
                   void *ws, size_t ws_bytes, float *sums, float *loss, void *stream);
/* dlogits (bf16) = d loss / d logits, from the sums of mi3d_dice_loss. */
int mi3d_dice_grad(const void *logits, const uint8_t *labels, size_t voxels, int classes, float eps,
                   const float *sums, void *dlogits, void *stream);

/* The two calls above on fp32 logits / gradients (the fp32 training step); same sums, same order. */
int mi3d_dice_loss_f32(const float *logits, const uint8_t *labels, size_t voxels, int classes, float eps,
                       void *ws, size_t ws_bytes, float *sums, float *loss, void *stream);
int mi3d_dice_grad_f32(const float *logits, const uint8_t *labels, size_t voxels, int classes, float eps,
                       const float *sums, float *dlogits, void *stream);

/* Instance normalisation (Section 4.1: every convolution of the network is followed by an instance normalisation
 * and a LeakyReLU), without learnable scale and shift.  Tensors are bf16 NDHWC with `voxels` voxels per sample and C
 * channels (C % 8 == 0, C <= 512); stats is N x C x 2 floats (mean, 1 / sqrt(var + eps), biased variance over the
 * voxels of one sample and channel); ws needs mi3d_instnorm_workspace_bytes(N, C) bytes.  The reductions use a fixed
 * partition and order (bit-reproducible).
 *   _stats      statistics of the convolution output z.
 *   _lrelu_fwd  z <- a = lrelu((z - mean) * rstd), in place.
 *   _lrelu_bwd  da <- dz, in place, from the gradient da with respect to a, the activated tensor a itself (the
 *               normalised value is taken back from it: a positive slope makes LeakyReLU invertible) and stats:
 *               g = da * lrelu'(xhat), dz = rstd * (g - mean(g) - xhat * mean(g * xhat)).  0 < slope <= 1.
 *   _lrelu_bwd_sums  the same with the two means given (sums: N x C x 2 floats, device, (mean g, mean g xhat), as
 *               mi3d_conv3d_dgrad_insums delivers them): the elementwise pass alone, no workspace. */
size_t mi3d_instnorm_workspace_bytes(int N, int C);
int mi3d_instnorm_stats(const void *z, int N, size_t voxels, int C, float eps, float *stats, void *ws, size_t ws_bytes,
                        void *stream);
int mi3d_instnorm_lrelu_fwd(void *z, const float *stats, int N, size_t voxels, int C, float slope, void *stream);
int mi3d_instnorm_lrelu_bwd(void *da, const void *a, const float *stats, int N, size_t voxels, int C, float slope,
                            void *ws, size_t ws_bytes, void *stream);
int mi3d_instnorm_lrelu_bwd_sums(void *da, const void *a, const float *stats, const float *sums, int N, size_t voxels,
                                 int C, float slope, void *stream);
/* The same three passes on fp32 tensors (the precision Section 4.1's network presumably ran in); statistics,
 * workspace, order of the sums and error codes as above. */
int mi3d_instnorm_stats_f32(const void *z, int N, size_t voxels, int C, float eps, float *stats, void *ws,
                            size_t ws_bytes, void *stream);
int mi3d_instnorm_lrelu_fwd_f32(void *z, const float *stats, int N, size_t voxels, int C, float slope, void *stream);
int mi3d_instnorm_lrelu_bwd_f32(void *da, const void *a, const float *stats, int N, size_t voxels, int C, float slope,
                                void *ws, size_t ws_bytes, void *stream);

/* w[i] <- w[i] - lr * dw[i] on the fp32 master weights; w_bf16[i] <- the
 * updated value rounded to bf16 (the copy the bf16 convolutions read; NULL in
 * the fp32 step, whose convolutions read w itself). */
int mi3d_sgd_update(float *w, const float *dw, void *w_bf16, size_t n, float lr, void *stream);
/* Adam, the optimiser the paper trains with (Section 4.1), on fp32 state (m, v: first and second moment, n values each,
 * zero before step 1): m <- beta1 m + (1 - beta1) dw, v <- beta2 v + (1 - beta2) dw^2,
 * w <- w - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps); w_bf16 as in mi3d_sgd_update.
 * step counts from 1.  MI3D_ERR_INVALID_ARG for step < 1, a beta outside [0, 1) or eps <= 0. */
int mi3d_adam_update(float *w, const float *dw, float *m, float *v, void *w_bf16, size_t n, float lr, float beta1,
                     float beta2, float eps, int step, void *stream);

/* ------------------------------------------------------------------------ */
/* Data-swapping engine                                                     */
/* ------------------------------------------------------------------------ */

/*
 * Vocabulary.  A training step is a list of ops with indices 0..n_ops-1:
 * forward ops first, then backward ops.  A saved tensor (feature map) is
 * produced by op `produce_op`, last read in the forward pass by op
 * `last_fwd_use_op`, and read again by backward ops `bwd_first_use_op` ..
 * `bwd_last_use_op`.  Between last_fwd_use_op and bwd_first_use_op it only
 * occupies memory; that is the interval the engine can move it to the host.
 *
 * Planner knobs, after Section 3.2:
 *   policy MI3D_SWAP_BUDGET   swap the smallest set that brings the peak under
 *                             budget_bytes, earliest-produced / longest-idle /
 *                             largest first (the heuristic of Section 3.2 that
 *                             early feature maps are large and live long)
 *   policy MI3D_SWAP_ALL      swap every eligible tensor          (n_tensors = -1)
 *   policy MI3D_SWAP_FIRST_N  swap the first n_tensors eligible tensors in
 *                             production order                    (n_tensors = N)
 *   exclude_tags              tensors carrying any of these tag bits are never
 *                             swapped (excl_scopes, e.g. the synthesis path)
 *   include_tags              if non-zero, only tensors carrying one of these
 *                             bits are eligible (incl_scopes)
 *   lookahead                 swap-in for a tensor first used by backward op j
 *                             is to be issued when op j - lookahead is launched
 *                             (the `lb` knob: larger = earlier)
 */
enum { MI3D_SWAP_BUDGET = 0, MI3D_SWAP_ALL = 1, MI3D_SWAP_FIRST_N = 2 };
/* What happens to a tensor the policy removes from the device between its
 * last forward and first backward use (Section 5 compares the two and proposes
 * their mix for slow host links):
 *   MI3D_EVICT_SWAP       copied to the pinned pool and back (the paper's method; default)
 *   MI3D_EVICT_RECOMPUTE  dropped and produced again by the caller at its first backward
 *                         use, from the tensors named in mi3d_swap_set_recompute;
 *                         tensors without that option stay on the device
 *   MI3D_EVICT_HYBRID     re-computed where the stated cost is below the time the
 *                         swap-in alone would take on the link, swapped otherwise */
enum { MI3D_EVICT_SWAP = 0, MI3D_EVICT_RECOMPUTE = 1, MI3D_EVICT_HYBRID = 2 };
enum { MI3D_TAG_ENCODER = 1u, MI3D_TAG_DECODER = 2u, MI3D_TAG_INPUT = 4u, MI3D_TAG_HEAD = 8u };

typedef struct {
    size_t budget_bytes;     /* device bytes the step may hold at any op (saved tensors + transients) */
    void  *dev_arena;        /* optional device block sub-allocated by mi3d_swap_alloc(); may be NULL */
    size_t arena_bytes;      /* size of dev_arena (0 if none) */
    size_t host_pool_bytes;  /* pinned host memory to allocate at create (0 = planner-only engine, no HIP calls) */
    int    lookahead;        /* >= 0 */
    int    policy;           /* MI3D_SWAP_* */
    int    n_tensors;        /* for MI3D_SWAP_FIRST_N */
    unsigned exclude_tags;
    unsigned include_tags;
} mi3d_swap_config;

typedef struct {
    uint64_t bytes_out, bytes_in;        /* bytes copied device->host / host->device since create or reset */
    double   copy_ms_out, copy_ms_in;    /* summed event-timed copy durations per direction (completed copies) */
    double   busy_ms;                    /* length of the union of the copy intervals of both side streams */
    uint64_t peak_arena_bytes;           /* peak of the arena bytes in use: handed out by mi3d_swap_alloc(), or freed
                                            but still read by a swap-out in flight (since create or reset) */
    uint64_t arena_high_water_bytes;     /* highest end offset of such a block: the arena the step really needed */
    uint64_t planned_arena_bytes;        /* bytes of saved tensors at the peak of the planner's model (256-byte
                                            units); mi3d_swap_alloc stays below this offset while it can */
    uint64_t static_arena_bytes;         /* extent of the plan's static placement: the arena mi3d_swap_alloc_tensor needs */
    int      n_arena_overflow;           /* allocations that fragmentation pushed above planned_arena_bytes, or that
                                            mi3d_swap_alloc_tensor could not put at their planned place */
    uint64_t planned_peak_bytes;         /* peak of the planner's residency model with the chosen swap set */
    uint64_t unswapped_peak_bytes;       /* same model with nothing swapped */
    int      n_registered, n_planned;    /* tensors known / chosen for swapping */
    int      n_swapped_out, n_swapped_in;/* copies actually issued */
    int      n_recompute;                /* tensors the plan re-computes */
    double   recompute_ms;               /* sum of their stated costs */
    int      n_checksummed;              /* checksum mode: tensors that went out and came back ... */
    int      n_checksum_mismatch;        /* ... and those whose checksum after the swap-in differs from the one before the swap-out */
} mi3d_swap_stats_t;

typedef struct mi3d_swap_engine mi3d_swap_engine;

/* Creates an engine on the current device.  With host_pool_bytes > 0 it
 * allocates that much pinned host memory and two side streams (one per copy
 * direction, default priority).  Returns MI3D_ERR_HIP if that fails. */
int mi3d_swap_create(const mi3d_swap_config *cfg, mi3d_swap_engine **out);
/* Waits for outstanding copies, frees the pool, streams and events. */
int mi3d_swap_destroy(mi3d_swap_engine *e);

/* Ops 0..n_fwd_ops-1 are the forward pass, n_fwd_ops..n_ops-1 the backward pass. */
int mi3d_swap_set_timeline(mi3d_swap_engine *e, int n_fwd_ops, int n_ops);
/* Declares a saved tensor.  ids are caller-chosen, unique, >= 0. */
int mi3d_swap_register(mi3d_swap_engine *e, int id, size_t bytes, int produce_op, int last_fwd_use_op,
                       int bwd_first_use_op, int bwd_last_use_op, unsigned tags);
/* Device bytes op `op` holds besides saved tensors (gradients, workspaces, weights). */
int mi3d_swap_set_transient(mi3d_swap_engine *e, int op, size_t bytes);

/* Optional: measured duration of every op of the timeline (ms, n values) and
 * the host-link rate (GB/s).  With them mi3d_swap_plan schedules the swap-ins
 * by time instead of by op count: the copies share one stream, so they are
 * laid out back to back, latest use first, each ending before its tensor's
 * first backward use (duration = bytes / rate + 15 % + 50 us) and issued at
 * the latest op that starts early enough; `lookahead` stays the minimum
 * distance in ops.  n = 0 returns to the op-count rule.  Invalidates the plan. */
int mi3d_swap_set_op_times(mi3d_swap_engine *e, const float *ms, int n, float link_gbs);
/* Optional: how evicted tensors are handled (MI3D_EVICT_*; default swap) and,
 * per tensor, that the caller can produce it again: cost_ms is the compute
 * time of doing so, dep0 / dep1 the ids of registered tensors that must be on
 * the device for it (-1 = none).  The plan then treats a re-computed tensor as
 * absent between its last forward use and its first backward use, where the
 * caller re-runs the producer, and makes its dependencies present at that op
 * (their swap-ins are scheduled for it; a dependency that is re-computed itself
 * comes first).  The engine issues no work for such tensors: the caller frees
 * the block after the last forward use and allocates a new one before it
 * re-runs the producer.  Both calls invalidate the plan. */
int mi3d_swap_set_eviction(mi3d_swap_engine *e, int eviction);
int mi3d_swap_set_recompute(mi3d_swap_engine *e, int id, float cost_ms, int dep0, int dep1);
/* 1 if the plan re-computes the tensor, 0 if not, <0 on error. */
int mi3d_swap_is_recomputed(mi3d_swap_engine *e, int id);
/* First backward op at which the tensor must be on the device under the
 * current plan: the registered one, or earlier if a re-computation reads it. */
int mi3d_swap_first_use_op(mi3d_swap_engine *e, int id);

/* Host-only: chooses the swap set.  MI3D_ERR_OVER_BUDGET if even the chosen
 * policy's full set leaves the modelled peak above budget_bytes (the plan is
 * still filled in, so callers may inspect and run it), MI3D_ERR_HOST_POOL if
 * the set does not fit the pinned pool (then there is no plan: the queries
 * below and mi3d_swap_out return MI3D_ERR_BAD_STATE until a plan succeeds). */
int mi3d_swap_plan(mi3d_swap_engine *e);
/* 1 if the tensor is in the swap set, 0 if not, <0 on error. */
int mi3d_swap_is_planned(mi3d_swap_engine *e, int id);
/* Op index at whose launch the swap-in of `id` is to be issued:
 * max(first backward op, bwd_first_use_op - lookahead). */
int mi3d_swap_prefetch_op(mi3d_swap_engine *e, int id);
/* Modelled resident bytes at op `op` under the current plan. */
int mi3d_swap_planned_bytes_at(mi3d_swap_engine *e, int op, uint64_t *bytes);

/* Sub-allocates `bytes` (rounded up to 256) from dev_arena for work on
 * `stream`.  A block that was released while copies or kernels were still
 * using it is handed out again only together with a stream wait on those
 * events, so the caller may use it on `stream` at once.  With a plan the
 * allocation stays below planned_arena_bytes (the saved bytes the budget
 * leaves room for) as long as a block there fits, even if `stream` then has
 * to wait for a swap-out that still reads that block.
 * MI3D_ERR_OVER_BUDGET when no block is large enough. */
int mi3d_swap_alloc(mi3d_swap_engine *e, size_t bytes, void *stream, void **dev_ptr);
/* Static placement.  mi3d_swap_plan also lays the saved tensors out in one arena from their lifetimes under the plan:
 * every stay of a tensor on the device gets a fixed offset (largest tensors first, lowest free offset among the stays it
 * shares an op with; the first stay of a swapped tensor lasts until its modelled copy-out has finished).
 * mi3d_swap_static_arena_bytes returns the extent of that layout: an arena of this size holds the whole step, so a
 * caller that allocates exactly this much (mi3d_swap_set_arena, any time no block is handed out) has a device
 * footprint that is fixed by the plan.  mi3d_swap_alloc_tensor hands out the planned range of tensor `id` (first call
 * in a step: its first stay; second call, for a tensor that is swapped or re-computed: its second stay) with the
 * stream waits of mi3d_swap_alloc; if the range is not free (the caller's order of allocations and frees differs
 * from the registered lifetimes) it falls back to mi3d_swap_alloc and counts an overflow.  Freed with mi3d_swap_free /
 * mi3d_swap_release as any block. */
int mi3d_swap_set_arena(mi3d_swap_engine *e, void *dev_arena, size_t arena_bytes);
/* Changes budget_bytes of the configuration (a caller that measures its real footprint tightens the planner's budget by
 * what the measurement exceeds the budget it was given).  Invalidates the plan. */
int mi3d_swap_set_budget(mi3d_swap_engine *e, size_t budget_bytes);
int mi3d_swap_static_arena_bytes(mi3d_swap_engine *e, uint64_t *bytes);
int mi3d_swap_alloc_tensor(mi3d_swap_engine *e, int id, void *stream, void **dev_ptr);
/* Offset of stay 0 or 1 of tensor `id` in the static placement (stay 1 only for tensors that leave the device). */
int mi3d_swap_planned_offset(mi3d_swap_engine *e, int id, int stay, uint64_t *offset);
/* Returns a block; it becomes reusable once the work enqueued on `stream` so
 * far has finished (and, for a tensor being swapped out, once its copy has). */
int mi3d_swap_free(mi3d_swap_engine *e, void *dev_ptr, void *stream);

/* Swap-out (Section 3.1): asynchronous device->host copy of tensor `id` from
 * dev_src into the pinned pool.  The copy starts after the work enqueued on
 * producer_stream so far.  The host thread does not block. */
int mi3d_swap_out(mi3d_swap_engine *e, int id, const void *dev_src, void *producer_stream);
/* The forward pass is done with the device copy of `id`: after the work
 * enqueued on last_consumer_stream so far AND the swap-out copy, dev_src may
 * be reused.  If dev_src came from mi3d_swap_alloc() it is returned to the
 * arena with those two conditions attached; otherwise the call makes
 * last_consumer_stream wait for the copy so that the caller may reuse the
 * memory on that stream. */
int mi3d_swap_release(mi3d_swap_engine *e, int id, void *last_consumer_stream);
/* Swap-in: asynchronous host->device copy of `id` into dev_dst, started after
 * the work enqueued on consumer_stream so far (dev_dst may have been in use
 * there).  Does not make consumer_stream wait; see mi3d_swap_wait_in. */
int mi3d_swap_in(mi3d_swap_engine *e, int id, void *dev_dst, void *consumer_stream);
/* Makes consumer_stream wait until the swap-in of `id` has landed.  Call
 * right before the backward op that reads it. */
int mi3d_swap_wait_in(mi3d_swap_engine *e, int id, void *consumer_stream);
/* The backward pass is done with `id`: its host slot is recycled. */
int mi3d_swap_done(mi3d_swap_engine *e, int id);
/* Checksum mode (a safety net for the event ordering the engine rests on: Section 5 takes for granted that swapping
 * does not change a value).  While on, every swap-out is preceded by a 64-bit checksum of the device block it reads,
 * and every swap-in is followed by one of the block it wrote, both on the side streams; mi3d_swap_stats compares
 * them (n_checksummed, n_checksum_mismatch).  Switch it on after the tensors are registered and before the step;
 * costs two small kernels and one pass over the tensor per copy.  Needs an engine with a pinned pool.
 * mi3d_checksum64 is the same function on any device buffer (8-byte aligned): sum over its 8-byte words of
 * word * (2 * index + 1) modulo 2^64, a trailing piece of fewer than 8 bytes zero-extended; synchronises `stream`
 * and allocates a few KB of device scratch for the call; *value is a host pointer. */
int mi3d_swap_set_verify(mi3d_swap_engine *e, int on);
int mi3d_checksum64(const void *dev, size_t bytes, uint64_t *value, void *stream);
/* Blocks the host until every copy issued so far has finished. */
int mi3d_swap_sync(mi3d_swap_engine *e);
/* Forgets per-step state (tensor residency, host slots, counters) but keeps
 * registrations and the plan, so the same step can run again.  Blocks of
 * mi3d_swap_alloc that were never returned (a step that ended early) go back to
 * the arena after a device synchronisation; their pointers become invalid. */
int mi3d_swap_reset_step(mi3d_swap_engine *e);
/* Collects counters; synchronises with the side streams to time the copies. */
int mi3d_swap_stats(mi3d_swap_engine *e, mi3d_swap_stats_t *out);

#ifdef __cplusplus
}
#endif
#endif /* MI3D_H */
