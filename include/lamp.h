/*
 * lamp.h -- C ABI of the MI355X (gfx950) compute library for the per-device hot path of the
 * large 3D U-Net of LAMP (arXiv 2006.12575).
 *
 * The paper pipelines a sequential U-Net over devices (Sec. 2.1, Eq. 1: a partition's forward
 * F_k is the composition of its layers, its backward B_k the chain rule; Sec. 2.2, Eq. 2-3: the
 * U-Net as encoder blocks, skip concatenations and decoder blocks).  This library is what runs
 * on ONE device: the layers themselves, a whole U-Net forward / forward+backward, one encoder
 * partition, and sliding-window inference (Sec. 3, Tables 3 and 5 compare windows with one
 * whole-image pass).
 *
 * Conventions, valid for every entry point:
 *   - All tensor pointers are DEVICE pointers unless a comment says "host".  Descriptor structs
 *     and the `params` / `grads` pointer tables are HOST memory, read during the call only.
 *   - Activations are NDHWC: element (n,d,h,w,c) lives at ((((n*D+d)*H+h)*W+w)*ldc + c).
 *     ldc >= c is the channel stride of a voxel, so a tensor may be a channel slice of a wider
 *     (concatenation) buffer.  Batch/spatial strides are dense in units of ldc.
 *   - dtype LAMP_F32: 4-byte IEEE floats.  LAMP_BF16: 2-byte bfloat16 storage, fp32 accumulation,
 *     round-to-nearest-even on store.  Weights have the activation dtype; gamma/beta, statistics,
 *     logits, the loss and every weight gradient are fp32.
 *   - Conv weight W[Co][3][3][3][Ci]; transposed-conv weight Wt[Ci][2][2][2][Co]; head Wh[K][C].
 *   - Ownership: the caller owns every buffer including the workspace; the library allocates
 *     nothing, frees nothing and keeps no pointer after the call returns.
 *   - Asynchrony: a call only enqueues work on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream); outputs are valid once the caller has synchronised the stream.
 *   - Errors: every argument error is detected on the host before anything is launched and
 *     returned as a negative lamp_status; nothing is thrown, nothing aborts.  Device data is
 *     never validated (an out-of-range label is the caller's bug).
 *   - Determinism: the same inputs give bit-identical outputs from call to call (no
 *     floating-point atomics; every reduction has a fixed order).
 *   - Workspace: each call states its need through the matching *_workspace_bytes query;
 *     pointers must be 16-byte aligned (hipMalloc / torch allocations are).
 *   - One tuning switch, read once per process from the environment: LAMP_TUNE="key=value,...".
 *     Results do not depend on it beyond floating-point summation order; it exists for measurements
 *     and for tests that must reach a particular kernel instantiation on a small volume.  Keys:
 *       tile_depth=4|8        depth of the matrix-core conv tile (default: chosen per shape)
 *       no_pack=1             batches of tiny volumes are not packed into one volume
 *       no_split=1            no input-channel split for few-tile, many-channel layers
 *       cb_outer=1            output-channel blocks as grid.y instead of side by side on one XCD
 *       materialise_concat=1  the network entry points keep one concat buffer per decoder level
 *       no_norm_on_load=1     the network entry points write every activated tensor instead of normalising
 *                             a block's first conv output while the second conv loads it
 *       no_bsum=1             lamp_conv3d_dgrad_inorm_relu_bwd runs its two steps as separate passes (the sums of
 *                             the backward from a reduction pass instead of the data gradient's epilogue)
 *       no_walk_stats=1       the matrix-core conv writes its statistics partials per tile for every shape (default:
 *                             per workgroup walk where the output-channel block is 32 wide and walks are long)
 */
#ifndef LAMP_H
#define LAMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LAMP_OK = 0,
    LAMP_ERR_NULL = -1,        /* a required pointer is NULL */
    LAMP_ERR_SHAPE = -2,       /* non-positive / mismatching / unsupported dimension */
    LAMP_ERR_ALIGN = -3,       /* pointer or channel stride not aligned as required */
    LAMP_ERR_DTYPE = -4,       /* unknown or mismatching dtype */
    LAMP_ERR_WORKSPACE = -5,   /* workspace missing or smaller than the query says */
    LAMP_ERR_UNSUPPORTED = -6, /* valid request this build cannot serve */
    LAMP_ERR_HIP = -7          /* a HIP runtime call or kernel launch failed */
} lamp_status;

typedef enum { LAMP_F32 = 0, LAMP_BF16 = 1 } lamp_dtype;

/* NDHWC tensor view. */
typedef struct {
    int32_t n, d, h, w, c;
    int32_t ldc;   /* channel stride of a voxel, >= c */
    int32_t dtype; /* lamp_dtype */
} lamp_tensor_desc;

/*
 * Optional "normalise + ReLU while loading" of an input tensor: channels [0,c_norm) are read as
 *   max(0, gamma[c]*(v - mean[n,c])*rstd[n,c] + beta[c])        (max skipped when relu == 0)
 * and channels [c_norm, c) are read unchanged (the transposed-conv half of a concat buffer).
 * Zero padding is applied AFTER the transform (out-of-volume reads are literal zeros).
 * mean_rstd: fp32 [N][c_norm][2]; gamma, beta: fp32 [c_norm], NULL = 1 / 0.
 */
typedef struct {
    const float *mean_rstd;
    const float *gamma;
    const float *beta;
    int32_t c_norm;
    int32_t relu;
} lamp_norm_in;

const char *lamp_status_string(lamp_status s);
/* Library version and the GPU architecture its kernels were compiled for ("gfx950"). */
const char *lamp_build_info(void);
/* RMSProp update of a set of parameter tensors in one pass (training recipe of Sec. 3: RMSProp, learning
 * rate 1e-3; the update rule is the usual one, v <- alpha v + (1 - alpha) g^2, w <- w - lr g / (sqrt(v) + eps),
 * no momentum, not centred).  For tensor i < count (numel[i] elements, all device pointers): w[i] fp32 master
 * weights and v[i] fp32 running mean squares are updated in place from the fp32 gradient g[i] (as written by
 * the backward entry points); w_out[i], if w_out and w_out[i] are non-null, receives the new weights in
 * out_dtype[i] (LAMP_BF16: rounded to nearest even; LAMP_F32: copied unless it is w[i] itself): the working
 * copy the forward pass reads.  The pointer tables and numel are host arrays, read during the call.  Nothing
 * is allocated; the launches are enqueued on `stream`.
 * Errors: LAMP_ERR_NULL, LAMP_ERR_SHAPE (count or numel negative, lr / alpha / eps out of range),
 * LAMP_ERR_DTYPE (out_dtype), LAMP_ERR_HIP. */
lamp_status lamp_rmsprop_step(int32_t count, const int64_t *numel, float *const *w, float *const *v, const float *const *g,
                              void *const *w_out, const int32_t *out_dtype, float lr, float alpha, float eps, void *stream);

/* ---------------------------------------------------------------------------------------------
 * 3x3x3 convolution, padding 1, stride 1 (the conv of every U-Net block, Sec. 2.2 / Sec. 3).
 *   z[n,d,h,w,co] = bias[co] + sum_{kd,kh,kw,ci} X[n,d+kd-1,h+kh-1,w+kw-1,ci] * W[co,kd,kh,kw,ci]
 * with X = x, or x transformed by *xnorm.  Cross-correlation; out-of-volume reads are zero.
 *   x, z      : activations described by xd, zd (same n,d,h,w; same dtype).
 *   xnorm     : nullable.
 *   bias      : nullable, fp32 [Co].
 *   stats_out : nullable, fp32 [N][Co][2] = (mean, rstd = 1/sqrt(biased var + eps)) of the STORED
 *               z over d,h,w -- the InstanceNorm statistics, produced in the conv epilogue.
 * bf16 requires pointers 16-byte aligned; any Ci, Co >= 1 is accepted (multiples of 32 take the
 * matrix-core kernels).
 */
size_t lamp_conv3d_fwd_workspace_bytes(const lamp_tensor_desc *xd, const lamp_tensor_desc *zd, int want_stats);
lamp_status lamp_conv3d_fwd(const lamp_tensor_desc *xd, const void *x, const lamp_norm_in *xnorm,
                            const void *w, const float *bias,
                            const lamp_tensor_desc *zd, void *z,
                            float *stats_out, float eps,
                            void *ws, size_t ws_bytes, void *stream);

/* Data gradient of the convolution (the adjoint in x; B_k of Sec. 2.1):
 *   dx[n,i,j,k,ci] = sum_{kd,kh,kw,co} dz[n,i-kd+1,j-kh+1,k-kw+1,co] * W[co,kd,kh,kw,ci]  */
size_t lamp_conv3d_dgrad_workspace_bytes(const lamp_tensor_desc *dzd, const lamp_tensor_desc *dxd);
lamp_status lamp_conv3d_dgrad(const lamp_tensor_desc *dzd, const void *dz, const void *w,
                              const lamp_tensor_desc *dxd, void *dx,
                              void *ws, size_t ws_bytes, void *stream);

/* Data gradient of a conv followed by the InstanceNorm + ReLU backward of the layer below it -- the step from the
 * second conv of a U-Net block to its first (Sec. 2.2; B_k of Sec. 2.1 through two layers):
 *   g  = data gradient of the conv, as lamp_conv3d_dgrad(dz, w)        -> g  (described by gd)
 *   dzb = InstanceNorm + ReLU backward of g, as lamp_inorm_relu_bwd(g, z, stats, gamma, beta) -> dzb (described by dzbd)
 * z, stats, gamma, beta: raw conv output, statistics and affine parameters of the layer below, whose activated
 * output was the conv's input in the forward (z has g's n,d,h,w,c).  dzb may be g itself (in place).  dgamma,
 * dbeta, beta_acc as in lamp_inorm_relu_bwd.  On the matrix-core path (bf16, channel counts the tiled kernel takes,
 * z with g's channel stride) the two sums of the backward are taken in the data gradient's epilogue, from the values
 * it stores, and the separate reduction pass over (g, z) is not run; otherwise the two calls above run one after the
 * other.  Either way the results are those of the two calls up to the summation order of the two sums. */
size_t lamp_conv3d_dgrad_inorm_relu_bwd_workspace_bytes(const lamp_tensor_desc *dzd, const lamp_tensor_desc *gd);
lamp_status lamp_conv3d_dgrad_inorm_relu_bwd(const lamp_tensor_desc *dzd, const void *dz, const void *w,
                                             const lamp_tensor_desc *gd, void *g,
                                             const lamp_tensor_desc *zd, const void *z, const float *stats,
                                             const float *gamma, const float *beta,
                                             const lamp_tensor_desc *dzbd, void *dzb,
                                             float *dgamma, float *dbeta, float beta_acc,
                                             void *ws, size_t ws_bytes, void *stream);

/* Weight gradient, always fp32:
 *   dW[co,kd,kh,kw,ci] = beta*dW + sum_{n,d,h,w} dz[n,d,h,w,co] * X[n,d+kd-1,h+kh-1,w+kw-1,ci]
 *   dbias[co]          = beta*dbias + sum dz[...,co]                       (dbias nullable)
 * beta is 0 (overwrite; previous contents ignored) or 1 (accumulate: the synchronous gradient
 * accumulation over micro-batches of Sec. 2.1).  X = x or x transformed by *xnorm. */
size_t lamp_conv3d_wgrad_workspace_bytes(const lamp_tensor_desc *xd, const lamp_tensor_desc *dzd);
lamp_status lamp_conv3d_wgrad(const lamp_tensor_desc *xd, const void *x, const lamp_norm_in *xnorm,
                              const lamp_tensor_desc *dzd, const void *dz,
                              float *dw, float *dbias, float beta,
                              void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * InstanceNorm + ReLU of a conv output (the normalisation/activation of every block).
 * Per (n,c) over V = d*h*w: mean, biased variance, rstd = 1/sqrt(var+eps);
 *   y = max(0, gamma[c]*(z-mean)*rstd + beta[c]).
 *   stats     : fp32 [N][C][2] (mean, rstd).  If stats_given != 0 it is an INPUT (e.g. produced by
 *               lamp_conv3d_fwd) and only the apply pass runs; otherwise it is computed and written.
 *   y         : same shape/dtype as z (own descriptor: ldc may differ); may alias z.
 *   gamma/beta: fp32 [C], NULL = 1 / 0.
 */
size_t lamp_inorm_relu_workspace_bytes(const lamp_tensor_desc *zd);
lamp_status lamp_inorm_relu(const lamp_tensor_desc *zd, const void *z,
                            const float *gamma, const float *beta, float eps,
                            const lamp_tensor_desc *yd, void *y,
                            float *stats, int stats_given,
                            void *ws, size_t ws_bytes, void *stream);

/* lamp_inorm_relu for callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): the same operation with stats_given = 0 and no workspace argument.  The partial moments of
 * the statistics pass live in a fixed device array of LAMP_NOALLOC_SCRATCH_BYTES (8 MiB) inside the library, one
 * copy per GPU, held until the process ends; the call allocates and frees nothing.  The scratch's device address is
 * looked up on the first call on each device (that first call must happen outside a stream capture).
 * Limit: lamp_inorm_relu_workspace_bytes(zd) <= 8 MiB (e.g. 2 x 128^3 x 256 channels), else LAMP_ERR_WORKSPACE and
 * nothing is launched.  Every call on one GPU shares the scratch: calls that overlap on one GPU (two streams, two
 * threads) race; calls on one stream are ordered and need no clearing in between.
 * Errors: as lamp_inorm_relu, plus LAMP_ERR_WORKSPACE (need above the limit), LAMP_ERR_HIP (symbol lookup). */
#define LAMP_NOALLOC_SCRATCH_BYTES (8u << 20)
lamp_status lamp_inorm_relu_noalloc(const lamp_tensor_desc *zd, const void *z, const float *gamma, const float *beta,
                                    float eps, const lamp_tensor_desc *yd, void *y, float *stats, void *stream);

/* Backward of InstanceNorm + ReLU.  With zh = (z-mean)*rstd, u = gamma*zh+beta, g = dy*[u>0]:
 *   dz = gamma*rstd*( g - mean_v(g) - zh*mean_v(g*zh) )        per (n,c)
 *   dgamma[c] = beta_acc*dgamma + sum_{n,v} g*zh ; dbeta[c] = beta_acc*dbeta + sum_{n,v} g   (nullable)
 *   dy, z, dz : same n,d,h,w,c; dz may alias dy.  stats: fp32 [N][C][2] from the forward. */
size_t lamp_inorm_relu_bwd_workspace_bytes(const lamp_tensor_desc *zd);
lamp_status lamp_inorm_relu_bwd(const lamp_tensor_desc *dyd, const void *dy,
                                const lamp_tensor_desc *zd, const void *z, const float *stats,
                                const float *gamma, const float *beta,
                                const lamp_tensor_desc *dzd, void *dz,
                                float *dgamma, float *dbeta, float beta_acc,
                                void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * InstanceNorm + ReLU followed by a squeeze-and-excitation gate (the SEU-Net variant that Sec. 1
 * names through its citations; the gate is the cited squeeze-and-excitation block written out):
 *   a = max(0, gamma*zh + beta)                       (not stored)
 *   m[n,c] = mean_v a                                 squeeze
 *   h = max(0, W1 m + b1),  e = sigmoid(W2 h + b2)    excitation; W1 fp32 [cr][C], W2 fp32 [C][cr],
 *                                                     b1 [cr], b2 [C] nullable (= 0)
 *   y = a * e[n,c] (+ residual)                       residual nullable, same shape/dtype as z
 *   stats     : fp32 [N][C][2] (mean, rstd), an INPUT (from lamp_conv3d_fwd or lamp_inorm_relu).
 *   gate_save : fp32 [N][4*C + cr] output = (m [C], e [C], h [cr], sum_v [u>0] [C], sum_v [u>0]*zh [C])
 *               per sample; the backward reads it.
 * Backward, for upstream dy (the residual's gradient is dy itself, nothing to compute):
 *   de = sum_v dy*a;  through sigmoid, W2, the hidden ReLU and W1 to dm[n,c];
 *   g = [u>0] * (dy*e + dm/V);  dz = gamma*rstd*( g - mean_v(g) - zh*mean_v(g*zh) );
 *   dgamma, dbeta as in lamp_inorm_relu_bwd with this g; dw1, db1, dw2, db2 fp32, all nullable,
 *   all accumulated with beta_acc in {0,1}.  dz may alias dy.
 * 1 <= cr <= 1024, C <= 4096.  One workspace size serves both calls. */
size_t lamp_inorm_relu_se_workspace_bytes(const lamp_tensor_desc *zd, int cr);
lamp_status lamp_inorm_relu_se(const lamp_tensor_desc *zd, const void *z, const float *stats,
                               const float *gamma, const float *beta,
                               int cr, const float *w1, const float *b1, const float *w2, const float *b2,
                               const lamp_tensor_desc *rd, const void *residual,
                               const lamp_tensor_desc *yd, void *y, float *gate_save,
                               void *ws, size_t ws_bytes, void *stream);
lamp_status lamp_inorm_relu_se_bwd(const lamp_tensor_desc *dyd, const void *dy,
                                   const lamp_tensor_desc *zd, const void *z, const float *stats,
                                   const float *gamma, const float *beta,
                                   int cr, const float *w1, const float *w2, const float *gate_save,
                                   const lamp_tensor_desc *dzd, void *dz,
                                   float *dgamma, float *dbeta,
                                   float *dw1, float *db1, float *dw2, float *db2, float beta_acc,
                                   void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * 2x2x2 max pooling, stride 2 (between encoder blocks).  d,h,w of x must be even.
 *   y[n,d,h,w,c] = max_{i,j,k in {0,1}} X[n,2d+i,2h+j,2w+k,c]
 * Backward: dx = dy at the arg-max (first in (i,j,k) raster order under strict '>'), 0 elsewhere,
 * plus add[...] when `add` is given (the gradient arriving through the skip copy of the same
 * tensor, Eq. 3).  x in the backward is the tensor the forward pooled (after *xnorm). */
lamp_status lamp_maxpool2_fwd(const lamp_tensor_desc *xd, const void *x, const lamp_norm_in *xnorm,
                              const lamp_tensor_desc *yd, void *y, void *stream);
lamp_status lamp_maxpool2_bwd(const lamp_tensor_desc *xd, const void *x, const lamp_norm_in *xnorm,
                              const lamp_tensor_desc *dyd, const void *dy,
                              const lamp_tensor_desc *addd, const void *add,
                              const lamp_tensor_desc *dxd, void *dx, void *stream);

/* ---------------------------------------------------------------------------------------------
 * 2x2x2 stride-2 transposed convolution (decoder upsampling; "decoder symmetric", Sec. 3).
 *   y[n,2d+i,2h+j,2w+k,co] = bias[co] + sum_ci X[n,d,h,w,ci] * Wt[ci,i,j,k,co]
 * yd may have ldc = 2*Co with y pointing at channel Co of a concat buffer (zero-copy skip concat).
 * Backward (each output nullable):
 *   dx[n,d,h,w,ci]   = sum_{i,j,k,co} dy[n,2d+i,2h+j,2w+k,co] * Wt[ci,i,j,k,co]
 *   dWt[ci,i,j,k,co] = beta*dWt + sum_{n,d,h,w} X[n,d,h,w,ci] * dy[n,2d+i,2h+j,2w+k,co]   (fp32)
 *   dbias[co]        = beta*dbias + sum dy[...,co]                                          (fp32) */
size_t lamp_convtr3d_workspace_bytes(const lamp_tensor_desc *xd, const lamp_tensor_desc *yd);
lamp_status lamp_convtr3d(const lamp_tensor_desc *xd, const void *x, const lamp_norm_in *xnorm,
                          const void *wt, const float *bias,
                          const lamp_tensor_desc *yd, void *y,
                          void *ws, size_t ws_bytes, void *stream);
size_t lamp_convtr3d_bwd_workspace_bytes(const lamp_tensor_desc *xd, const lamp_tensor_desc *dyd);
lamp_status lamp_convtr3d_bwd(const lamp_tensor_desc *xd, const void *x, const lamp_norm_in *xnorm,
                              const void *wt, const lamp_tensor_desc *dyd, const void *dy,
                              const lamp_tensor_desc *dxd, void *dx,
                              float *dwt, float *dbias, float beta,
                              void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * 1x1x1 head + softmax (+ cross entropy): "a softmax function after decoder D" (Sec. 2.2).
 *   logits[v,k] = bh[k] + sum_c X[v,c]*Wh[k,c]   (fp32 [N,D,H,W,K], dense)
 * lamp_head_fwd writes logits only.  lamp_head_ce additionally takes int32 labels [N,D,H,W] and
 * produces  loss = -(1/V) sum_v log softmax(logits_v)[label_v]  (V = n*d*h*w, device fp32 scalar),
 *   dlogits = (softmax - onehot)/V, and from it dx[v,c] = sum_k dlogits[v,k]*Wh[k,c] (dtype of x),
 *   dWh[k,c] = beta*dWh + sum_v dlogits[v,k]*X[v,c], dbh[k] = beta*dbh + sum_v dlogits[v,k].
 * logits may be NULL in lamp_head_ce.  K <= 16. */
size_t lamp_head_ce_workspace_bytes(const lamp_tensor_desc *xd, int classes);
lamp_status lamp_head_fwd(const lamp_tensor_desc *xd, const void *x, const lamp_norm_in *xnorm,
                          const void *wh, const float *bh, int classes, float *logits, void *stream);
lamp_status lamp_head_ce(const lamp_tensor_desc *xd, const void *x, const lamp_norm_in *xnorm,
                         const void *wh, const float *bh, int classes, const int32_t *labels,
                         float *logits, float *loss,
                         const lamp_tensor_desc *dxd, void *dx, float *dwh, float *dbh, float beta,
                         void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Whole U-Net (Sec. 2.2 Eq. 2; channel schedule of Sec. 3).
 *   levels encoder blocks; block l has C_l = base*2^(l-1) filters; block = two
 *   [conv3x3x3 (no bias) -> InstanceNorm -> ReLU]; 2x2x2 max-pool after every encoder block but the
 *   last; decoder block l = block applied to concat[e_l , convtr(d_{l+1})] (skip first, Eq. 2's
 *   argument order s_l(e_l, d_{l+1})); d_levels is the encoder output; 1x1x1 head to `classes`.
 *   d, h, w must be divisible by 2^(levels-1).
 * Parameter table (host array of device pointers), in this order:
 *   for l = 1..levels:      enc l conv1 W [, gamma, beta], conv2 W [, gamma, beta]
 *   for l = levels-1..1:    up Wt [2C_l][2][2][2][C_l], up bias [C_l] (fp32),
 *                           dec l conv1 W [C_l][3][3][3][2C_l] [, gamma, beta], conv2 W [, gamma, beta]
 *   head Wh [classes][C_1], head bias [classes] (fp32)
 * gamma/beta entries exist only when affine != 0 (fp32 [C]).  W/Wt/Wh have dtype `dtype`.
 * Squeeze-and-excitation variant (the SEU-Net that Sec. 1 names through its citations; se_ratio > 0): every block
 * becomes  a1 = unit1(x),  a2 = ReLU(InstanceNorm(conv2(a1))),  out = a1 + gate(mean_v a2) * a2  with the gate of
 * lamp_inorm_relu_se and cr = max(1, C_l / se_ratio) hidden units; four fp32 entries follow the block's two convs in
 * the table: gate W1 [cr][C_l], b1 [cr], W2 [C_l][cr], b2 [C_l].  Served by lamp_unet_fwd and lamp_unet_fwd_bwd;
 * the partition, tail, pipeline entry points return LAMP_ERR_UNSUPPORTED for it (lamp_sliding_window_fwd serves it).
 * `grads` has the same order; every entry fp32 with the parameter's shape; beta = 0 overwrites,
 * beta = 1 accumulates (micro-batch accumulation, Sec. 2.1).
 */
typedef struct {
    int32_t levels, base, in_ch, classes;
    int32_t n, d, h, w;
    int32_t dtype; /* lamp_dtype of activations and weights */
    float eps;
    int32_t affine;
    int32_t se_ratio; /* 0: plain U-Net; r > 0: squeeze-and-excitation blocks with reduction ratio r */
} lamp_unet_desc;

/* Number of entries of the parameter table, and the element count of entry idx (0 on bad idx). */
int32_t lamp_unet_param_count(const lamp_unet_desc *desc);
int64_t lamp_unet_param_numel(const lamp_unet_desc *desc, int32_t idx);
size_t lamp_unet_workspace_bytes(const lamp_unet_desc *desc, int with_backward);

/* x: [N,D,H,W,in_ch] dense, dtype desc->dtype.  logits: fp32 [N,D,H,W,classes]. */
lamp_status lamp_unet_fwd(const lamp_unet_desc *desc, const void *const *params, const void *x,
                          float *logits, void *ws, size_t ws_bytes, void *stream);
/* Forward, mean softmax cross entropy against int32 labels [N,D,H,W], and the gradient of the loss
 * with respect to every parameter.  loss: device fp32 scalar.  logits nullable. */
lamp_status lamp_unet_fwd_bwd(const lamp_unet_desc *desc, const void *const *params, const void *x,
                              const int32_t *labels, float *logits, float *loss,
                              float *const *grads, float beta,
                              void *ws, size_t ws_bytes, void *stream);

/* One pipeline partition made of encoder blocks first_level..last_level (Sec. 2.1: a partition is a
 * run of consecutive layers; Sec. 2.2 Eq. 3: each e_l leaves the partition twice, as the pooled
 * tensor that feeds the next block and as the skip copy e_{l,1}).  Requires last_level < levels.
 *   x          : input of block first_level ([N,D,H,W,in_ch] when first_level == 1), already at the
 *                resolution of that level (desc->d,h,w are the partition's input dims).
 *   params     : table of the partition's own conv parameters in the order above.
 *   pooled     : output, pool(e_last) [N, D/2^k.., C_last], k = number of blocks.
 *   skips[i]   : output, e_{first+i} (activated), dense.
 * Backward takes x and skips again (the forward's input and outputs, unchanged), the gradients of
 * all outputs, and the SAME workspace the forward ran in, untouched since (it holds the saved conv
 * outputs and statistics); it returns the partition's weight gradients and, when dx != NULL and
 * first_level > 1, the gradient of its input.  desc->d,h,w are the partition's input dims and must
 * be divisible by 2^(number of blocks). */
size_t lamp_unet_stage_workspace_bytes(const lamp_unet_desc *desc, int first_level, int last_level, int with_backward);
lamp_status lamp_unet_stage_fwd(const lamp_unet_desc *desc, int first_level, int last_level,
                                const void *const *params, const void *x,
                                void *pooled, void *const *skips,
                                void *ws, size_t ws_bytes, void *stream);
lamp_status lamp_unet_stage_bwd(const lamp_unet_desc *desc, int first_level, int last_level,
                                const void *const *params, const void *x, const void *const *skips,
                                const void *d_pooled, const void *const *d_skips,
                                float *const *grads, float beta, void *dx,
                                void *ws, size_t ws_bytes, void *stream);

/* The net's tail as the last pipeline partition (Sec. 2.2 Eq. 3: the sequential form of the U-Net,
 * in which the skip copies e_{l,1} of the blocks before the cut travel on to the decoder): encoder
 * blocks first_level..levels, every decoder block and the head.  2 <= first_level <= levels.
 * desc is the WHOLE net's descriptor (d,h,w = the network input's dims).
 *   params / grads : the whole net's tables from entry lamp_unet_tail_param_offset(desc, first_level) on.
 *   x              : pool(e_{first_level-1}), dense [N, D/2^(first_level-1).., C_{first_level-1}].
 *   skips[l-1]     : e_l (activated, dense [N, D/2^(l-1).., C_l]) for l = 1..first_level-1, i.e. what
 *                    lamp_unet_stage_fwd(desc, 1, first_level-1, ...) returns.
 *   d_x, d_skips   : outputs of the backward, the gradients of x (nullable) and of every skip — the
 *                    d_pooled / d_skips that lamp_unet_stage_bwd takes.
 * Only where the decoder reads its concat input from two tensors (bf16, base a multiple of 32, the
 * shapes the matrix-core kernels serve); otherwise LAMP_ERR_UNSUPPORTED and a workspace size of 0. */
int32_t lamp_unet_tail_param_offset(const lamp_unet_desc *desc, int32_t first_level);
size_t lamp_unet_tail_workspace_bytes(const lamp_unet_desc *desc, int first_level, int with_backward);
lamp_status lamp_unet_tail_fwd(const lamp_unet_desc *desc, int first_level, const void *const *params,
                               const void *x, const void *const *skips, float *logits,
                               void *ws, size_t ws_bytes, void *stream);
lamp_status lamp_unet_tail_fwd_bwd(const lamp_unet_desc *desc, int first_level, const void *const *params,
                                   const void *x, const void *const *skips, const int32_t *labels,
                                   float *logits, float *loss, float *const *grads, float beta,
                                   void *d_x, void *const *d_skips,
                                   void *ws, size_t ws_bytes, void *stream);

/* Two partitions, M micro-batches, in the order of the micro-batch pipeline schedule (Sec. 2.1,
 * Fig. 2c), on ONE device: partition 0 = encoder blocks 1..cut on `stream`, partition 1 = the tail
 * on `aux_stream` (a different stream, same device, default priority).  Forward: at clock t
 * partition 0 runs micro-batch t while partition 1 runs micro-batch t-1; backward: micro-batches in
 * reverse, partition 1 one clock ahead of partition 0.  Every micro-batch keeps its activations
 * (no recomputation).  desc describes ONE micro-batch (desc->n samples); x [M*n,D,H,W,in_ch],
 * labels [M*n,D,H,W], logits (nullable) [M*n,D,H,W,classes].
 * Results: loss = mean cross entropy over all M*n samples; grads = beta*grads + its gradient —
 * the same function as lamp_unet_fwd_bwd on the whole mini-batch (InstanceNorm statistics are per
 * sample, so micro-batching changes no activation); only the order of the fp32 sums over samples
 * differs.  Deterministic: the order of accumulation is fixed by the schedule.
 * Stream contract: the call waits (on the device) for the work already enqueued on `stream`, and
 * `stream` waits for everything the call enqueued on `aux_stream`: synchronising `stream` is enough.
 * The call creates and destroys 2M+2 HIP events (no device memory).  1 <= cut < levels, M <= 64.
 * Restrictions of lamp_unet_tail_fwd_bwd apply. */
size_t lamp_unet_pipeline_workspace_bytes(const lamp_unet_desc *desc, int cut, int micro_batches);
lamp_status lamp_unet_pipeline_fwd_bwd(const lamp_unet_desc *desc, int cut, int micro_batches,
                                       const void *const *params, const void *x, const int32_t *labels,
                                       float *logits, float *loss, float *const *grads, float beta,
                                       void *ws, size_t ws_bytes, void *stream, void *aux_stream);

/* ---------------------------------------------------------------------------------------------
 * Sliding-window inference (Sec. 3, Tables 3/5: windows versus one whole-image pass).
 * The volume [1,D,H,W,in_ch] is covered by cubic windows of side `patch` with stride
 * round(patch*(1-overlap)), the last window of an axis clamped to the border; the windows are run
 * through the U-Net as one batch (patch_desc->n must equal the window count and d=h=w=patch), and
 * the window logits are blended with a Gaussian weight of sigma = sigma_scale*patch centred on the
 * window:  out[v] = sum_win g*logits_win[v] / sum_win g.   out: fp32 [1,D,H,W,classes]. */
int32_t lamp_sliding_window_count(int32_t D, int32_t H, int32_t W, int32_t patch, float overlap);
size_t lamp_sliding_window_workspace_bytes(const lamp_unet_desc *patch_desc, int32_t D, int32_t H, int32_t W);
lamp_status lamp_sliding_window_fwd(const lamp_unet_desc *patch_desc, const void *const *params,
                                    const void *vol, int32_t D, int32_t H, int32_t W,
                                    float overlap, float sigma_scale, float *out,
                                    void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LAMP_H */
