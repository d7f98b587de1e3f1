/*
 * rn50.h - C ABI of librn50.so: one GPU's share of the synchronous data-parallel ResNet-50
 * training step of "Extremely Large Minibatch SGD: Training ResNet-50 on ImageNet in 15 Minutes",
 * as hand-written HIP kernels for gfx950 (MI355X).
 *
 * Conventions that hold for every entry point
 *   - Every pointer named x, w, y, dx, ..., theta, grad, ws is DEVICE memory owned by the caller,
 *     unless the comment says "host".  Descriptors and hyper-parameter structs are host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work on that stream: they never synchronise, allocate or free device memory.  (rn50_step and
 *     rn50_forward_backward also use two helper streams owned by the context, forked from and joined
 *     back to `stream` with events inside the call, for the filter gradients and for the projection
 *     shortcuts; to the caller the call still behaves as work enqueued on `stream`.)
 *   - Outputs are fully overwritten (no accumulate-into semantics).  Inputs are not modified,
 *     except theta/delta/m which the update rule replaces in place.
 *   - Device pointers must be 16-byte aligned.
 *   - Return value: RN50_OK, or a negative error code; rn50_last_error() gives the text (per
 *     thread).  Arguments are validated before the first HIP call, so every RN50_EINVAL /
 *     RN50_EUNSUPPORTED / RN50_EWORKSPACE path is reachable without a GPU.
 *   - Physical layout: activations NHWC (channels fastest), filters KRSC (input channels fastest),
 *     all fp32.  Logical NCHW / KCRS tensors must be transposed by the caller.
 *   - No C++ exception crosses this boundary.
 */
#ifndef RN50_H
#define RN50_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RN50_OK            0
#define RN50_EINVAL       -1  /* null / misaligned pointer, non-positive dimension, inconsistent arguments */
#define RN50_EUNSUPPORTED -2  /* shape, layout or dtype for which no kernel exists */
#define RN50_EWORKSPACE   -3  /* workspace smaller than rn50_*_workspace_bytes() */
#define RN50_EHIP         -4  /* a HIP call failed; see rn50_last_error() */

#define RN50_LAYOUT_NCHW 0    /* declared for completeness; every kernel returns RN50_EUNSUPPORTED for it */
#define RN50_LAYOUT_NHWC 1

#define RN50_DTYPE_F32  0     /* fp32 operands, fp32 MFMA accumulate (the paper computes in single precision, Section 3) */
#define RN50_DTYPE_BF16 1     /* operands rounded to bf16 (RNE) on the way into LDS, fp32 accumulate and outputs */
/* bf16 activations in memory: the tensors x, y, dy and dx of a call hold bfloat16 bits (2 bytes per element, stored with
 * round-to-nearest-even from the fp32 value the kernel formed; pass them through the float pointers of the signatures),
 * filters and filter gradients stay fp32, products run on the bf16 MFMA (filters rounded on the way into LDS), sums are fp32.
 * conv2d_fwd_bnrelu_input / conv2d_bwd_weight_bnrelu_input form max(0, x*scale + shift) in fp32 and round it once, which is
 * the value a normalising kernel would have stored.  conv2d_bwd_weight needs K % 8 == 0 and C % 8 == 0. */
#define RN50_DTYPE_BF16_ACT 2
/* The same with the layer input x in fp32 (the network's first layer reads the image): conv2d_fwd (x fp32, y bf16) and
 * conv2d_bwd_weight (x fp32, dy bf16) only; conv2d_bwd_weight needs K % 8 == 0. */
#define RN50_DTYPE_BF16_ACT_F32IN 3

#define RN50_OP_FWD        0
#define RN50_OP_BWD_DATA   1
#define RN50_OP_BWD_WEIGHT 2
#define RN50_OP_BWD_DATA_FLIPPED 3 /* conv2d_bwd_data_flipped: no room for the flipped filter */
#define RN50_OP_FWD_BNSTATS 4      /* conv2d_fwd_bnstats: the forward workspace plus the per-tile statistics */

const char *rn50_last_error(void);

/* Tuning and test switches.  None is needed for normal use; every switched path computes the same results.  The library
 * keeps one immutable snapshot of them: a call uses the snapshot current when it starts, rn50_set_option replaces the
 * snapshot (thread-safe), and a context keeps the values it was created under.  The first snapshot takes its values from
 * the environment variables RN50_<NAME IN CAPITALS>, read once.  value_or_null NULL or "" restores the built-in default.
 *   "side_stream"    0/1  rn50_create: filter gradients and projection shortcuts on helper streams (default 1)
 *   "fuse_bn"        0..7 rn50_create: bit mask of the BN + ReLU outputs applied by their consumer: 1 stem -> max pooling,
 *                         2 b -> c, 4 a -> b (default 3; 1 for a context with bf16 activations)
 *   "relu_mask"      0/1  rn50_create: the c layers' BN backward reads a byte mask instead of the block output (default 1)
 *   "igemm_plan"     "bm,bn,split": tile shape (64 or 128 each) and tail split of every forward / data-gradient call
 *   "wgrad_plan"     "bm,bn,split": the same for every filter-gradient call
 *   "plan_overrides" "op,n,c,h,k,r,stride,pad,bm,bn,split;...": rows placed before the measured plan table; rows that
 *                         do not parse are skipped
 *   "no_tuned"       0/1  ignore the measured plan table (cost model only)
 *   "no_stem_kernel" 0/1  send the first layer through the implicit GEMM instead of its own kernel
 *   "conv_bn_stats"  0/1  rn50_create: the forward convolutions gather the BN statistics of their output as they write it
 *                         (conv2d_fwd_bnstats) instead of a separate pass over the tensor (default 1)
 *   "wgrad_group"    0..64 rn50_create (fp32 contexts): 0 = one filter-gradient call per layer (default); k > 0 = the layers
 *                         of k consecutive blocks in one conv2d_bwd_weight_group launch (16 or more: all 52 behind the first)
 *   "wgrad_group_stages"  pixel stages of 32 per work item of a grouped plan (default 48, at least 2; rn50_create: at least 16)
 *   "wgrad_group_tile"    "bm,bn": tile of a grouped plan (64 or 128 each, default 64,64)
 *   "wgrad_group_wgs_per_cu"  0..8: workgroups of a grouped launch that may share a CU (0: as many as fit, default)
 * Host only.  Returns RN50_EINVAL for an unknown name or a malformed plan. */
int rn50_set_option(const char *name, const char *value_or_null);

/* ------------------------------------------------------------------------------------------
 * Convolutions of ResNet-50 (the model of Section 1; geometry from He et al. 2016, Table 1).
 * Cross-correlation, zero padding, square stride, no bias:
 *   y[n,p,q,k] = sum_{r,s,c} x[n, p*stride+r-pad, q*stride+s-pad, c] * w[k,r,s,c]
 * with P = (H + 2*pad - R)/stride + 1 (floor), Q likewise.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    int n, c, h, w;      /* input  N x H x W x C */
    int k, r, s;         /* filter K x R x S x C */
    int stride, pad;
    int layout;          /* RN50_LAYOUT_NHWC */
    int in_dtype;        /* RN50_DTYPE_* */
} rn50_conv_desc;

/* Bytes of scratch the given operation needs for this shape (0 is possible).  Returns 0 for an
 * invalid descriptor as well: the operation itself reports the error. */
size_t rn50_conv_workspace_bytes(const rn50_conv_desc *d, int op);

/* The launch plan the given operation would use for this shape, for reports: tile of bm output rows x bn output columns
 * (output pixels x channels for the forward pass and the data gradient, output channels x filter elements for the filter
 * gradient), number of pieces the reduction is cut into (forward / data gradient: only the last, partial round of tiles
 * is cut; 1 = no partial sums in memory) and workgroups of the main kernel (RN50_OP_FWD_BNSTATS: the forward plan).  Any output
 * pointer may be NULL.  Host only. */
int rn50_conv_plan(const rn50_conv_desc *d, int op, int *bm, int *bn, int *split, int *workgroups);

/* y (N x P x Q x K) = conv(x, w).  ws may be NULL when the required size is 0. */
int conv2d_fwd(const rn50_conv_desc *d, const float *x, const float *w, float *y,
               void *ws, size_t ws_bytes, void *stream);

/* dx[n,h,w,c] = sum over (k,r,s) and (p,q) with h = p*stride+r-pad, w = q*stride+s-pad of
 * dy[n,p,q,k] * w[k,r,s,c].  Every element of dx (N x H x W x C) is written, zeros included. */
int conv2d_bwd_data(const rn50_conv_desc *d, const float *dy, const float *w, float *dx,
                    void *ws, size_t ws_bytes, void *stream);
/* The same in two calls, for callers that compute many data gradients with one set of filters (a training step flips
 * every filter once, in one launch): conv2d_filter_flip writes wt[c][R-1-r][S-1-s][k] = w[k][r][s][c] (K*R*S*C floats,
 * not in place), conv2d_bwd_data_flipped takes it.  conv2d_bwd_data is exactly these two, with wt in its workspace;
 * the results are bit-identical.  Workspace size: rn50_conv_workspace_bytes(d, RN50_OP_BWD_DATA_FLIPPED). */
int conv2d_filter_flip(const rn50_conv_desc *d, const float *w, float *wt, void *stream);
int conv2d_bwd_data_flipped(const rn50_conv_desc *d, const float *dy, const float *wt, float *dx,
                            void *ws, size_t ws_bytes, void *stream);

/* dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride+r-pad, q*stride+s-pad, c].
 * The reduction over n,p,q is split across workgroups and combined in a fixed order: the result
 * is bit-identical from call to call. */
int conv2d_bwd_weight(const rn50_conv_desc *d, const float *x, const float *dy, float *dw,
                      void *ws, size_t ws_bytes, void *stream);

/* The same two operations for a layer whose input is the output of BN + ReLU (Section 2's BN with the statistics of the
 * current minibatch, followed by the ReLU of the bottleneck block) that was never written to memory: the convolution's
 * input is max(0, x[n,h,w,c]*in_scale[c] + in_shift[c]) (one fused multiply-add, then the maximum, in fp32), computed
 * as x is gathered; zero padding stays zero.  in_scale, in_shift: C device floats, 16-byte aligned, as bn_stats_scale_shift
 * writes them.  conv2d_fwd_bnrelu_input needs C % 32 == 0, conv2d_bwd_weight_bnrelu_input C % 4 == 0 (else
 * RN50_EUNSUPPORTED).  Workspace sizes are those of conv2d_fwd / conv2d_bwd_weight for the same descriptor. */
int conv2d_fwd_bnrelu_input(const rn50_conv_desc *d, const float *x, const float *in_scale, const float *in_shift,
                            const float *w, float *y, void *ws, size_t ws_bytes, void *stream);
int conv2d_bwd_weight_bnrelu_input(const rn50_conv_desc *d, const float *x, const float *in_scale, const float *in_shift,
                                   const float *dy, float *dw, void *ws, size_t ws_bytes, void *stream);

/* conv2d_bwd_weight / conv2d_bwd_weight_bnrelu_input for several layers in ONE pair of launches (the filter gradients of a
 * backward pass need nothing from each other, only each its own dy; Section 3's framework computes them layer by layer, the
 * sums are the same).  A layer-sized launch starts, ramps and drains on its own; here the work items of all layers are one
 * list, so a finished workgroup is followed by the next item whatever layer it belongs to.  fp32 operands, C % 4 == 0 and
 * K % 4 == 0 for every layer (else RN50_EUNSUPPORTED).  Per layer the result equals conv2d_bwd_weight's up to the order of
 * the fp32 partial sums (the pixel ranges are cut differently), and is bit-identical from call to call.
 *
 * rn50_wgrad_group_item: one layer.  x, dy, in_scale, in_shift: device pointers, 16-byte aligned (in_scale and in_shift both
 * NULL: plain input; both given: the fused BN + ReLU input of conv2d_bwd_weight_bnrelu_input).  dw_offset: where the layer's
 * gradient [K][R][S][C] starts, in elements from the dw_base given at launch (a multiple of 4).
 *
 * The plan is a blob of rn50_wgrad_group_table_bytes(count) bytes that rn50_wgrad_group_plan writes into HOST memory
 * (table_host; it touches no device memory and launches nothing).  The caller copies the same bytes to device memory (16-byte
 * aligned) and keeps both; conv2d_bwd_weight_group(table_host, table_device, dw_base, stream) reads the launch sizes from
 * the host copy and enqueues the two kernels, which read the device copy.  ws: device workspace of at least
 * rn50_wgrad_group_workspace_bytes(count, items) bytes (0 on invalid arguments), named in the plan and used by every launch
 * of it; launches of one plan (or of plans sharing a workspace) that overlap in time race.  The tuning options in force when
 * the plan is written (wgrad_group_stages, wgrad_group_tile, wgrad_group_wgs_per_cu) are part of it.  Tensors must be
 * smaller than 2^31 elements, as for every convolution call.  Nothing is owned by the library. */
typedef struct rn50_wgrad_group_item {
    rn50_conv_desc desc;
    const float *x;
    const float *in_scale;
    const float *in_shift;
    const float *dy;
    size_t dw_offset;
} rn50_wgrad_group_item;
size_t rn50_wgrad_group_table_bytes(int count);
size_t rn50_wgrad_group_workspace_bytes(int count, const rn50_wgrad_group_item *items);
int rn50_wgrad_group_plan(int count, const rn50_wgrad_group_item *items, void *ws, size_t ws_bytes, void *table_host,
                          size_t table_bytes);
int conv2d_bwd_weight_group(const void *table_host, const void *table_device, float *dw_base, void *stream);

/* conv2d_fwd (in_scale_or_null and in_shift_or_null both NULL) or conv2d_fwd_bnrelu_input (both given) together with
 * the statistics half of the BN that follows the convolution (Section 2's BN with the statistics of the current
 * minibatch): besides y it writes, for the K output channels, save_mean, save_invstd, scale and shift exactly as
 * bn_stats_scale_shift(n, K, P, Q, ..., y, gamma, beta, eps, ...) defines them, with y never read back: every output
 * tile leaves the mean and the sum of squared deviations of its rows per channel (of the values as stored), and one small
 * kernel merges the tiles in tile order (Chan et al.'s pairwise update), so results are bit-identical from call to call.
 * The values differ from bn_stats_scale_shift's only by the order of the fp32 sums.  gamma, beta, save_mean, save_invstd,
 * scale, shift: K device floats each, 16-byte aligned; K % 4 == 0.  Shapes whose forward pass does not run through the
 * tiled kernel (the first layer's own kernel) fall back to the separate statistics pass inside this call.
 * Workspace: rn50_conv_workspace_bytes(d, RN50_OP_FWD_BNSTATS). */
int conv2d_fwd_bnstats(const rn50_conv_desc *d, const float *x, const float *in_scale_or_null, const float *in_shift_or_null,
                       const float *w, float *y, const float *gamma, const float *beta, float eps, float *save_mean,
                       float *save_invstd, float *scale, float *shift, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Batch normalization that uses ONLY the current minibatch's statistics (Section 2, "Batch
 * Normalization without Moving Averages"): no running average is read or written anywhere.
 * Per channel c over the M = N*H*W elements:
 *   mean = (1/M) sum x,  var = (1/M) sum (x-mean)^2,  invstd = 1/sqrt(var + eps)
 *   y = gamma*(x-mean)*invstd + beta  [+ residual]  [then ReLU]
 * save_mean / save_invstd (C floats each) are the "last minibatch" statistics the paper keeps.
 * ------------------------------------------------------------------------------------------ */
size_t rn50_bn_workspace_bytes(int n, int c, int h, int w);

int bn_fwd_batchstats(int n, int c, int h, int w, int layout,
                      const float *x, const float *gamma, const float *beta, float eps,
                      const float *residual_or_null, int relu,
                      float *y, float *save_mean, float *save_invstd,
                      void *ws, size_t ws_bytes, void *stream);

/* bn_fwd_batchstats for callers that cannot allocate device memory or carry a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments less the workspace, same kernels, bit-identical
 * results.  The band partials live in a buffer built into the library (RN50_BN_STATIC_SCRATCH_BYTES of device memory per
 * GPU, held until the process ends); the call allocates and frees nothing.  Shapes whose rn50_bn_workspace_bytes()
 * exceeds the buffer return RN50_EWORKSPACE (every ResNet-50 BN shape up to 2048 channels fits).  All calls on one GPU
 * share the buffer: calls that overlap on one GPU (different streams, or different threads) race; calls ordered on one
 * stream do not.  Nothing in the buffer has to be cleared between calls. */
#define RN50_BN_STATIC_SCRATCH_BYTES ((2 * 512 + 4) * 2048 * 4)
int bn_fwd_batchstats_static(int n, int c, int h, int w, int layout,
                             const float *x, const float *gamma, const float *beta, float eps,
                             const float *residual_or_null, int relu,
                             float *y, float *save_mean, float *save_invstd, void *stream);

/* bn_fwd_batchstats(relu = 1) that also writes what the backward pass needs of y: relu_mask, one byte per four
 * consecutive channels (N*H*W*C/4 device bytes; byte i covers elements 4i .. 4i+3, bit e = [y[4i+e] > 0]).
 * bn_bwd_batchstats_mask is bn_bwd_batchstats(relu = 1) reading that mask instead of y (4 bytes less per element). */
int bn_fwd_batchstats_mask(int n, int c, int h, int w, int layout, const float *x, const float *gamma, const float *beta,
                           float eps, const float *residual_or_null, float *y, uint8_t *relu_mask, float *save_mean,
                           float *save_invstd, void *ws, size_t ws_bytes, void *stream);
int bn_bwd_batchstats_mask(int n, int c, int h, int w, int layout, const float *x, const float *dy, const float *dy2_or_null,
                           const uint8_t *relu_mask, const float *gamma, const float *save_mean, const float *save_invstd,
                           float *dx, float *dresidual_or_null, float *dgamma, float *dbeta,
                           void *ws, size_t ws_bytes, void *stream);

/* The statistics half of bn_fwd_batchstats alone, for a consumer that normalises as it loads (the *_bnrelu_input calls):
 * writes save_mean, save_invstd and scale[c] = gamma[c]*invstd[c], shift[c] = fma(-mean[c], scale[c], beta[c]) (C device
 * floats each, 16-byte aligned), so that BN(x) = fma(x, scale, shift): exactly the values bn_fwd_batchstats normalises
 * with.  Same workspace as bn_fwd_batchstats. */
int bn_stats_scale_shift(int n, int c, int h, int w, int layout, const float *x, const float *gamma, const float *beta,
                         float eps, float *save_mean, float *save_invstd, float *scale, float *shift,
                         void *ws, size_t ws_bytes, void *stream);

/* The normalising half of bn_fwd_batchstats alone, with the coefficients bn_stats_scale_shift or conv2d_fwd_bnstats
 * left: y = fma(x, scale[c], shift[c]) [+ residual] [then ReLU]; relu_mask_or_null (relu must be 1) receives the byte
 * mask of bn_fwd_batchstats_mask.  No workspace.  bn_fwd_apply_bf16: the same for bfloat16 tensors (x, residual, y). */
int bn_fwd_apply(int n, int c, int h, int w, int layout, const float *x, const float *scale, const float *shift,
                 const float *residual_or_null, int relu, float *y, uint8_t *relu_mask_or_null, void *stream);
int bn_fwd_apply_bf16(int n, int c, int h, int w, int layout, const uint16_t *x, const float *scale, const float *shift,
                      const uint16_t *residual_or_null, int relu, uint16_t *y, uint8_t *relu_mask_or_null, void *stream);

/* bn_bwd_batchstats for the common case BN -> ReLU with no residual, one incoming gradient and no residual gradient,
 * WITHOUT the forward output: where no residual was added the forward output is max(0, fma(x, scale, shift)) with
 * scale = gamma*invstd, shift = fma(-mean, scale, beta), so the mask [y > 0] is rebuilt bit for bit from x, beta and
 * the saved statistics (8 fewer bytes per element).  beta: C device floats, the forward's.  Otherwise as
 * bn_bwd_batchstats(relu = 1). */
int bn_bwd_batchstats_xmask(int n, int c, int h, int w, int layout, const float *x, const float *dy, const float *gamma,
                            const float *beta, const float *save_mean, const float *save_invstd, float *dx, float *dgamma,
                            float *dbeta, void *ws, size_t ws_bytes, void *stream);

/* The same family for activations kept as bfloat16 in memory (RN50_DTYPE_BF16_ACT): x, y, residual, dy, dy2, dx and
 * dresidual hold bfloat16 bits (2 bytes per element, N x H x W x C); gamma, beta, statistics, scale, shift, dgamma, dbeta
 * and the workspace are fp32 as above.  Values are widened exactly on load, all arithmetic and every sum is fp32, a store
 * rounds to nearest even.  Same workspace size, alignment rules and error codes as the fp32 calls.
 *   bn_fwd_batchstats_bf16: bn_fwd_batchstats; when relu_mask_or_null is given (relu must be 1) it also writes the byte
 *     mask of bn_fwd_batchstats_mask.  The ReLU decision is the sign of the value AS STORED (a tiny positive value that
 *     rounds to zero counts as zero), so that the backward pass, which sees only stored tensors, takes the same one.
 *   bn_stats_scale_shift_bf16: bn_stats_scale_shift.
 *   bn_bwd_batchstats_bf16: the three backward calls in one; the ReLU mask (relu != 0) comes from y_or_null, else from
 *     relu_mask_or_null, else it is rebuilt from x as bn_bwd_batchstats_xmask does, which needs beta_or_null and allows
 *     neither dy2 nor dresidual.  When dresidual is requested, dz is rounded to bf16 first and that value is what the
 *     sums and dx are formed from (it is the one value of dz that exists in memory). */
int bn_fwd_batchstats_bf16(int n, int c, int h, int w, int layout, const uint16_t *x, const float *gamma, const float *beta,
                           float eps, const uint16_t *residual_or_null, int relu, uint16_t *y, uint8_t *relu_mask_or_null,
                           float *save_mean, float *save_invstd, void *ws, size_t ws_bytes, void *stream);
int bn_stats_scale_shift_bf16(int n, int c, int h, int w, int layout, const uint16_t *x, const float *gamma, const float *beta,
                              float eps, float *save_mean, float *save_invstd, float *scale, float *shift,
                              void *ws, size_t ws_bytes, void *stream);
int bn_bwd_batchstats_bf16(int n, int c, int h, int w, int layout, const uint16_t *x, const uint16_t *dy,
                           const uint16_t *dy2_or_null, const uint16_t *y_or_null, const uint8_t *relu_mask_or_null,
                           const float *gamma, const float *beta_or_null, const float *save_mean, const float *save_invstd,
                           int relu, uint16_t *dx, uint16_t *dresidual_or_null, float *dgamma, float *dbeta,
                           void *ws, size_t ws_bytes, void *stream);

/* Validation-side BN (Section 2: no moving averages; the last minibatch's statistics are used, averaged
 * over the workers before validation):
 *   y = gamma*(x - mean)*invstd + beta [+ residual] [ReLU]   with the GIVEN per-channel mean and invstd.
 * Same layout, alignment and workspace rules as bn_fwd_batchstats (workspace: rn50_bn_workspace_bytes).
 * x, y, residual: N x H x W x C device floats; gamma, beta, mean, invstd: C device floats.  y is overwritten. */
int bn_fwd_inference(int n, int c, int h, int w, int layout, const float *x, const float *gamma, const float *beta,
                     const float *mean, const float *invstd, const float *residual_or_null, int relu, float *y,
                     void *ws, size_t ws_bytes, void *stream);
/* The averaging itself, after the sets have been gathered (with one GPU: n_sets = 1, the identity):
 * means, invstds: n_sets x c device floats as bn_fwd_batchstats saved them (invstd = 1/sqrt(var + eps));
 * mean_out = arithmetic mean of the means, invstd_out = 1/sqrt(arithmetic mean of the variances + eps).
 * Sets are added in index order.  Outputs: c device floats each, overwritten. */
int bn_stats_average(int c, int n_sets, const float *means, const float *invstds, float eps, float *mean_out,
                     float *invstd_out, void *stream);

/* Backward of the above.  The incoming gradient is dy (+ dy2 when not NULL: the two consumers of a
 * residual-network activation).  dz = (dy+dy2) * [y > 0] when relu != 0 (mask taken from the stored
 * forward output y, never recomputed; derivative at exactly 0 is 0), else dz = dy+dy2.
 *   dbeta = sum dz,  dgamma = sum dz*xhat,  xhat = (x-mean)*invstd
 *   dx = gamma*invstd*(dz - dbeta/M - xhat*dgamma/M)
 *   dresidual = dz  (written when dresidual_or_null != NULL)
 * y_or_null is required when relu != 0. */
int bn_bwd_batchstats(int n, int c, int h, int w, int layout,
                      const float *x, const float *dy, const float *dy2_or_null, const float *y_or_null,
                      const float *gamma, const float *save_mean, const float *save_invstd, int relu,
                      float *dx, float *dresidual_or_null, float *dgamma, float *dbeta,
                      void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * The remaining layers of ResNet-50 (He et al. 2016), NHWC.
 * ------------------------------------------------------------------------------------------ */
/* 3x3 / stride 2 / pad 1 max pooling (padding never wins).  y is N x P x Q x C with P = (H-1)/2+1.
 * argidx (uint8, same shape as y) receives r*3+s of the first maximal element in row-major window
 * order; the backward routes the gradient there. */
int maxpool3x3s2_fwd(int n, int c, int h, int w, const float *x, float *y, uint8_t *argidx, void *stream);
/* The same over max(0, x*in_scale[c] + in_shift[c]) (the stem's BN + ReLU applied to every value as it is loaded;
 * in_scale, in_shift: C device floats from bn_stats_scale_shift). */
int maxpool3x3s2_fwd_bnrelu_input(int n, int c, int h, int w, const float *x, const float *in_scale, const float *in_shift,
                                  float *y, uint8_t *argidx, void *stream);
/* dx[n,h,w,c] = sum of (dy+dy2)[n,p,q,c] over the windows whose arg-max is (h,w). */
int maxpool3x3s2_bwd(int n, int c, int h, int w, const float *dy, const float *dy2_or_null,
                     const uint8_t *argidx, float *dx, void *stream);
/* Global average pooling: y[n,c] = mean over H*W; dx[n,h,w,c] = dy[n,c]/(H*W). */
int avgpool_fwd(int n, int c, int h, int w, const float *x, float *y, void *stream);
int avgpool_bwd(int n, int c, int h, int w, const float *dy, float *dx, void *stream);
/* The pooling layers for activations kept as bfloat16 in memory: x, y, dy, dy2, dx of the max pooling and x / dx of the
 * average pooling hold bfloat16 bits; the pooled features and their gradient (N x C) are fp32.  maxpool3x3s2_fwd_bf16 with
 * in_scale / in_shift pools max(0, x*in_scale[c] + in_shift[c]) rounded to bf16 (the BN + ReLU output as stored); both NULL
 * pools x itself. */
int maxpool3x3s2_fwd_bf16(int n, int c, int h, int w, const uint16_t *x, const float *in_scale_or_null,
                          const float *in_shift_or_null, uint16_t *y, uint8_t *argidx, void *stream);
int maxpool3x3s2_bwd_bf16(int n, int c, int h, int w, const uint16_t *dy, const uint16_t *dy2_or_null,
                          const uint8_t *argidx, uint16_t *dx, void *stream);
int avgpool_fwd_bf16(int n, int c, int h, int w, const uint16_t *x, float *y, void *stream);
int avgpool_bwd_bf16(int n, int c, int h, int w, const float *dy, uint16_t *dx, void *stream);
/* Fully connected layer: y[n,k] = sum_j f[n,j]*w[k,j] + b[k]. */
int fc_fwd(int n, int j, int k, const float *f, const float *w, const float *b, float *y, void *stream);
/* df[n,j] = sum_k dy[n,k] w[k,j];  dw[k,j] = sum_n dy[n,k] f[n,j];  db[k] = sum_n dy[n,k]. */
int fc_bwd(int n, int j, int k, const float *f, const float *w, const float *dy,
           float *df, float *dw, float *db, void *stream);
/* Softmax cross-entropy, mean over the local minibatch: loss[0] = -(1/N) sum_n log softmax(z_n)[label_n],
 * dlogits = (softmax - onehot)/N.  labels: N int32 in [0,K) on the device (a label outside that range is not an error
 * code, since the labels are device memory: it makes the loss NaN and contributes no one-hot term).  N <= 1024. */
int softmax_ce(int n, int k, const float *logits, const int32_t *labels, float *loss, float *dlogits, void *stream);

/* ------------------------------------------------------------------------------------------
 * Half-precision communication buffer (Section 3, "Software": compute in single precision,
 * all-reduce in half precision).  out16[i] = IEEE binary16 of g[i], round-to-nearest-even,
 * overflow to +-inf, gradual underflow, signed zero kept.  One flat buffer, no padding.
 * ------------------------------------------------------------------------------------------ */
int grad_pack_fp16(size_t count, const float *g, uint16_t *out16, void *stream);
/* g[i] = float(in16[i]) * scale (scale = 1/#workers; exact for a power of two). */
int grad_unpack_fp16(size_t count, const uint16_t *in16, float scale, float *g, void *stream);

/* ------------------------------------------------------------------------------------------
 * Update rule of Appendix A.1, per element, in this order:
 *   g' = g_scale * g  (+ wd * theta where decay applies; not part of the paper's equations)
 *   m     <- mu2*m + (1-mu2)*g'^2
 *   delta <- mu1*delta - (a_sgd + a_rms/(sqrt(m)+eps))*g'
 *   theta <- theta + eta*delta
 * a_rms = 0, a_sgd = 1 is momentum SGD; a_sgd = 0 is RMSprop with momentum.
 * Exactly one of g (fp32) and g16 (the half-precision buffer, unpack fused) must be non-NULL.
 * wd_mask_or_null: one byte per group of RN50_WD_GROUP consecutive elements, non-zero = decay
 * applies to that group; NULL = decay applies everywhere.  Ignored when wd == 0.
 * ------------------------------------------------------------------------------------------ */
#define RN50_WD_GROUP 64
typedef struct { float eta, mu1, mu2, eps, a_sgd, a_rms, wd, g_scale; } rn50_opt_hparams;
int opt_update(size_t count, float *theta, float *delta, float *m,
               const float *g_or_null, const uint16_t *g16_or_null,
               const uint8_t *wd_mask_or_null, const rn50_opt_hparams *hp /* host */, void *stream);

/* Schedules of Appendix A.1 / A.2 (host scalars).  rn50_alpha_sgd uses slope 1/period on the linear
 * branch, which is the reading under which the function reaches 1 at center+period/2 as the text
 * says (the printed slope 2/period would give 1.5 there). */
double rn50_alpha_sgd(double epoch, double center, double period);
/* Appendix A.1 also names the transitions it examined and rejected (a sudden switch as in the Adam-to-SGD scheme it
 * cites, a linear and a sigmoid function) without giving formulas.  They are offered as scalar variants, each the plainest
 * function of its name through 1/2 at `center`, the smooth ones with slope 1/period there like the paper's own:
 *   RN50_TRANSITION_ELU     the paper's function (rn50_alpha_sgd)
 *   RN50_TRANSITION_LINEAR  clip(1/2 + (epoch-center)/period, 0, 1)
 *   RN50_TRANSITION_SIGMOID 1 / (1 + exp(-4 (epoch-center)/period))
 *   RN50_TRANSITION_SUDDEN  0 before center, 1 from it on
 * Returns NaN for any other `transition`. */
#define RN50_TRANSITION_ELU 0
#define RN50_TRANSITION_LINEAR 1
#define RN50_TRANSITION_SIGMOID 2
#define RN50_TRANSITION_SUDDEN 3
double rn50_alpha_sgd_transition(double epoch, double center, double period, int transition);
double rn50_alpha_rmsprop(double a_sgd, double eta_rmsprop, double eta_sgd);
double rn50_lr_base(int n_workers, int b_local);
double rn50_lr_slow_start(double epoch, int n_workers, int b_local);
/* All scalars of one iteration of the paper's recipe at (real-valued) `epoch`, for n_workers workers of b_local
 * images each (Section 4: 1024 x 32): eta = the slow-start learning rate (Appendix A.2), a_sgd / a_rms = the warm-up
 * blend (Appendix A.1; center 10, period 5, eta_RMSprop 3e-4), mu1 = 0.9, mu2 = 0.99, eps = 1e-8 (Appendix A.1),
 * wd = 1e-4 (inherited, see opt_update), g_scale = 1/n_workers (the all-reduce sums, the rule wants the mean).
 * Host only.  Returns RN50_EINVAL for a null pointer, negative epoch or non-positive counts. */
int rn50_recipe_hparams(double epoch, int n_workers, int b_local, rn50_opt_hparams *hp_out /* host */);
/* The same with one of the transition functions above in place of the paper's (Appendix A.1's comparison); also
 * RN50_EINVAL for an unknown `transition`. */
int rn50_recipe_hparams_transition(double epoch, int n_workers, int b_local, int transition, rn50_opt_hparams *hp_out /* host */);

/* ------------------------------------------------------------------------------------------
 * Whole training step: forward, loss, backward, half-precision pack, unpack*g_scale, update.
 * Parameters, gradients and optimizer state are flat fp32 arenas of rn50_param_count() elements
 * in parameter-table order (forward traversal: conv filter, BN scale, BN shift per layer, then
 * FC weight, FC bias); this is also the order of the half-precision buffer.
 * ------------------------------------------------------------------------------------------ */
#define RN50_KIND_CONV_W 0
#define RN50_KIND_BN_G   1
#define RN50_KIND_BN_B   2
#define RN50_KIND_FC_W   3
#define RN50_KIND_FC_B   4

#define RN50_VARIANT_V1 0     /* stride 2 on the first 1x1 of the first block of stages 3-5 */
#define RN50_VARIANT_V15 1    /* stride 2 on the 3x3 of those blocks instead (same parameters; 4.09 instead of 3.86 GMAC/image) */

size_t rn50_param_count(void);
int rn50_param_table_size(void);
/* Entry idx of the table.  name: static string.  dims: K,R,S,C for filters; K,J,1,1 for the FC weight;
 * count,1,1,1 otherwise.  offset, count in elements of the flat arenas. */
int rn50_param_table(int idx, const char **name, size_t *offset, size_t *count, int dims[4], int *kind);

typedef struct rn50_ctx rn50_ctx;
/* Bytes of device memory rn50_step needs for activations, gradients of activations and kernel scratch. */
size_t rn50_activation_bytes(int batch, int variant);
/* Plans the step for `batch` images of 3x224x224 inside the caller's arena (act_bytes >= the above;
 * 256-byte aligned).  Host-side only, except one small upload (the weight-decay mask) into the arena. */
int rn50_create(rn50_ctx **out, int batch, int variant, int conv_dtype, void *act_arena, size_t act_bytes);
/* conv_dtype: RN50_DTYPE_F32 (the paper's single precision), RN50_DTYPE_BF16 (convolution operands rounded to bf16 on the
 * way into LDS, everything in memory fp32) or RN50_DTYPE_BF16_ACT (every activation and activation gradient the step
 * keeps in memory is bfloat16; the image, parameters, parameter gradients, BN statistics, pooled features, logits, the
 * loss and every sum are fp32).  rn50_peek then returns bfloat16 tensors for what = 0, 1 and 4 (count is still in
 * elements); rn50_forward_eval is not built for such a context (RN50_EUNSUPPORTED). */
void rn50_destroy(rn50_ctx *ctx);
/* images: N x 224 x 224 x 3 fp32; labels: N int32; theta/grad/delta/m: rn50_param_count() floats;
 * grad16: rn50_param_count() halfs; loss_out: 1 float on the device.  After the call grad holds the
 * local fp32 gradient, grad16 its half-precision image, theta/delta/m the updated state. */
int rn50_step(rn50_ctx *ctx, const float *images, const int32_t *labels,
              float *theta, float *grad, float *delta, float *m, uint16_t *grad16,
              const rn50_opt_hparams *hp /* host */, float bn_eps, float *loss_out, void *stream);
/* Forward + loss + backward only (fills grad and loss_out); used by tests to grade gradients. */
int rn50_forward_backward(rn50_ctx *ctx, const float *images, const int32_t *labels, const float *theta,
                          float *grad, float bn_eps, float *loss_out, void *stream);
/* Device pointer (inside the arena) of a stored tensor of the last step, for inspection by tests:
 * what = 0 convolution output, 1 BN(+ReLU) output, 2 saved mean, 3 saved invstd of conv layer `layer`
 * (0..52 in parameter-table order); with `layer` ignored: 4 max-pool output, 5 max-pool arg index (uint8,
 * count in bytes), 6 pooled features, 7 logits, 8 gradient of the logits.  NULL for an invalid request.
 * A BN + ReLU output that the step left to its consumer (never written) is produced by one kernel enqueued on
 * `stream`, which should be the stream the step ran on: like every call this only enqueues, so the pointer's contents
 * are valid for work ordered after it on `stream` (or after the caller has synchronised). */
const float *rn50_peek(rn50_ctx *ctx, int layer, int what, size_t *count, void *stream);
/* The step's filter preparation alone: every convolution filter of theta flipped and transposed for the data gradients,
 * in the one launch rn50_step uses, into the context's arena (what the next step would overwrite anyway).  For timing. */
int rn50_filter_flip_all(rn50_ctx *ctx, const float *theta, void *stream);
/* The step's grouped filter-gradient launches alone (a context created with option wgrad_group > 0 in fp32: every
 * convolution behind the first layer), back to back on `stream`, on whatever the last step left in the context's buffers;
 * the gradients go to their places in grad.  Returns the number of grouped launches enqueued (0: the context launches its
 * filter gradients layer by layer), negative on error.  For timing. */
int rn50_wgrad_groups_run(rn50_ctx *ctx, float *grad, void *stream);
/* Validation-side forward (Section 2): conv -> BN with the statistics held by the context (those the last
 * rn50_step / rn50_forward_backward saved, or what rn50_set_bn_stats stored) -> ... -> FC.  images: N x 224 x 224 x 3,
 * theta: the flat parameter arena, logits_out: N x 1000 device floats (overwritten).  The activations stored by the
 * last training step are overwritten; the statistics are not. */
int rn50_forward_eval(rn50_ctx *ctx, const float *images, const float *theta, float *logits_out, void *stream);
/* Stores per-channel mean and invstd (device floats, one per output channel of convolution `layer`, table order) as
 * BN layer `layer`'s statistics, e.g. after bn_stats_average over the workers' sets. */
int rn50_set_bn_stats(rn50_ctx *ctx, int layer, const float *mean, const float *invstd, void *stream);

/* ------------------------------------------------------------------------------------------
 * Measurement aids (not part of the training step): kernels of known work, so that a benchmark can state what the
 * machine sustains next to the data-sheet peaks its roofline fractions are quoted against.
 * ------------------------------------------------------------------------------------------ */
/* Nothing but matrix instructions on register operands: 256 * wgs_per_cu workgroups of four wavefronts, each wavefront
 * issuing 32 * iters MFMAs (v_mfma_f32_32x32x2_f32 for RN50_DTYPE_F32, v_mfma_f32_32x32x16_bf16 for RN50_DTYPE_BF16) on four
 * independent accumulators.  *flop_out (host, may be NULL) receives the floating-point operations of the launch.
 * sink: 65536 * wgs_per_cu device floats, overwritten (keeps the loop alive).  wgs_per_cu in [1, 8].
 * ticks_or_null: two device int64, written by the first wavefront of the launch: [0] shader-clock cycles and [1] ticks of
 * the constant 100 MHz reference counter it spent in the loop; 100 * [0] / [1] is the shader clock in MHz the loop ran at
 * (the clock of a kernel of some tens of microseconds stays below the one a long kernel settles at). */
int rn50_probe_mfma(int dtype, int iters, int wgs_per_cu, float *sink, long long *ticks_or_null /* device */, double *flop_out /* host */,
                    void *stream);
/* dst[i] = src[i] for count floats (a multiple of 4), 16 bytes per lane: 4*count bytes read and 4*count written. */
int rn50_probe_copy(size_t count, const float *src, float *dst, void *stream);
/* `launches` kernels of `workgroups` x 256 threads that do nothing (sink may be NULL), enqueued back to back on the stream
 * from one call: the time per launch is the least a dependent kernel launch costs on the machine (no caller-side
 * overhead between them), which bounds what a chain of small kernels can reach.  launches in [1, 65536]. */
int rn50_probe_empty(int workgroups, int launches, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RN50_H */
