/*
 * nsk.h -- C ABI of libnsk: the residual-CNN training hot path on one MI355X (gfx950).
 *
 * The paper's system hands 2-D convolutions to a vendor library and runs batch-norm, ReLU and
 * the residual add as separate kernels (abstract; section "Experiments and Discussion";
 * ReLU fusion is named as future work in the conclusion).  This library is that device layer,
 * hand-written: implicit-GEMM convolution forward / backward-data / backward-weight on the
 * MFMA units, and fused batch-norm + ReLU + residual-add forward / backward, plus the 3x3
 * max pooling the large-image stem needs, and (last section) the small operations that close
 * a training step: network head, loss and optimizer updates.
 *
 * Calling convention, taken from what the paper says about its runtime:
 *  - Tensors are raw DEVICE pointers owned by the caller (section "Caching and Pooling": a
 *    pool hands out raw float pointers and nothing is malloc'd after the first iteration).
 *    No entry point allocates or frees device memory; scratch space is a caller-provided
 *    `workspace` whose size comes from a host-only query.
 *  - Every call is asynchronous on the caller's stream (section "Operation Overlapping");
 *    `stream` is a hipStream_t passed as void* (NULL = the default stream).  No call
 *    synchronises the device.
 *  - Gradients ACCUMULATE when asked to (section "Automatic Differentiation": the gradient
 *    reaching an operand is added to the one it already holds; section "Caching and
 *    Pooling": weight gradients are accumulated until the optimizer zeroes them):
 *    `accumulate` = 0 overwrites the whole output (elements no product reaches become 0),
 *    `accumulate` = 1 adds to what the buffer holds.
 *
 * Layouts and types.  Activations are NSK_NCHW (filters KCRS) or NSK_NHWC (filters KRSC),
 * dense and C-contiguous; NHWC is the fast path, NCHW is converted inside the call through
 * the workspace.  Element type NSK_F32 or NSK_BF16 (bfloat16, fp32 accumulation, round to
 * nearest even on store).  Filter gradients, batch-norm parameters, statistics and their
 * gradients are always float.  There is no convolution bias (batch-norm follows each one).
 *
 * Errors.  Every entry point returns an nsk_status_t and never throws or aborts.  Argument
 * validation happens on the host BEFORE any HIP call, so it behaves the same without a GPU.
 * All pointers must be 16-byte aligned.  Outputs must not overlap inputs.
 */
#ifndef NSK_H
#define NSK_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NSK_OK = 0,
    NSK_ERR_NULL = 1,        /* a required pointer is NULL */
    NSK_ERR_BAD_DESC = 2,    /* a descriptor field is out of range or the output would be empty */
    NSK_ERR_UNSUPPORTED = 3, /* valid request this build has no kernel for */
    NSK_ERR_WORKSPACE = 4,   /* workspace is NULL or smaller than the query says */
    NSK_ERR_ALIGNMENT = 5,   /* a pointer is not 16-byte aligned */
    NSK_ERR_HIP = 6          /* a HIP runtime call failed; see nsk_last_hip_error() */
} nsk_status_t;

enum { NSK_F32 = 0, NSK_BF16 = 1 };
enum { NSK_NCHW = 0, NSK_NHWC = 1 };
enum { NSK_PASS_FWD = 0, NSK_PASS_DGRAD = 1, NSK_PASS_WGRAD = 2 };
enum { NSK_BN_FWD = 0, NSK_BN_BWD = 1 };

/* Convolution y[N,K,P,Q] = x[N,C,H,W] (*) w[K,C,R,S]: cross-correlation, zero padding,
 * P = floor((H + 2*pad_h - dil_h*(R-1) - 1)/stride_h) + 1, Q likewise. */
typedef struct {
    int N, C, H, W;
    int K, R, S;
    int stride_h, stride_w;
    int pad_h, pad_w;
    int dil_h, dil_w;
    int dtype;  /* NSK_F32 | NSK_BF16: type of x, w, y, dy, dx */
    int layout; /* NSK_NCHW (w is KCRS) | NSK_NHWC (w is KRSC) */
} nsk_conv_desc_t;

/* Batch-norm over (n,h,w) per channel of a tensor [N,C,H,W], with optional ReLU. */
typedef struct {
    int N, C, H, W;
    int dtype;      /* of x, residual, out, dout, dx, dresidual */
    int layout;
    float eps;      /* added to the biased batch variance */
    float momentum; /* running = (1-momentum)*running + momentum*batch */
    int relu;       /* 0 | 1 */
} nsk_bn_desc_t;

/* Max pooling with window R x S over a tensor [N,C,H,W]; padding counts as -infinity. */
typedef struct {
    int N, C, H, W;
    int R, S;
    int stride_h, stride_w;
    int pad_h, pad_w;
    int dtype;
    int layout;
} nsk_pool_desc_t;

/* Library version as major*10000 + minor*100 + patch.  Host only. */
int nsk_version(void);

/* Static, never-NULL description of a status code.  Host only. */
const char *nsk_status_string(int status);

/* The hipError_t (as int) of the last HIP call that failed on this thread, 0 if none. */
int nsk_last_hip_error(void);

/* Test and A/B switches.  The library reads these environment variables once, at its first call (never on the
 * launch path); a process that changes them afterwards calls nsk_test_hooks_reload().  Host only.  Every switch
 * only moves a problem between kernels that compute the same result, so none changes any output beyond rounding
 * order (and none is needed in production):
 *   NSK_NO_BIG, NSK_NO_BIG_MULTI, NSK_NO_PW, NSK_NO_HALO, NSK_NO_FS, NSK_NO_HALO_WIDE, NSK_HALO_SINGLE, NSK_NO_STEM,
 *   NSK_NO_STEM_HALO, NSK_NO_TINY, NSK_NO_WIDE, NSK_NO_DEPTHWISE, NSK_DEPTHWISE_NO_ROWS, NSK_DEPTHWISE_NO_COLS,
 *   NSK_POOL_GENERAL, NSK_REDUCE4, NSK_WH_NO_SPLIT   (set = that special kernel or variant is not chosen);
 *   NSK_HALO_WIDE_ALWAYS, NSK_STATS_ALWAYS          (set = chosen also where it does not pay);
 *   NSK_BIG_MIN_TILES, NSK_PW_MIN_ROWS, NSK_WIDE_MIN_ROWS = n   (size threshold of a special kernel);
 *   NSK_IGEMM_TILE = 1..3                           (tile shape of the generic kernel). */
void nsk_test_hooks_reload(void);

/* Output extent of a convolution.  Host only.  NSK_ERR_BAD_DESC if the descriptor is invalid
 * (then *P and *Q are not written); an extent may legitimately come out as 0. */
int nsk_conv2d_out_dims(const nsk_conv_desc_t *desc, int *P, int *Q);

/* Bytes of workspace the given pass (NSK_PASS_*) needs for this descriptor; 0 for an invalid
 * descriptor or pass.  Host only, deterministic, never exceeds what the call will use. */
size_t nsk_conv2d_workspace_bytes(const nsk_conv_desc_t *desc, int pass);

/* Forward convolution.  x: [N,C,H,W] in desc->layout, w: [K,C,R,S] (KCRS or KRSC),
 * y: [N,K,P,Q] in desc->layout; all of desc->dtype, device memory.  y is overwritten. */
int nsk_conv2d_fwd(const nsk_conv_desc_t *desc, const void *x, const void *w, void *y,
                   void *workspace, size_t workspace_bytes, void *stream);

/* Forward convolution that also leaves per-channel partial sums of its output for a batch-norm that follows
 * (the statistics pass of that batch-norm then need not read y again).  stats: device memory for
 * 2 * rows * K floats with rows = nsk_conv2d_stats_rows(desc) (host only, 0 for an invalid descriptor):
 * stats[r*K + k] and stats[(rows + r)*K + k] receive the sum and the sum of squares of y[.., k], as stored, over
 * the r-th of `rows` disjoint shares of the output pixels; every entry is written.  Where the kernel that
 * computes y has no such epilogue the sums come from a separate pass over y; the result is the same. */
int nsk_conv2d_stats_rows(const nsk_conv_desc_t *desc);
int nsk_conv2d_fwd_stats(const nsk_conv_desc_t *desc, const void *x, const void *w, void *y, float *stats,
                         void *workspace, size_t workspace_bytes, void *stream);

/* Backward-data: dx = adjoint of the forward map with respect to x applied to dy.
 * dy: [N,K,P,Q], w as in forward, dx: [N,C,H,W].  accumulate: see the header comment;
 * with accumulate = 0 input positions that no filter tap reaches (strided cases) are
 * written as 0. */
int nsk_conv2d_dgrad(const nsk_conv_desc_t *desc, const void *dy, const void *w, void *dx,
                     int accumulate, void *workspace, size_t workspace_bytes, void *stream);

/* Backward-weight: dw[K,C,R,S] (always float, laid out like w for desc->layout) =
 * sum over (n,p,q) of dy * shifted x.  The reduction is split over (n,p,q) into float
 * partials in the workspace and combined in a fixed order, so results are bitwise
 * reproducible from run to run. */
int nsk_conv2d_wgrad(const nsk_conv_desc_t *desc, const void *x, const void *dy, float *dw,
                     int accumulate, void *workspace, size_t workspace_bytes, void *stream);

/* Grouped convolution (not used by the paper's networks; the residual-network family that the paper's recipe
 * belongs to has grouped and depthwise members, and the definition is the textbook one): the C input channels and
 * the K output channels are split into `groups` equal runs, output run g sees input run g only, and the filter is
 * w[K][C/groups][R][S] (KCRS) or w[K][R][S][C/groups] (KRSC); dw has the same shape.  desc describes the whole
 * tensors (C and K are the totals).  groups must divide C and K (else NSK_ERR_BAD_DESC); groups = 1 is exactly the
 * plain call.  Everything else (layouts, types, accumulate, workspace, stream, errors) is as in the plain calls; the
 * workspace size comes from nsk_conv2d_grouped_workspace_bytes (host only, 0 for an invalid request). */
size_t nsk_conv2d_grouped_workspace_bytes(const nsk_conv_desc_t *desc, int groups, int pass);
int nsk_conv2d_grouped_fwd(const nsk_conv_desc_t *desc, int groups, const void *x, const void *w, void *y,
                           void *workspace, size_t workspace_bytes, void *stream);
int nsk_conv2d_grouped_dgrad(const nsk_conv_desc_t *desc, int groups, const void *dy, const void *w, void *dx,
                             int accumulate, void *workspace, size_t workspace_bytes, void *stream);
int nsk_conv2d_grouped_wgrad(const nsk_conv_desc_t *desc, int groups, const void *x, const void *dy, float *dw,
                             int accumulate, void *workspace, size_t workspace_bytes, void *stream);

/* Workspace bytes for the batch-norm pass (NSK_BN_FWD | NSK_BN_BWD); 0 if invalid. */
size_t nsk_bn_workspace_bytes(const nsk_bn_desc_t *desc, int pass);

/* out = relu?( gamma*(x-mean)*invstd + beta [+ residual] ), with mean and the biased variance
 * taken over (n,h,w) of this batch and invstd = 1/sqrt(var + eps).
 * residual may be NULL.  save_mean / save_invstd ([C] float) receive the batch statistics
 * for the backward pass.  running_mean / running_var ([C] float, both or neither NULL) are
 * updated in place with desc->momentum, the variance in its unbiased form. */
int nsk_bn_relu_add_fwd(const nsk_bn_desc_t *desc, const void *x, const void *residual,
                        const float *gamma, const float *beta, void *out, float *save_mean,
                        float *save_invstd, float *running_mean, float *running_var,
                        void *workspace, size_t workspace_bytes, void *stream);

/* nsk_bn_relu_add_fwd for callers that cannot allocate device memory or carry a workspace around: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, arithmetic and results as
 * nsk_bn_relu_add_fwd, without the workspace: the per-block partial sums go to a device array that is part of the
 * library image (nsk_static_scratch_bytes() = 8 MiB, held by every GPU the library runs on until the process ends).
 * No hipMalloc, hipFree or other allocating call is made.  Descriptors whose nsk_bn_workspace_bytes(desc, NSK_BN_FWD)
 * exceeds that size are rejected with NSK_ERR_WORKSPACE before any HIP call.  All calls on one GPU share the
 * array: calls that overlap in time on one GPU (two streams, two threads) race and must not be issued; calls on
 * one stream are ordered and safe.  The array's address is looked up once per device at the first call on that
 * device (that first call must not be under stream capture). */
size_t nsk_static_scratch_bytes(void);
int nsk_bn_relu_add_fwd_static(const nsk_bn_desc_t *desc, const void *x, const void *residual,
                               const float *gamma, const float *beta, void *out, float *save_mean,
                               float *save_invstd, float *running_mean, float *running_var, void *stream);

/* Backward of nsk_bn_relu_add_fwd.  x, out: the forward input and its stored result;
 * dout: gradient of out.  With dz = relu ? dout*[out>0] : dout and xhat = (x-mean)*invstd:
 *   dbeta = sum dz, dgamma = sum dz*xhat  (overwritten, [C] float),
 *   dx = gamma*invstd*(dz - dbeta/M - xhat*dgamma/M),  dresidual = dz (NULL to skip).
 * dx and dresidual are overwritten; dresidual may later be the target of an accumulating
 * nsk_conv2d_dgrad. */
int nsk_bn_relu_add_bwd(const nsk_bn_desc_t *desc, const void *x, const void *out,
                        const void *dout, const float *gamma, const float *save_mean,
                        const float *save_invstd, void *dx, void *dresidual, float *dgamma,
                        float *dbeta, void *workspace, size_t workspace_bytes, void *stream);

/* The same two calls with the ReLU mask handed from forward to backward, so that the backward pass does not
 * read `out` (one tensor read less in each of its two kernels).  Only for NSK_NHWC descriptors with relu = 1
 * whose channel count lets the kernels use 16-byte vectors (C a multiple of 8 for bf16, 4 for f32, and a
 * divisor of 256 vectors: nsk_bn_mask_bytes returns 0 otherwise and the plain calls must be used).
 * relu_mask: nsk_bn_mask_bytes(desc) bytes of device memory, one byte per 16-byte vector of `out` in storage
 * order, bit e set iff element e of that vector is > 0 as stored.  The forward call writes it, the backward
 * call reads it; the backward call takes no `out`. */
size_t nsk_bn_mask_bytes(const nsk_bn_desc_t *desc);
int nsk_bn_relu_add_fwd_mask(const nsk_bn_desc_t *desc, const void *x, const void *residual,
                             const float *gamma, const float *beta, void *out, unsigned char *relu_mask,
                             float *save_mean, float *save_invstd, float *running_mean,
                             float *running_var, void *workspace, size_t workspace_bytes, void *stream);
/* nsk_bn_relu_add_fwd with the batch statistics taken from partial sums of x and x*x (layout as written by
 * nsk_conv2d_fwd_stats: [2][stats_rows][C] floats) instead of a reduction pass over x.  relu_mask: NULL, or as in
 * nsk_bn_relu_add_fwd_mask.  The variance is formed as E[x*x] - E[x]^2 in double precision from float partial sums
 * that are not shifted: a float partial sum is good to about 3e-8, which is 3e-8 * (mean/sigma)^2 of the variance, so
 * invstd is off by 1e-4 where |mean| is about 80 standard deviations (measured on a 1x1 layer fed an all-positive
 * input; the zero padding of a 3x3 layer keeps its outputs below 10).  nsk_bn_relu_add_fwd, which subtracts a
 * per-channel shift first, has no such limit. */
int nsk_bn_relu_add_fwd_stats(const nsk_bn_desc_t *desc, const void *x, const void *residual,
                              const float *gamma, const float *beta, void *out, unsigned char *relu_mask,
                              float *save_mean, float *save_invstd, float *running_mean,
                              float *running_var, const float *stats, int stats_rows, void *workspace,
                              size_t workspace_bytes, void *stream);
int nsk_bn_relu_add_bwd_mask(const nsk_bn_desc_t *desc, const void *x, const unsigned char *relu_mask,
                             const void *dout, const float *gamma, const float *save_mean,
                             const float *save_invstd, void *dx, void *dresidual, float *dgamma,
                             float *dbeta, void *workspace, size_t workspace_bytes, void *stream);

/* ---- Batch-norm + ReLU applied by the consumers of a convolution's output (the conclusion of the paper names ReLU-fused
 * operations as future work).  In conv -> batch-norm -> ReLU -> conv the normalised activation a = relu(scale*y + shift)
 * need not be stored: the second convolution (and, in the backward pass, its backward-weight call) applies it to the raw
 * y while loading its operand, and the backward pass of the batch-norm takes the ReLU mask from y as well.  One write
 * and one read of the activation disappear.  NHWC only, relu = 1, no residual on the fused batch-norm (NSK_ERR_UNSUPPORTED
 * otherwise, and for channel counts the 16-byte vector kernels do not take: see nsk_bn_mask_bytes).
 *
 * nsk_bn_fwd_coeffs: the batch statistics from partial sums of y and y*y (as nsk_bn_relu_add_fwd_stats takes them) and
 *   coeffs[c] = scale = gamma*invstd, coeffs[C + c] = shift = beta - mean*scale (2*C floats, device memory); no pass
 *   over y.  Workspace: nsk_bn_workspace_bytes(desc, NSK_BN_FWD).
 * nsk_conv2d_fwd_act / nsk_conv2d_wgrad_act: nsk_conv2d_fwd[_stats] / nsk_conv2d_wgrad with x replaced by
 *   relu(coeffs[c]*x + coeffs[C + c]) rounded to desc->dtype, the value the apply pass would have stored (zero padding
 *   stays zero); coeffs belong to the C input channels of desc.  stats may be NULL.  Kernels with a fused operand load
 *   (the fp32 3x3 64 -> 64 layers on 32-pixel-wide images) read x once and store nothing extra; every other layer is
 *   served by applying the activation into the workspace first (same results, no saving).  Workspace:
 *   nsk_conv2d_act_workspace_bytes(desc, NSK_PASS_FWD | NSK_PASS_WGRAD) (host only; may be 0 for a fused kernel);
 *   nsk_conv2d_act_supported(desc) says whether the two calls take the layer at all.
 * nsk_bn_relu_bwd_act: nsk_bn_relu_add_bwd for that batch-norm without `out` and without a residual: the ReLU mask is
 *   [coeffs[c]*x + coeffs[C + c] > 0], the expression the consumers used.  Workspace: nsk_bn_workspace_bytes(desc,
 *   NSK_BN_BWD). */
int nsk_bn_fwd_coeffs(const nsk_bn_desc_t *desc, const float *gamma, const float *beta, const float *stats,
                      int stats_rows, float *save_mean, float *save_invstd, float *running_mean,
                      float *running_var, float *coeffs, void *workspace, size_t workspace_bytes, void *stream);
int nsk_conv2d_act_supported(const nsk_conv_desc_t *desc);   /* 1 / 0, host only */
size_t nsk_conv2d_act_workspace_bytes(const nsk_conv_desc_t *desc, int pass);
int nsk_conv2d_fwd_act(const nsk_conv_desc_t *desc, const void *x, const float *coeffs, const void *w, void *y,
                       float *stats, void *workspace, size_t workspace_bytes, void *stream);
int nsk_conv2d_wgrad_act(const nsk_conv_desc_t *desc, const void *x, const float *coeffs, const void *dy, float *dw,
                         int accumulate, void *workspace, size_t workspace_bytes, void *stream);
int nsk_bn_relu_bwd_act(const nsk_bn_desc_t *desc, const void *x, const float *coeffs, const void *dout,
                        const float *gamma, const float *save_mean, const float *save_invstd, void *dx,
                        float *dgamma, float *dbeta, void *workspace, size_t workspace_bytes, void *stream);

/* Output extent of a pooling descriptor.  Host only. */
int nsk_maxpool2d_out_dims(const nsk_pool_desc_t *desc, int *P, int *Q);

/* y[N,C,P,Q] = window maximum; idx (signed char, same shape and layout as y) = r*S+s of the
 * FIRST maximum in row-major window order, -1 for a window with no input element (y = -inf).
 * Needs R*S <= 127.  No workspace. */
int nsk_maxpool2d_fwd(const nsk_pool_desc_t *desc, const void *x, void *y, signed char *idx,
                      void *stream);

/* dx[N,C,H,W] = sum of dy over the windows whose idx names that element (dx overwritten). */
int nsk_maxpool2d_bwd(const nsk_pool_desc_t *desc, const void *dy, const signed char *idx,
                      void *dx, void *stream);

/* ---------------------------------------------------------------------------------------------------------------
 * The tail that closes a training step behind the residual blocks: the head of the ResNet recipe the paper
 * trains (global average pool, fully connected layer), the loss node that must end every step, and the optimizer
 * updates (sections "Automatic Differentiation", "Caching and Pooling", "Experiments and Discussion").  The
 * paper gives no formulas for them; the textbook definitions below are used.
 * --------------------------------------------------------------------------------------------------------------- */

/* Global average pool: y[n][c] = mean over (h, w) of x[n][c][h][w].  x: [N,C,H,W] in `layout`, y: [N,C], both of
 * `dtype`; sums in float.  No workspace.  NSK_ERR_BAD_DESC for non-positive extents. */
int nsk_global_avgpool_fwd(int dtype, int layout, int N, int C, int H, int W, const void *x, void *y,
                           void *stream);
/* Its adjoint: dx[n][c][h][w] (+)= dy[n][c] / (H*W); accumulate as in the header comment. */
int nsk_global_avgpool_bwd(int dtype, int layout, int N, int C, int H, int W, const void *dy, void *dx,
                           int accumulate, void *stream);

/* Fully connected layer, the `@` operator of section "Automatic Differentiation": y = x @ w multiplies by the
 * TRANSPOSED weight, y[n][k] = sum_c x[n][c] * w[k][c] (+ bias[k]).  x: [N,C], w: [K,C], y: [N,K] of `dtype`,
 * row-major; bias, dw, db are float.  The three calls run on the convolution kernels (a 1x1 filter on a 1x1
 * image); `workspace` must hold nsk_linear_workspace_bytes(desc, NSK_PASS_*) bytes. */
typedef struct {
    int N, C, K;
    int dtype;
} nsk_linear_desc_t;
size_t nsk_linear_workspace_bytes(const nsk_linear_desc_t *desc, int pass);
/* bias may be NULL. */
int nsk_linear_fwd(const nsk_linear_desc_t *desc, const void *x, const void *w, const float *bias, void *y,
                   void *workspace, size_t workspace_bytes, void *stream);
/* dx[n][c] (+)= sum_k dy[n][k] * w[k][c]. */
int nsk_linear_dgrad(const nsk_linear_desc_t *desc, const void *dy, const void *w, void *dx, int accumulate,
                     void *workspace, size_t workspace_bytes, void *stream);
/* dw[k][c] (+)= sum_n dy[n][k] * x[n][c];  db[k] (+)= sum_n dy[n][k] (db may be NULL).  Fixed summation order. */
int nsk_linear_wgrad(const nsk_linear_desc_t *desc, const void *x, const void *dy, float *dw, float *db,
                     int accumulate, void *workspace, size_t workspace_bytes, void *stream);

/* dst[c][r] = src[r][c] for a row-major [rows][cols] matrix of `dtype` (dst must not overlap src).  A caller that
 * multiplies few rows by the same weight many times (a recurrent layer) keeps a transposed copy: the product with
 * W^T read row by row is then nsk_linear_dgrad on the copy, whose memory accesses are contiguous. */
int nsk_transpose2d(int dtype, int rows, int cols, const void *src, void *dst, void *stream);

/* Softmax cross-entropy, the loss node: per_sample[n] = log sum_k exp(z[n][k]) - z[n][label_n] (computed with
 * the row maximum subtracted), loss[0] = mean over n, summed in a fixed order.  logits: [N,K] of `dtype`;
 * labels: [N] int, each in [0,K) (a label outside that range gives NaN for its sample and for the loss);
 * per_sample: [N] float, loss: [1] float, all device memory. */
int nsk_softmax_xent_fwd(int dtype, int N, int K, const void *logits, const int *labels, float *per_sample,
                         float *loss, void *stream);
/* dlogits[n][k] = dloss/N * (softmax(z[n])[k] - [k == label_n]), of `dtype`, overwritten. */
int nsk_softmax_xent_bwd(int dtype, int N, int K, const void *logits, const int *labels, float dloss,
                         void *dlogits, void *stream);

/* Optimizer updates over one parameter tensor of n floats (master weights, gradient and state are float).  Each
 * call is asynchronous on its stream, so parameter groups can be updated on streams of their own (section
 * "Operation Overlapping").  The gradient buffer is overwritten with zeros (section "Caching and Pooling").
 * w_lp: NULL, or n bf16 elements that receive the updated weights rounded to bf16 (the copy the bf16 kernels
 * read).  grad_scale: NULL, or a device float (4-byte aligned, like the other single-float arguments below) that
 * multiplies every gradient first (see nsk_clip_scale).
 *
 * SGD with momentum (the ResNet recipe):  g' = scale*g + weight_decay*w;  v <- momentum*v + g';  w <- w - lr*v. */
int nsk_sgd_momentum_step(size_t n, float *w, float *grad, float *velocity, void *w_lp, float lr,
                          float momentum, float weight_decay, const float *grad_scale, void *stream);
/* AdamW (the recurrent experiment of section "Experiments and Discussion"), step counted from 1:
 * w <- w*(1 - lr*weight_decay);  m <- beta1*m + (1-beta1)*g;  v <- beta2*v + (1-beta2)*g*g;
 * w <- w - lr * (m/(1-beta1^step)) / (sqrt(v/(1-beta2^step)) + eps). */
int nsk_adamw_step(size_t n, float *w, float *grad, float *m, float *v, void *w_lp, int step, float lr,
                   float beta1, float beta2, float eps, float weight_decay, const float *grad_scale,
                   void *stream);
/* The same updates for `count` parameter tensors in one launch per 32 tensors (a network has many small ones, and a
 * launch per tensor costs more than the update).  params: HOST array of `count` records; state1 is the velocity
 * (SGD) or m (AdamW), state2 is v (AdamW; ignored by SGD); w_lp NULL or the bf16 copy; each tensor has its own
 * weight decay.  All records are validated before anything is launched. */
typedef struct {
    float *w, *grad, *state1, *state2;
    void *w_lp;
    size_t n;
    float weight_decay;
} nsk_param_t;
int nsk_sgd_momentum_step_multi(int count, const nsk_param_t *params, float lr, float momentum,
                                const float *grad_scale, void *stream);
int nsk_adamw_step_multi(int count, const nsk_param_t *params, int step, float lr, float beta1, float beta2,
                         float eps, const float *grad_scale, void *stream);
/* Gradient clip by global norm (the "gradient clip of 5" of the same experiment), in two steps that never
 * synchronise: nsk_sumsq_accumulate adds the sum of squares of g[0..n) to the device float *sumsq (zero it before
 * the first tensor; `partials`: NSK_SUMSQ_PARTIALS floats of device scratch; fixed summation order), then
 * nsk_clip_scale writes *scale = min(1, max_norm / (sqrt(*sumsq) + 1e-6)) for the optimizer calls to read. */
#define NSK_SUMSQ_PARTIALS 256
int nsk_sumsq_accumulate(size_t n, const float *g, float *partials, float *sumsq, void *stream);
int nsk_clip_scale(const float *sumsq, float max_norm, float *scale, void *stream);

/* ---------------------------------------------------------------------------------------------------------------
 * The recurrent workload (section "Experiments and Discussion": an embedding over the vocabulary, one GRU layer, an
 * output layer, cross entropy, AdamW with a gradient clip).  Its matrix products are the `@` operator
 * (nsk_linear_*): gi = x @ W_ih for all time steps in one call, gh = h @ W_hh once per step, and their gradients.
 * What is declared here is the rest: the embedding lookup with its gradient, and the elementwise part of one GRU step
 * in one kernel per direction (the paper ran it as separate unfused operations and names that as the cause of its
 * slowdown on this experiment).  Gate order (r, z, n); weights W_ih [3H][E], W_hh [3H][H]; biases float [3H]:
 *   r = sigmoid(gi_r + b_ir + gh_r + b_hr),  z = sigmoid(gi_z + b_iz + gh_z + b_hz),
 *   q = gh_n + b_hn,  n = tanh(gi_n + b_in + r*q),  h_new = (1 - z)*n + z*h_prev.
 * --------------------------------------------------------------------------------------------------------------- */

/* out[i][0..E) = table[tokens[i]][0..E) for i < n.  tokens: int [n], each in [0,V) (a token outside that range gives
 * a row of NaN); table [V,E] and out [n,E] of `dtype`. */
int nsk_embedding_fwd(int dtype, int n, int E, int V, const int *tokens, const void *table, void *out,
                      void *stream);
/* dtable[v][e] (+)= sum over the positions i with tokens[i] == v of dout[i][e]; dtable is float [V,E] and with
 * accumulate = 0 it is overwritten as a whole.  No atomics: every element is summed in position order (bitwise
 * reproducible).  Tokens outside [0,V) are ignored. */
int nsk_embedding_bwd(int dtype, int n, int E, int V, const int *tokens, const void *dout, float *dtable,
                      int accumulate, void *stream);
/* Elementwise part of a GRU step.  gi, gh: [N,3H]; h_prev, h_new: [N,H]; saved: [N,4H] receives (r, z, n, q) for
 * the backward call; all of `dtype`, math in float. */
int nsk_gru_gates_fwd(int dtype, int N, int H, const void *gi, const void *gh, const float *b_ih,
                      const float *b_hh, const void *h_prev, void *h_new, void *saved, void *stream);
/* Its gradient.  dh = dh_a + dh_b + dh_c is the gradient of h_new (dh_b, dh_c may be NULL: the contributions of the
 * following step arrive in separate buffers).  Writes dgi, dgh [N,3H] (the gradients of the two products; their
 * column sums are the bias gradients) and dh_direct [N,H] = dh * z, the part of the gradient of h_prev that does not
 * pass through gh; the rest is nsk_linear_dgrad(dgh, W_hh). */
int nsk_gru_gates_bwd(int dtype, int N, int H, const void *saved, const void *h_prev, const void *dh_a,
                      const void *dh_b, const void *dh_c, void *dgi, void *dgh, void *dh_direct, void *stream);

/* A whole GRU step in one launch per direction, for the few-row case of the same experiment (batch 50): the
 * recurrent product and the gate arithmetic fused, so that gh is never stored and a sequence of T steps is 2T
 * dependent launches instead of 4T.  Same gate convention, same `saved` layout as the two calls above.
 * nsk_gru_step_supported(N, H) says (1 / 0, host only) whether the sizes are taken: at most 256 rows (the case these
 * calls are for) and H % 4 == 0; otherwise the calls return NSK_ERR_UNSUPPORTED and the caller uses nsk_linear_* with
 * nsk_gru_gates_*.
 * forward: gi [N,3H] (= x_t @ W_ih, without biases), w_hh [3H,H], h_prev -> h_new [N,H], saved [N,4H].
 * backward: the gradient of h_new is dh_a + dh_direct_next + dgh_next @ W_hh (each may be NULL, not all three):
 * dh_a arrives from outside the recurrence, dh_direct_next and dgh_next [N,3H] are what this same call wrote for the
 * step after; w_hh_t [H,3H] is the TRANSPOSED recurrent weight (nsk_transpose2d), so that the column of W_hh a hidden
 * unit needs is contiguous.  Writes dgi, dgh [N,3H] and dh_direct [N,H] = dh * z as nsk_gru_gates_bwd does. */
int nsk_gru_step_supported(int N, int H);
int nsk_gru_step_fwd(int dtype, int N, int H, const void *gi, const void *w_hh, const float *b_ih, const float *b_hh,
                     const void *h_prev, void *h_new, void *saved, void *stream);
int nsk_gru_step_bwd(int dtype, int N, int H, const void *saved, const void *h_prev, const void *dh_a,
                     const void *dh_direct_next, const void *dgh_next, const void *w_hh_t, void *dgi, void *dgh,
                     void *dh_direct, void *stream);

/* ---------------------------------------------------------------------------------------------------------------
 * Device memory pool and cache (section "Caching and Pooling"): what hands out the raw pointers every entry point
 * above takes, for callers that have no allocator of their own.  Host code; no entry point above uses it.
 *
 * Pool: a dictionary from a byte size (rounded up to 256) to a list of free pointers of exactly that size.
 * nsk_pool_get pops one, or allocates when the list is empty; nsk_pool_put appends the pointer to its size's list
 * instead of freeing it.  A step that requests the same sizes every iteration allocates nothing from the second
 * iteration on.  Cache: nsk_pool_cached maps a name to a buffer that lives until the pool is destroyed (the
 * paper keeps parameter gradients this way); *created (may be NULL) says whether this call allocated it, so the
 * caller can zero it once.  kind: NSK_POOL_DEVICE (hipMalloc on the current device) or NSK_POOL_HOST (plain host
 * memory, 256-byte aligned).  Not thread-safe.  nsk_pool_put returns NSK_ERR_BAD_DESC for a pointer that is not
 * out on loan from this pool (foreign, or returned twice); nsk_pool_cached for a known name with another size.
 * nsk_pool_destroy frees everything the pool ever allocated, on loan or not.  Contents of a buffer are whatever its
 * last user left.
 * --------------------------------------------------------------------------------------------------------------- */
enum { NSK_POOL_DEVICE = 0, NSK_POOL_HOST = 1 };
typedef struct nsk_pool nsk_pool_t;
int nsk_pool_create(int kind, nsk_pool_t **pool);
int nsk_pool_get(nsk_pool_t *pool, size_t bytes, void **ptr);
int nsk_pool_put(nsk_pool_t *pool, void *ptr);
int nsk_pool_cached(nsk_pool_t *pool, const char *name, size_t bytes, void **ptr, int *created);
/* Any output pointer may be NULL.  allocations = calls that reached the backing allocator; hits = requests served
 * from a free list. */
int nsk_pool_stats(const nsk_pool_t *pool, size_t *bytes_allocated, size_t *allocations, size_t *requests,
                   size_t *hits);
int nsk_pool_destroy(nsk_pool_t *pool);

#ifdef __cplusplus
}
#endif
#endif /* NSK_H */
