/*
 * owt.h -- C ABI of libowt: one worker's compute hot path of the training
 * scheme of "One weird trick for parallelizing convolutional neural networks"
 * on one AMD MI355X (gfx950).
 *
 * In that scheme (Section 4) every worker runs all convolutional layers
 * data-parallel on its own batch (about 128 examples; forward steps 1-2,
 * backward step 2) and owns 1/K of the neurons of every fully-connected
 * layer (forward step 3, backward step 1).  This library is that per-worker
 * computation: convolution forward / backward-data / backward-filter with a
 * fused bias+ReLU, the worker's fully-connected column shard forward and
 * backward, and the max-pooling that sits between the convolution layers of
 * the Section 5 model.  Exchanges between workers are not part of it.
 *
 * Conventions for every call
 *  - All data pointers are DEVICE pointers, 16-byte aligned, dense row-major:
 *    activations NHWC [n][h][w][c], filters KRSC [k][r][s][c], fully-connected
 *    weights [o][i].  The caller owns every buffer; the library never
 *    allocates, frees or keeps a pointer.  Buffers must not alias unless
 *    stated otherwise.
 *  - Work is enqueued on `hip_stream` (a hipStream_t cast to void*, NULL = the
 *    default stream) and the call returns without waiting for it.
 *  - `ws` is caller-provided device scratch of at least the number of bytes the
 *    matching *_workspace_bytes query returns (may be NULL when that is 0).
 *    Its contents are undefined after the call.
 *  - Return value OWT_OK, or an error code; on error nothing was launched and
 *    no output was touched.  owt_last_error() gives a message for the calling
 *    thread's most recent error.
 *  - Results are deterministic run to run (no floating-point atomics).
 *  - dtype names the STORAGE type of x, w, y, dy, dx.  Products are
 *    accumulated in fp32; bias, dw and dbias are always fp32.  bf16 results are
 *    rounded to nearest-even once, when stored.
 *  - Output size P = floor((H + 2*pad_h - R)/stride_h) + 1, Q likewise.
 */
#ifndef OWT_H
#define OWT_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OWT_OK = 0,
    OWT_EINVAL = 1,       /* bad descriptor, null or misaligned pointer                  */
    OWT_EUNSUPPORTED = 2, /* valid request this build has no kernel for                  */
    OWT_EWORKSPACE = 3,   /* ws_bytes smaller than the workspace query                   */
    OWT_ELAUNCH = 4       /* the HIP runtime refused a launch (message has the HIP text) */
} owt_status;

typedef enum { OWT_F32 = 0, OWT_BF16 = 1 } owt_dtype;

enum { OWT_BIAS = 1u, OWT_RELU = 2u };

enum { OWT_PASS_FWD = 0, OWT_PASS_BWD_DATA = 1, OWT_PASS_BWD_FILTER = 2 };

/* One convolution layer on a batch of N images (Section 4, forward step 2). */
typedef struct {
    int N, C, H, W;         /* input batch, channels, height, width          */
    int K, R, S;            /* filters, filter height, filter width          */
    int stride_h, stride_w; /* >= 1                                          */
    int pad_h, pad_w;       /* zero padding on each side, 0 <= pad < R (S)   */
    owt_dtype dtype;
    unsigned flags;         /* OWT_BIAS | OWT_RELU                           */
} owt_conv_desc;

/* One fully-connected layer split by output column over `workers` workers
 * (Section 4, forward step 3: each worker holds 1/K of the neurons; the
 * Section 5.1 footnote sizes the K = 8 shard at 4096 x 512).  This worker owns
 * O_local = O_total / workers columns; `w` is its [O_local][I] block. */
typedef struct {
    int N;       /* batch the shard runs on (128 in schemes (b) and (c)) */
    int I;       /* inputs                                               */
    int O_total; /* outputs of the whole layer, divisible by workers     */
    int workers; /* K                                                    */
    int rank;    /* 0 <= rank < workers (checked, otherwise unused)      */
    owt_dtype dtype;
    unsigned flags; /* OWT_BIAS | OWT_RELU                               */
} owt_fc_desc;

/* Scratch bytes a pass needs (pass = OWT_PASS_*).  (size_t)-1 on a bad descriptor. */
size_t owt_conv_workspace_bytes(const owt_conv_desc *d, int pass);
size_t owt_fc_workspace_bytes(const owt_fc_desc *d, int pass);

/* Diagnostics: writes a one-line description of the kernel variant, tile shape,
 * split-K factor and grid the planner picks for this pass into buf (NUL
 * terminated, truncated to buf_bytes).  Returns the untruncated length, or -1
 * on a bad argument.  Host only. */
int owt_conv_plan_describe(const owt_conv_desc *d, int pass, char *buf, size_t buf_bytes);

/* Convolution forward (Section 4, forward step 2):
 *   y[n,p,q,k] = act(bias[k] + sum_{r,s,c} x[n, p*stride_h-pad_h+r, q*stride_w-pad_w+s, c] * w[k,r,s,c])
 * taps outside the image count as 0; act = max(0,.) with OWT_RELU, identity
 * otherwise; bias is read only with OWT_BIAS (else may be NULL).
 * x [N,H,W,C], w [K,R,S,C], bias [K] fp32, y [N,P,Q,K] (written). */
owt_status owt_conv_fwd(const owt_conv_desc *d, const void *x, const void *w, const float *bias,
                        void *y, void *ws, size_t ws_bytes, void *hip_stream);

/* Convolution backward w.r.t. the input (Section 4, backward step 2):
 *   dz = dy * [y > 0] if the descriptor has OWT_RELU (y = the forward output, required then), else dy
 *   dx[n,h,w,c] = sum of dz[n,p,q,k] * w[k,r,s,c] over all (p,q,k,r,s) with
 *                 p*stride_h-pad_h+r == h and q*stride_w-pad_w+s == w
 * dy, y [N,P,Q,K]; w [K,R,S,C]; dx [N,H,W,C] (written, every element). */
owt_status owt_conv_bwd_data(const owt_conv_desc *d, const void *dy, const void *y_or_null,
                             const void *w, void *dx, void *ws, size_t ws_bytes, void *hip_stream);

/* owt_conv_bwd_data with the backward pass of the PRECEDING ReLU fused into its
 * store: x is this layer's input [N,H,W,C]; where x <= 0 the stored dx is 0.
 * Use it when x is itself the output of a bias+ReLU layer: the result is that
 * layer's dz, and its own backward calls can then run without OWT_RELU.  Saves
 * every later kernel a second read of the mask source.  Same arithmetic as
 * Section 4, backward step 2, only the place where the mask is applied moves. */
owt_status owt_conv_bwd_data_relu_in(const owt_conv_desc *d, const void *dy, const void *y_or_null,
                                     const void *w, const void *x, void *dx, void *ws, size_t ws_bytes,
                                     void *hip_stream);

/* Convolution backward w.r.t. filters and bias (Section 4, backward step 2):
 *   dw[k,r,s,c] = alpha * sum_{n,p,q} dz[n,p,q,k] * x[n, p*stride_h-pad_h+r, q*stride_w-pad_w+s, c] + beta * dw
 *   dbias[k]    = alpha * sum_{n,p,q} dz[n,p,q,k] + beta * dbias          (skipped when dbias_or_null is NULL)
 * dz as in owt_conv_bwd_data.  beta == 0 overwrites without reading the old
 * contents.  alpha = 1/N gives the batch-mean gradient the update rule of
 * Section 5 uses; beta = 1 accumulates over several calls (Section 4.2).
 * dw [K,R,S,C] and dbias [K] are fp32 whatever the dtype. */
owt_status owt_conv_bwd_filter(const owt_conv_desc *d, const void *x, const void *dy,
                               const void *y_or_null, float alpha, float beta, float *dw,
                               float *dbias_or_null, void *ws, size_t ws_bytes, void *hip_stream);

/* owt_conv_bwd_filter for callers that CANNOT ALLOCATE device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * result as owt_conv_bwd_filter minus ws / ws_bytes: the partial sums of the split reduction go to
 * a static array of device memory inside the library (owt_static_scratch_bytes() = 64 MiB, one copy
 * per GPU, held until the process ends).  The call allocates and frees nothing.  It runs the variant
 * owt_conv_bwd_filter would run when that variant's partial sums fit the array, otherwise the
 * cheapest variant that does (results then differ in summation order only); if none fits it returns
 * OWT_EWORKSPACE and launches nothing.  Nothing in the array has to start at zero (every partial sum
 * that is read was written by the same call).  All calls on one GPU share the array: calls that
 * overlap in time on one GPU (different streams or threads) race and give wrong results; calls on
 * one stream are ordered and safe. */
owt_status owt_conv_bwd_filter_static(const owt_conv_desc *d, const void *x, const void *dy, const void *y_or_null,
                                      float alpha, float beta, float *dw, float *dbias_or_null, void *hip_stream);
size_t owt_static_scratch_bytes(void);

/* Optional tuning.  Runs every kernel variant the planner knows for this pass
 * on the caller's buffers (three timed repetitions each, HIP events on
 * hip_stream), and remembers the fastest: later owt_conv_* calls in this
 * process with an identical descriptor use it.  Blocks until the timing is
 * done.  Buffers are those of the pass itself (others may be NULL):
 *   OWT_PASS_FWD        reads x, w, bias              writes y
 *   OWT_PASS_BWD_DATA   reads dy, y (mask), w         writes dx
 *   OWT_PASS_BWD_FILTER reads x, dy, y (mask)         writes dw, dbias (alpha 1, beta 0)
 * ws must hold owt_conv_workspace_bytes(d, pass).  Without this call a cost
 * model picks the variant; results are identical up to summation order.
 * For callers that can afford a few milliseconds of set-up per layer. */
owt_status owt_conv_autotune(const owt_conv_desc *d, int pass, const void *x, const void *w, const float *bias,
                             void *y, const void *dy, void *dx, float *dw, float *dbias_or_null, void *ws,
                             size_t ws_bytes, void *hip_stream);

/* Fully-connected column shard forward (Section 4, forward step 3):
 *   y[n,o] = act(bias[o] + sum_i x[n,i] * w[o,i]),  o over this worker's O_local columns.
 * x [N,I], w [O_local,I], bias [O_local] fp32, y [N,O_local] (written). */
owt_status owt_fc_shard_fwd(const owt_fc_desc *d, const void *x, const void *w, const float *bias,
                            void *y, void *ws, size_t ws_bytes, void *hip_stream);

/* Fully-connected column shard backward (Section 4, backward step 1):
 *   dz = dy * [y > 0] with OWT_RELU (y required), else dy
 *   dx_partial[n,i] = sum_o dz[n,o] * w[o,i]     this worker's addend of the sum over workers;
 *                                                skipped when dx_partial_or_null is NULL
 *   dw[o,i] = alpha * sum_n dz[n,o] * x[n,i] + beta * dw;   dbias[o] likewise (NULL to skip)
 * dy, y [N,O_local]; dx_partial [N,I]; dw [O_local,I] fp32; dbias [O_local] fp32.
 * ws (owt_fc_workspace_bytes of pass OWT_PASS_BWD_DATA; that figure covers both
 * products) holds a masked, zero-padded copy of dz and the partial sums of a split
 * reduction while the call runs. */
owt_status owt_fc_shard_bwd(const owt_fc_desc *d, const void *x, const void *w, const void *y_or_null,
                            const void *dy, float alpha, float beta, void *dx_partial_or_null,
                            float *dw, float *dbias_or_null, void *ws, size_t ws_bytes,
                            void *hip_stream);

/* Optional tuning of a dense shard, as owt_conv_autotune does for a convolution:
 * times every kernel variant of the three passes (forward; the two halves of
 * owt_fc_shard_bwd, and whether those two run faster as one launch or as two)
 * on the caller's buffers and remembers the fastest for later
 * owt_fc_shard_* calls with an identical descriptor in this process.  Reads x,
 * w, bias, y (ReLU mask), dy; writes y, dx_partial, dw, dbias (alpha 1, beta 0).
 * All of these are required except dbias.  ws must hold the larger of the two
 * owt_fc_workspace_bytes values.  Blocks until the timing is done. */
owt_status owt_fc_autotune(const owt_fc_desc *d, const void *x, const void *w, const float *bias, void *y,
                           const void *dy, void *dx_partial, float *dw, float *dbias_or_null, void *ws,
                           size_t ws_bytes, void *hip_stream);

/* Max pooling between the convolution layers of the Section 5 model, window
 * win x win (2..15), stride >= 1, no padding: P = floor((H-win)/stride)+1.
 *   y[n,p,q,c] = max_{r,s<win} x[n, p*stride+r, q*stride+s, c]
 *   argmax[n,p,q,c] = r*win+s of the first maximum in row-major (r,s) order.
 * x [N,H,W,C], y [N,P,Q,C], argmax [N,P,Q,C] bytes (both written). */
owt_status owt_maxpool_fwd(int N, int H, int W, int C, int win, int stride, owt_dtype dtype,
                           const void *x, void *y, unsigned char *argmax, void *hip_stream);

/* Max pooling backward: dx[n,h,w,c] = sum of dy[n,p,q,c] over the windows
 * (p,q) whose argmax names (h,w); dx [N,H,W,C] is written everywhere. */
owt_status owt_maxpool_bwd(int N, int H, int W, int C, int win, int stride, owt_dtype dtype,
                           const void *dy, const unsigned char *argmax, void *dx, void *hip_stream);

/* owt_maxpool_bwd with the backward pass of a ReLU that sits between a
 * convolution and this pooling fused in: y_pooled [N,P,Q,C] is the pooling
 * OUTPUT; windows whose pooled value is <= 0 contribute nothing.  Exactly equal
 * to masking dx with [pool input > 0] afterwards, because the element a window
 * routes its gradient to holds that window's maximum. */
owt_status owt_maxpool_bwd_relu(int N, int H, int W, int C, int win, int stride, owt_dtype dtype,
                                const void *dy, const unsigned char *argmax, const void *y_pooled, void *dx,
                                void *hip_stream);

/* Weight update rule of Section 5, in place, one launch per tensor:
 *     vel := mu*vel + eps*(gscale*g - omega*w);   w := w + vel
 * mu = momentum, eps = learning rate, omega = weight decay.  g is the gradient as
 * the caller holds it (e.g. dw of owt_conv_bwd_filter / owt_fc_shard_bwd);
 * gscale folds in the batch mean when g is a sum (1/N) and the sign: the rule
 * as printed ADDS the gradient of an objective that is maximised, a caller that
 * minimises a loss passes a negative gscale.  w, vel, g: n fp32 values on the
 * device, 16-byte aligned, w and vel updated in place, g only read.  If
 * w_bf16_or_null is given it receives the new w rounded to bf16 (nearest even):
 * the weights a bf16-storage convolution then reads.  n == 0 is a no-op.
 * Errors: NULL/misaligned pointer or a non-finite coefficient -> OWT_EINVAL. */
owt_status owt_sgd_momentum_update(size_t n, float *w, float *vel, const float *g, float mu, float eps, float omega,
                                   float gscale, void *w_bf16_or_null, void *hip_stream);

/* Hyperparameters for a batch k times larger (Section 5, host arithmetic only):
 * eps_out = sqrt(k)*eps and omega_out = (1 - (1 - eps*omega)^k) / eps_out, so that
 * one application of weight decay at the new batch size shrinks a weight as much
 * as k applications did at the old one.  eps_out/omega_out are HOST pointers.
 * Errors: k or eps not positive and finite, NULL output -> OWT_EINVAL. */
owt_status owt_scale_hyperparameters(double k, double eps, double omega, double *eps_out, double *omega_out);

/* Output layer of Section 5: independent logistic units trained with
 * cross-entropy, on the O_local columns [col_offset, col_offset + O_local) of
 * the layer that this worker owns.  With s = 1/(1+exp(-z)) and target
 * t[n][j] = 1 if labels[n] == col_offset + j, else 0:
 *     loss[n]  = - sum_j ( t*log s + (1-t)*log(1-s) )     (this shard's share, fp32)
 *     dz[n][j] = scale * (s - t)                           (stored in `dtype`)
 * There is no normalisation across classes, so nothing is needed from the other
 * workers; the full loss of a sample is the sum of the shards' shares.
 * z, dz: [N, O_local] in `dtype` (dz may alias z); labels: N ints (class index in
 * the whole layer; one outside this shard means no positive target here);
 * loss: N floats.  All device pointers, 16-byte aligned.  Evaluated without
 * overflow for any finite z.  Errors: non-positive sizes, NULL/misaligned
 * pointers -> OWT_EINVAL; more than 2^31-1 elements -> OWT_EUNSUPPORTED. */
owt_status owt_logistic_xent(int N, int O_local, int col_offset, owt_dtype dtype, const void *z, const int *labels,
                             float scale, float *loss, void *dz, void *hip_stream);

/* Message for the calling thread's most recent non-OK return ("" if none).
 * Points at thread-local static storage; valid until the thread's next call. */
const char *owt_last_error(void);

/* TEST HOOK -- not part of the computation's interface.  The library's test suite has to run every
 * kernel instantiation, also those the planner would not pick for a small test shape.  This call
 * overrides the planner for ALL later calls of the process until it is called again with
 * (-1, 0, 0): `tile` >= 0 restricts the candidates to that tile / variant number of whichever kernel
 * family serves the pass (families with a variant table of their own count from 0; 10..12 are the fp32 filter
 * gradient with the pixel split inside the work-group, 16..19 the dense shard kernel's four tiles, 20/21 and
 * 22/23 the two fp32 first-layer forward / filter-gradient kernels, 24/25 the two bf16 first-layer
 * filter-gradient kernels, 30..36 the bf16 filter gradient that
 * streams its operands into LDS), `splitk` > 0 forces the
 * split count of the reduction (clamped to the number of reduction steps), `flags` is a set of
 * OWT_FORCE_* bits.  While an override is active, tuned and cached plans are ignored.  The three
 * values are stored atomically, but a launch that runs concurrently with this call may see the old
 * or the new setting: production code has no reason to call it. */
enum {
    OWT_FORCE_NO_DIRECT = 1u,       /* gather kernel only                                              */
    OWT_FORCE_ONLY_DIRECT = 2u,     /* never the gather kernel when another one qualifies              */
    OWT_FORCE_NO_BF16_MFMA = 4u,    /* bf16 storage on the fp32-MFMA kernels (widening loads)          */
    OWT_FORCE_FC_ONE_LAUNCH = 8u,   /* owt_fc_shard_bwd: both products in one launch                   */
    OWT_FORCE_FC_TWO_LAUNCHES = 16u /* owt_fc_shard_bwd: one launch per product                        */
};
void owt_test_force_variant(int tile, int splitk, unsigned flags);

/* Library ABI version (bumped on any signature change). */
int owt_abi_version(void);

/* Host-only self check of the index arithmetic helpers and the tile planner
 * (no GPU needed).  Returns 0 when everything holds; otherwise non-zero and
 * owt_last_error() names the failing case. */
int owt_selftest_host(void);

#ifdef __cplusplus
}
#endif
#endif /* OWT_H */
