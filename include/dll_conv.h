/*
 * dll_conv.h — C ABI of the MI355X (gfx950) implementation of the batched
 * 2D-convolution hot path of DLL (arxiv 1804.04512).
 *
 * What the paper defines (Section II-A): every minibatch of N images is convolved with
 * K kernels; the forward pass uses a "valid" convolution (the map shrinks), the backward
 * pass a "full" convolution (the map expands back), a third convolution of the layer
 * input with the output gradient yields the filter gradient; dense layers are matrix
 * products; activations and gradient operations are fused around them; all arithmetic
 * is single precision and works on whole minibatches; kernels are launched
 * asynchronously and data stays on the device.
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer to a contiguous, row-major tensor.  fp32
 *     unless stated; labels are int32; pooling indices are one byte each.
 *   - The CALLER owns all memory.  The library never allocates, frees or keeps a pointer
 *     after the call returns.  Scratch comes from `ws` (`ws_bytes` >= the matching
 *     *_workspace_bytes query, 256-byte aligned); its contents are undefined afterwards.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue work and return without synchronising.
 *   - Layouts: x [N][C][H][W]; w [K][C][R][S]; bias [K]; stride 1;
 *     Ho = H + 2*pad - R + 1, Wo = W + 2*pad - S + 1;
 *     y and pool_idx [N][K][Ho/pool][Wo/pool].
 *   - `dy` always means the gradient w.r.t. the layer OUTPUT y (after activation and
 *     pooling); the library applies the pooling/activation derivative itself.
 *   - Errors are reported as dll_status before anything is launched: a missing required
 *     pointer -> DLL_ERR_NULL; non-positive sizes, a filter larger than the padded input,
 *     pad > R-1 or S-1, pooling on an odd map, an input aliasing an output (exact pointer
 *     equality only; partial overlap is undetected and undefined) -> DLL_ERR_SHAPE; an
 *     activation or pooling mode outside the enums, or a tensor of 2^31 or more elements
 *     -> DLL_ERR_UNSUPPORTED; a workspace that is too small or misaligned ->
 *     DLL_ERR_WORKSPACE; a failed launch -> DLL_ERR_DEVICE.  No exception crosses the ABI.
 */
#ifndef DLL_CONV_H
#define DLL_CONV_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DLL_OK = 0,
  DLL_ERR_NULL = 1,
  DLL_ERR_SHAPE = 2,
  DLL_ERR_UNSUPPORTED = 3,
  DLL_ERR_WORKSPACE = 4,
  DLL_ERR_DEVICE = 5,
  DLL_ERR_SCRATCH_LIMIT = 6 /* dll_conv_valid_wgrad_noalloc only: the layer needs more than its built-in scratch */
} dll_status;

/* Activation functions the paper's networks use (Sections II-B, IV-B, V, VI). */
typedef enum { DLL_ACT_IDENTITY = 0, DLL_ACT_SIGMOID = 1, DLL_ACT_RELU = 2 } dll_act;

/* One stride-1 convolution layer (Section II-A: N images, K kernels). */
typedef struct {
  int N, C, H, W; /* input minibatch, NCHW                                        */
  int K, R, S;    /* K filters of C x R x S                                       */
  int pad;        /* zeros added on every side; 0 = the paper's "valid"           */
  int act;        /* dll_act applied to conv + bias                               */
  int pool;       /* 1 = none, 2 = 2x2 stride-2 max pooling (Ho and Wo even)      */
} dll_conv_desc;

/* One fully-connected layer, weights [out][in] (Section II-A). */
typedef struct {
  int in, out, act;
} dll_dense_desc;

/* A CNN: n_conv convolution layers (all with the same N, each consuming the previous
 * one's output), flattened NCHW row-major into n_dense dense layers; the last dense layer
 * is linear (its `act` is ignored) and feeds a softmax cross-entropy over `classes`.
 * n_conv may be 0: then the network is fully connected (Section IV-A), its input x is
 * [batch][dense[0].in] and `batch` gives the mini-batch size; with n_conv > 0 `batch` is
 * ignored (the batch is conv[0].N) and `conv` must not be NULL. */
typedef struct {
  int n_conv;
  const dll_conv_desc *conv; /* host pointer */
  int n_dense;
  const dll_dense_desc *dense; /* host pointer */
  int classes;
  int batch;
} dll_net_desc;

/* Visible unit types of the RBM steps (Section II). */
typedef enum { DLL_VISIBLE_BINARY = 0, DLL_VISIBLE_GAUSSIAN = 1 } dll_visible_unit;

const char *dll_status_string(dll_status s);

/* Bytes of scratch the three single-layer calls below need at most (host computation). */
size_t dll_conv_workspace_bytes(const dll_conv_desc *d);

/* Forward layer (Section II-A: the valid convolution of the forward pass):
 *   z[n,k,i,j] = bias[k] + sum_{c,r,s} xpad[n,c,i+r,j+s] * w[k,c,r,s]
 *   y = maxpool2x2(act(z)) when pool == 2, else act(z)
 * pool_idx (required iff pool == 2) receives, in bits 0-1 of each byte, 2*a+b of the window's
 * maximum (first one in the order (0,0),(0,1),(1,0),(1,1) on ties of the pre-activation).
 * When act is ReLU, bit 2 (value 4) is also set where the pooled output is zero, i.e. where
 * the unit passes no gradient; all other bits are zero.  bias may be NULL. */
dll_status dll_conv_valid_fwd(const dll_conv_desc *d, const float *x, const float *w,
                              const float *bias, float *y, unsigned char *pool_idx, void *ws,
                              size_t ws_bytes, void *stream);

/* Backward-data layer (Section II-A: the full convolution of the backward pass):
 *   dz = unpool(dy, pool_idx) * act'(y)          (never stored)
 *   dx[n,c,i,j] = sum_{k,r,s} dz[n,k,i+pad-r,j+pad-s] * w[k,c,r,s]
 * pool_idx is required iff pool == 2; only bits 0-1 of its bytes are read when y is given.
 * y may be NULL when act is the identity.  y may also be NULL when act is ReLU and pool == 2:
 * then act'(y) is taken from bit 2 of pool_idx as dll_conv_valid_fwd wrote it (zero gradient
 * where the bit is set) and the layer output is not read at all. */
dll_status dll_conv_full_bwd(const dll_conv_desc *d, const float *dy, const float *y,
                             const unsigned char *pool_idx, const float *w, float *dx, void *ws,
                             size_t ws_bytes, void *stream);

/* The same backward-data layer computed through the Fourier transform (Section II-A's first
 * implementation of the full convolution: image and filter padded to the output size,
 * transformed, multiplied point by point, transformed back, each image transformed once for all
 * filters).  Same arguments, same result up to rounding (fp32 throughout).  Padded sides are the
 * next powers of two: the full-convolution size (Ho + R - 1) x (Wo + S - 1) must not exceed
 * 64 x 64, else DLL_ERR_UNSUPPORTED (and a workspace size of 0); within that, filters may be
 * larger than the direct kernels take (R * S > 144).  ws holds the spectra:
 * dll_conv_full_fft_workspace_bytes(d) bytes, device memory, caller-owned, overwritten. */
size_t dll_conv_full_fft_workspace_bytes(const dll_conv_desc *d);
dll_status dll_conv_full_bwd_fft(const dll_conv_desc *d, const float *dy, const float *y,
                                 const unsigned char *pool_idx, const float *w, float *dx, void *ws,
                                 size_t ws_bytes, void *stream);

/* Filter-gradient layer (Section II-A, gradient computations):
 *   dw[k,c,r,s] = sum_{n,i,j} dz[n,k,i,j] * xpad[n,c,i+r,j+s];  dbias[k] = sum_{n,i,j} dz[n,k,i,j]
 * with dz as above (same rules for y and pool_idx).  dbias may be NULL.  The batch reduction is a fixed-order tree:
 * results are bit-identical from run to run. */
dll_status dll_conv_valid_wgrad(const dll_conv_desc *d, const float *x, const float *dy,
                                const float *y, const unsigned char *pool_idx, float *dw,
                                float *dbias, void *ws, size_t ws_bytes, void *stream);

/* The two launches of dll_conv_valid_wgrad as calls of their own, for callers that gather the
 * reductions of several layers behind their filter-gradient kernels (the training step below does
 * that with its closing launch) or that time the kernel alone.  _partial runs the filter-gradient
 * kernel: it leaves the per-workgroup partial sums of dw and dbias in ws (same size as above,
 * layout private to the library) and writes nothing else.  _finish adds them up in the fixed
 * order and writes dw (and dbias unless NULL); it reads ws as the _partial call of the SAME
 * descriptor left it, on the same stream or after it.  The two in a row give bit for bit what
 * dll_conv_valid_wgrad gives.  Errors as there; dw == ws -> DLL_ERR_SHAPE. */
dll_status dll_conv_valid_wgrad_partial(const dll_conv_desc *d, const float *x, const float *dy,
                                        const float *y, const unsigned char *pool_idx, void *ws,
                                        size_t ws_bytes, void *stream);
dll_status dll_conv_valid_wgrad_finish(const dll_conv_desc *d, float *dw, float *dbias,
                                       const void *ws, size_t ws_bytes, void *stream);

/* The same filter-gradient layer for callers that cannot allocate device memory or carry a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments (minus the workspace), same kernels, bit-identical results; the partial sums
 * live in an array built into the library, DLL_NOALLOC_SCRATCH_BYTES of device memory that every
 * GPU the library runs on holds until the process ends.  The call allocates and frees nothing.
 *   - A layer whose dll_conv_workspace_bytes(d) exceeds DLL_NOALLOC_SCRATCH_BYTES is rejected
 *     with DLL_ERR_SCRATCH_LIMIT before anything is launched (config 5's largest layer needs 3.7 MB).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race and give undefined results; calls on one stream are ordered.
 *     Nothing in the array has to be cleared between calls.
 *   - The first call on a device asks the runtime for the array's address on that device; make
 *     that first call outside graph capture. */
#define DLL_NOALLOC_SCRATCH_BYTES ((size_t)8 << 20)
dll_status dll_conv_valid_wgrad_noalloc(const dll_conv_desc *d, const float *x, const float *dy,
                                        const float *y, const unsigned char *pool_idx, float *dw,
                                        float *dbias, void *stream);

/* One CD-1 step of a convolutional RBM with binary visible and hidden units (Section II:
 * RBM/CRBM trained with Contrastive Divergence).  d->act and d->pool are ignored.
 *   h0p = sigmoid(b_hid[k] + valid(v0, W));   h0s = 1[uniform < h0p]   (or h0_sample_in)
 *   v1  = sigmoid(c_vis[ch] + full(h0s, W));  h1p = sigmoid(b_hid[k] + valid(v1, W))
 *   dW = (grad(v0,h0p) - grad(v1,h1p)) / N;   db[k] = sum(h0p - h1p) / N;
 *   dc[ch] = sum(v0 - v1) / N;                recon_mse = mean((v0 - v1)^2)
 *   lr != 0:  W += lr*dW, b_hid += lr*db, c_vis += lr*dc   (after all gradients are formed)
 * uniform [N][K][Ho][Wo] in [0,1) is required unless h0_sample_in is given.  dW, db, dc are
 * required; h0_prob, h0_sample, v1, h1_prob and recon_mse (device scalar) may be NULL. */
size_t dll_crbm_workspace_bytes(const dll_conv_desc *d);
dll_status dll_crbm_cd1_step(const dll_conv_desc *d, const float *v0, float *W, float *b_hid,
                             float *c_vis, const float *uniform, const float *h0_sample_in,
                             float lr, float *dW, float *db, float *dc, float *h0_prob,
                             float *h0_sample, float *v1, float *h1_prob, float *recon_mse,
                             void *ws, size_t ws_bytes, void *stream);

/* The CD-1 step with a choice of visible unit and of hidden layer (Section II: the RBM's unit
 * types; the CRBM's second version with probabilistic max pooling).  Everything not said here
 * is as in dll_crbm_cd1_step, which is this call with (DLL_VISIBLE_BINARY, hidden_pool 1).
 *   visible  DLL_VISIBLE_BINARY:   v1 = sigmoid(c_vis[ch] + full(h0s, W))
 *            DLL_VISIBLE_GAUSSIAN: v1 = c_vis[ch] + full(h0s, W)   (unit variance; the mean)
 *   hidden_pool 1: independent binary hidden units, uniform [N][K][Ho][Wo]
 *   hidden_pool 2: probabilistic max pooling over 2x2 blocks (Ho and Wo even, else
 *            DLL_ERR_SHAPE): with I = b_hid[k] + valid(v, W), P(h_i = 1) = exp(I_i) /
 *            (1 + sum over the block of exp(I_j)); at most one unit of a block is on.
 *            uniform [N][K][Ho/2][Wo/2] holds one number u per block: with the block's
 *            probabilities q0..q3 (order 2a+b) and fp32 running sums s_i = s_(i-1) + q_i,
 *            unit i is on iff s_(i-1) <= u < s_i, none when u >= s_3.
 *            pool_prob (nullable; must be NULL when hidden_pool is 1) [N][K][Ho/2][Wo/2]
 *            receives P(pooling unit on | v0) = q0 + q1 + q2 + q3. */
dll_status dll_crbm_cd1_step_units(const dll_conv_desc *d, int visible, int hidden_pool,
                                   const float *v0, float *W, float *b_hid, float *c_vis,
                                   const float *uniform, const float *h0_sample_in, float lr,
                                   float *dW, float *db, float *dc, float *h0_prob,
                                   float *h0_sample, float *pool_prob, float *v1, float *h1_prob,
                                   float *recon_mse, void *ws, size_t ws_bytes, void *stream);

/* One CD-1 step of a fully-connected RBM (Section II: RBM trained with Contrastive
 * Divergence; Section II-A: every dense product is one matrix-matrix multiplication).
 *   v0 [batch][n_vis], W [n_hid][n_vis], b_hid [n_hid], c_vis [n_vis], uniform [batch][n_hid]
 *   h0p = sigmoid(b_hid + v0 W^T);  h0s = 1[uniform < h0p]  (or h0_sample_in)
 *   v1  = sigmoid(c_vis + h0s W)  (DLL_VISIBLE_BINARY)  or  c_vis + h0s W  (DLL_VISIBLE_GAUSSIAN)
 *   h1p = sigmoid(b_hid + v1 W^T)
 *   dW = (h0p^T v0 - h1p^T v1) / batch;  db = colsum(h0p - h1p) / batch;
 *   dc = colsum(v0 - v1) / batch;  recon_mse = mean((v0 - v1)^2)
 *   lr != 0:  W += lr*dW, b_hid += lr*db, c_vis += lr*dc   (after all gradients are formed)
 * All pointers are device pointers, 16-byte aligned.  dW, db, dc are required; h0_prob,
 * h0_sample, v1, h1_prob [same shapes as above] and recon_mse (device scalar) may be NULL.
 * Returns DLL_ERR_WORKSPACE when ws is smaller than dll_rbm_workspace_bytes says. */
size_t dll_rbm_workspace_bytes(int batch, int n_vis, int n_hid);
dll_status dll_rbm_cd1_step(int batch, int n_vis, int n_hid, int visible, const float *v0,
                            float *W, float *b_hid, float *c_vis, const float *uniform,
                            const float *h0_sample_in, float lr, float *dW, float *db, float *dc,
                            float *h0_prob, float *h0_sample, float *v1, float *h1_prob,
                            float *recon_mse, void *ws, size_t ws_bytes, void *stream);

/* One mini-batch gradient-descent step of a CNN (Sections II, IV-B, V, VI): forward
 * through every layer, softmax cross-entropy averaged over the batch, backward (full
 * convolutions for the data gradients except into the network input, filter gradients,
 * dense products with the transposed weights), then theta <- theta - lr * grad.
 *   params  host array of 2*(n_conv+n_dense) device pointers: conv w0,b0,w1,b1,... then
 *           dense W0,b0,...; updated in place when lr != 0
 *   grads   NULL, or a host array in the same order; each non-NULL entry receives that
 *           gradient (taken at the parameters as they were on entry)
 *   labels  [N] int32 in [0, classes)
 *   loss    device scalar, required;  logits [N][classes], may be NULL
 *   pool_idx  NULL, or a host array of n_conv device pointers (entries may be NULL): each
 *           non-NULL entry of a pooled layer receives that layer's pooling indices, in the
 *           encoding dll_conv_valid_fwd writes */
size_t dll_cnn_workspace_bytes(const dll_net_desc *net);
dll_status dll_cnn_train_step(const dll_net_desc *net, float *const *params, float *const *grads,
                              const float *x, const int *labels, float lr, float *loss,
                              float *logits, unsigned char *const *pool_idx, void *ws,
                              size_t ws_bytes, void *stream);

/* The same step with momentum and weight decay (Section II names both as learning options,
 * Section IV trains with momentum 0.9).  Reading taken here, the classical form, per parameter:
 *   v <- momentum * v - lr * (g + weight_decay * theta);   theta <- theta + v
 * with weight_decay applied to filters and dense weights only (0 for biases).
 *   velocity  host array of device pointers, same order and shapes as params; required, updated
 *             in place when lr != 0 (start from zeros)
 * Everything else as in dll_cnn_train_step, which equals momentum = weight_decay = 0. */
dll_status dll_cnn_train_step_momentum(const dll_net_desc *net, float *const *params,
                                       float *const *velocity, float *const *grads, const float *x,
                                       const int *labels, float lr, float momentum,
                                       float weight_decay, float *loss, float *logits,
                                       unsigned char *const *pool_idx, void *ws, size_t ws_bytes,
                                       void *stream);

/* Inference pass of the same network description (Sections IV-VI: the networks the paper times
 * end in a softmax layer): the convolution blocks, the dense layers (the last one without
 * activation) and the softmax of its outputs.  Nothing is kept for a backward pass: activations
 * ping-pong between two workspace buffers and no pooling index is written.
 *   params  host array of 2*(n_conv+n_dense) device pointers, order as in dll_cnn_train_step; read only
 *   x       [N][C][H][W] of the first layer
 *   logits  [N][classes], may be NULL;  prob [N][classes], may be NULL (not both)
 * Errors as for dll_cnn_train_step. */
size_t dll_cnn_forward_workspace_bytes(const dll_net_desc *net);
dll_status dll_cnn_forward(const dll_net_desc *net, const float *const *params, const float *x,
                           float *logits, float *prob, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif
