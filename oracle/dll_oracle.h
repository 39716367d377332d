/*
 * CPU oracle for the batched 2D-convolution hot path of DLL (arxiv 1804.04512).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, direct-loop implementation of
 * what the paper's Section II-A names: the "valid" convolution used by the forward
 * pass, the "full" convolution used by the backward pass, the convolution that
 * yields the filter gradient, the dense-layer matrix products, the activation
 * functions, 2x2 max pooling, softmax cross-entropy, mini-batch gradient descent
 * (Section II) and the CD-1 step of a convolutional RBM (Section II, CRBM with
 * Contrastive Divergence; binary or Gaussian visible units; independent hidden units or
 * probabilistic max pooling) and of a fully-connected RBM.  The paper gives no formulas;
 * every function states the textbook definition it writes out.  Sums are accumulated in double and rounded to
 * the storage type once, on store.  Nothing here is blocked, fused or reordered,
 * and nothing here is used by, or shares code with, the GPU library.
 *
 * Every pointer is a HOST pointer.  Tensors are contiguous, row-major:
 *   x  [N][C][H][W]       minibatch of N images (Section II-A: N images per batch)
 *   w  [K][C][R][S]       K kernels
 *   y  [N][K][Ho/pool][Wo/pool]   with Ho = H + 2*pad - R + 1 (stride 1)
 *   pool_idx  same shape as y, one byte each: 2*a+b of the window's first maximum
 *
 * Two instantiations of the same source are exported:
 *   oracle_*    fp32 storage (the paper's precision), double accumulation
 *   oracle64_*  fp64 storage, used only by finite-difference pins
 */
#ifndef DLL_ORACLE_H
#define DLL_ORACLE_H

#ifdef __cplusplus
extern "C" {
#endif

enum { ORACLE_ACT_IDENTITY = 0, ORACLE_ACT_SIGMOID = 1, ORACLE_ACT_RELU = 2 };

typedef struct {
  int N, C, H, W; /* input minibatch */
  int K, R, S;    /* K filters of C x R x S */
  int pad;        /* zeros on every side; 0 = 'valid' */
  int act;        /* ORACLE_ACT_* */
  int pool;       /* 1 = none, 2 = 2x2 stride-2 max pool */
} oracle_conv_desc;

typedef struct {
  int in, out, act;
} oracle_dense_desc; /* W layout [out][in] */

typedef struct {
  int n_conv;
  const oracle_conv_desc *conv;
  int n_dense;
  const oracle_dense_desc *dense; /* last one: identity, followed by softmax-CE */
  int classes;
  int batch; /* minibatch size of a network without convolution layers (n_conv == 0: a
                fully-connected network, x is [batch][dense[0].in]); ignored otherwise */
} oracle_net_desc;

int oracle_max_threads(void);
void oracle_set_threads(int n);

#define ORACLE_DECLARE(PFX, REAL)                                                                \
  int PFX##conv_valid_fwd(const oracle_conv_desc *d, const REAL *x, const REAL *w,               \
                          const REAL *bias, REAL *y, unsigned char *pool_idx);                   \
  int PFX##conv_full_bwd(const oracle_conv_desc *d, const REAL *dy, const REAL *y,               \
                         const unsigned char *pool_idx, const REAL *w, REAL *dx);                \
  int PFX##conv_valid_wgrad(const oracle_conv_desc *d, const REAL *x, const REAL *dy,            \
                            const REAL *y, const unsigned char *pool_idx, REAL *dw, REAL *dbias);\
  int PFX##dense_fwd(int B, int in, int out, int act, const REAL *a, const REAL *W,              \
                     const REAL *b, REAL *h);                                                    \
  int PFX##dense_bwd(int B, int in, int out, int act, const REAL *a, const REAL *W,              \
                     const REAL *h, const REAL *dh, REAL *da, REAL *dW, REAL *db);               \
  int PFX##softmax_ce(int B, int classes, const REAL *logits, const int *labels, REAL *loss,     \
                      REAL *prob, REAL *dlogits);                                                \
  int PFX##sgd(long count, REAL *theta, const REAL *g, REAL lr);                                 \
  int PFX##sgd_momentum(long count, REAL *theta, REAL *vel, const REAL *g, REAL lr, REAL mu,     \
                        REAL decay);                                                             \
  int PFX##crbm_cd1_step(const oracle_conv_desc *d, const REAL *v0, REAL *W, REAL *b_hid,        \
                         REAL *c_vis, const REAL *uniform, const REAL *h0_sample_in, REAL lr,    \
                         REAL *dW, REAL *db, REAL *dc, REAL *h0_prob, REAL *h0_sample, REAL *v1, \
                         REAL *h1_prob, REAL *recon_mse);                                        \
  int PFX##crbm_cd1_step_units(const oracle_conv_desc *d, int visible, int hidden_pool,          \
                               const REAL *v0, REAL *W, REAL *b_hid, REAL *c_vis,                \
                               const REAL *uniform, const REAL *h0_sample_in, REAL lr, REAL *dW, \
                               REAL *db, REAL *dc, REAL *h0_prob, REAL *h0_sample,               \
                               REAL *pool_prob, REAL *v1, REAL *h1_prob, REAL *recon_mse);       \
  int PFX##rbm_cd1_step(int B, int nv, int nh, int visible, const REAL *v0, REAL *W,             \
                        REAL *b_hid, REAL *c_vis, const REAL *uniform, const REAL *h0_sample_in, \
                        REAL lr, REAL *dW, REAL *db, REAL *dc, REAL *h0_prob, REAL *h0_sample,   \
                        REAL *v1, REAL *h1_prob, REAL *recon_mse);                               \
  int PFX##cnn_train_step(const oracle_net_desc *net, REAL *const *params, REAL *const *grads,   \
                          const REAL *x, const int *labels, REAL lr, REAL *loss, REAL *logits,   \
                          const unsigned char *const *pool_idx_in, unsigned char *const *pool_idx_out, \
                          const unsigned char *const *active_in);                                \
  int PFX##cnn_forward(const oracle_net_desc *net, const REAL *const *params, const REAL *x,     \
                       REAL *logits, REAL *prob);

ORACLE_DECLARE(oracle_, float)
ORACLE_DECLARE(oracle64_, double)

#ifdef __cplusplus
}
#endif
#endif
