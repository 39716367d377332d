// Internal launch interfaces between the C-ABI layer and the gfx950 kernels.
// Host-side plain structs only; every pointer is a device pointer.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace dllk {

enum { ACT_IDENTITY = 0, ACT_SIGMOID = 1, ACT_RELU = 2 };
// Backward passes only: ReLU whose derivative comes from the flag bit in the pooling index
// (kIdxInactive) instead of from the layer output, which then is not read at all.
enum { ACT_RELU_FLAGGED = 3 };
// Forward epilogue only (pool == 1, even output extents): probabilistic max pooling over 2x2
// blocks, the hidden layer of the pooling CRBM (Section II).  `uniform` then holds one number per
// block, [N][Kout][Hout/2][Wout/2], and `out_pool` may receive the pooling units' probabilities.
enum { ACT_PMP = 4 };
// Pooling index byte: bits 0-1 hold the arg-max position 2a+b inside the 2x2 window; the
// forward pass of a ReLU layer also sets kIdxInactive where the pooled output is zero.
constexpr unsigned char kIdxPosMask = 3, kIdxInactive = 4;

// What the launchers need to know of the GPU they size their grids for: the number of compute
// units and the LDS of one compute unit, asked of the runtime once per device.
struct ChipInfo { int cus = 0; size_t lds_bytes = 0; };
const ChipInfo &chip();
// Kernels that use more than 64 KB of dynamic LDS need the limit raised once per kernel and device;
// this remembers which it has done.  A no-op for smaller sizes.
hipError_t allow_large_lds(const void *kernel, size_t lds_bytes);

// In-place parameter update, shared by every kernel that produces a gradient g of a parameter theta:
//   v == NULL:  theta += step * g                                    (plain descent, step = -lr)
//   v != NULL:  v = mu * v + step * (g + decay * theta);  theta += v  (momentum and weight decay)
__host__ __device__ __forceinline__ void update_param(float *theta, float *v, float g, float step, float mu, float decay) {
  if (v) {
    const float nv = mu * (*v) + step * (g + decay * (*theta));
    *v = nv;
    *theta += nv;
  } else {
    *theta += step * g;
  }
}

// ---------------------------------------------------------------------------------------
// Forward-form implicit-GEMM convolution engine (fp32 MFMA 16x16x4).
//   out[n,ko,i,j] = epilogue( sum_{ci,r,s} srcpad[n,ci,i+r,j+s] * wgt(ko,ci,r,s) )
// It serves the forward layer (src = x), the backward-data layer (src = dz derived on the
// fly from dy/y/pool_idx, filters flipped and transposed, pad' = R-1-pad: the paper's
// "full convolution = valid convolution with padding", Section II-A) and the CRBM
// reconstruction.
// ---------------------------------------------------------------------------------------
struct ConvEngineArgs {
  // logical source, extent [N][Cin][Hin][Win]
  const float *src = nullptr;             // plain: the tensor itself; dz mode: dy at output resolution
  const float *src_y = nullptr;           // dz mode: layer output (needed unless src_act is identity)
  const unsigned char *src_idx = nullptr; // dz mode with src_pool == 2
  int src_dz = 0;                         // 0 plain, 1 derive dz = unpool(dy) * act'(y)
  int src_act = ACT_IDENTITY, src_pool = 1;
  int N = 0, Cin = 0, Hin = 0, Win = 0;
  // filters
  const float *w = nullptr;
  int w_flip = 0;                         // 0: w[Kout][Cin][R][S];  1: w[Cin][Kout][R][S] rotated by 180 degrees
  int Kout = 0, R = 0, S = 0;
  int pad_h = 0, pad_w = 0;              // implicit zero border of the logical source
  // output, pre-pool extent Hout x Wout
  int Hout = 0, Wout = 0;
  const float *bias = nullptr;
  int act = ACT_IDENTITY, pool = 1;
  float *out = nullptr;
  unsigned char *out_idx = nullptr;           // pool == 2: optional (an inference pass does not keep the decisions)
  const float *uniform = nullptr;         // optional Bernoulli epilogue (pool == 1): sample = 1[uniform < out]
  float *sample = nullptr;
  float *out_pool = nullptr;              // act == ACT_PMP: optional P(pooling unit on), [N][Kout][Hout/2][Wout/2]
};

hipError_t launch_conv_engine(const ConvEngineArgs &a, hipStream_t stream);

// The same operation for at most three output channels (CRBM reconstruction, backward-data into a
// grey-scale or RGB input): output columns instead of output channels ride on the MFMA N axis.
// launch_conv_engine routes there by itself when it pays.
// Padded 3x3 layers with 16 or 32 channels in and out, ReLU + pooling, on whole 8 x 32 tiles, in the
// minimal-filtering form F(2x2, 3x3): the forward pass, and the backward-data pass from the pooled
// gradient with the ReLU flags in the pooling bytes.  launch_conv_engine routes there by itself.
bool conv_wino_applies(const ConvEngineArgs &a);
hipError_t launch_conv_wino(const ConvEngineArgs &a, hipStream_t stream);
// Forward pass of a padded 3x3 layer with one to three input channels and at most 16 filters, ReLU +
// pooling (the first layer of the image networks); launch_conv_engine routes there by itself.
bool conv_fwd_fewch_applies(const ConvEngineArgs &a);
hipError_t launch_conv_fwd_fewch(const ConvEngineArgs &a, hipStream_t stream);
// Forward pass of a padded 3x3 layer with 16 channels in and 16 filters, ReLU + pooling, in the
// minimal-filtering form as a wavefront-private streaming kernel; launch_conv_engine routes there by itself.
bool conv_wino_stream_applies(const ConvEngineArgs &a);
bool conv_wino_stream_bwd_applies(const ConvEngineArgs &a);   // the backward-data pass of such a layer (same launcher)
hipError_t launch_conv_wino_stream(const ConvEngineArgs &a, hipStream_t stream);

bool conv_fewout_applies(const ConvEngineArgs &a);
hipError_t launch_conv_fewout(const ConvEngineArgs &a, hipStream_t stream);

// Backward-data through the Fourier transform (Section II-A's second route for the full
// convolution): full-convolution sizes up to 64 x 64.  xf and wf are scratch for the spectra,
// ceil(N/2)*K and K*C images of F = PH*PW complex numbers (PH, PW from conv_fft_plan as powers of two).
struct ConvFftArgs {
  const float *dy = nullptr, *y = nullptr;
  const unsigned char *idx = nullptr;
  int act = ACT_IDENTITY, pool = 1;       // of the layer whose gradient comes in (ACT_RELU_FLAGGED: flags in idx)
  int N = 0, K = 0, C = 0, Ho = 0, Wo = 0, R = 0, S = 0, H = 0, W = 0, pad = 0;
  const float *w = nullptr;               // [K][C][R][S]
  float *dx = nullptr;                    // [N][C][H][W]
  float2 *xf = nullptr, *wf = nullptr;
};
bool conv_fft_plan(int Ho, int Wo, int R, int S, int *lph, int *lpw);
hipError_t launch_conv_full_fft(const ConvFftArgs &a, hipStream_t stream);

// ---------------------------------------------------------------------------------------
// Filter gradient: stage 1 leaves per-wave partial sums in `partial`, stage 2
// (launch_wgrad_reduce) adds them in a fixed order.
// ---------------------------------------------------------------------------------------
struct WgradArgs {
  const float *x = nullptr;               // [N][C][H][W]
  const float *dy = nullptr;              // gradient at output resolution [N][K][Ho/pool][Wo/pool]
  const float *y = nullptr;
  const unsigned char *idx = nullptr;
  int act = ACT_IDENTITY, pool = 1;
  int N = 0, C = 0, H = 0, W = 0, K = 0, R = 0, S = 0, pad = 0;
  float *partial = nullptr;               // wgrad_partial_floats(...) floats
};

struct WgradPlan {
  int MTF, NTT;        // 16-filter tiles, 16-tap tiles per channel chunk
  int CC, nchunks;     // channels per chunk
  int G;               // workgroups per chunk
  int TH;              // tile height (8 or 16); width is 32
  size_t lds_bytes;
  size_t partial_floats; // dw partials followed by db partials
  size_t db_offset;      // float offset of the db partials
  int n_partials;        // per chunk: one block per workgroup (G)
};

// `shared_launch`: the plan of a filter gradient that shares its launch with the layer's backward-data
// pass (half as many workgroups; only the minimal-filtering shapes have such a form, others plan as ever)
bool plan_wgrad(int N, int C, int H, int W, int K, int R, int S, int pad, int pool, WgradPlan *plan, bool shared_launch = false);
// Padded 3x3 layers with 16 or 32 channels in and out behind ReLU + pooling, gradient and pooling bytes
// alone (no layer output): the minimal-filtering form F(3x3, 2x2), same partial blocks as the direct
// kernel.  launch_wgrad routes there by itself.
bool wgrad_wino_shape(int C, int H, int W, int K, int R, int S, int pad, int pool);
bool wgrad_wino_applies(const WgradArgs &a, const WgradPlan &plan);
hipError_t launch_wgrad_wino(const WgradArgs &a, const WgradPlan &plan, hipStream_t stream);
// That filter gradient and the layer's backward-data pass (streaming form) in ONE launch, half of the
// workgroups each; `plan` must be one made for a shared launch (plan_wgrad's last argument).
bool wgrad_bwd_pair_applies(const WgradArgs &w, const WgradPlan &plan, const ConvEngineArgs &b);
hipError_t launch_wgrad_bwd_pair(const WgradArgs &w, const WgradPlan &plan, const ConvEngineArgs &b, hipStream_t stream);
// Padded 3x3 layers with one to three input channels and at most 16 filters behind ReLU + pooling
// (the first layer of the image networks), gradient and pooling bytes alone: the filter-side operand
// is formed in registers from the pooled tensors.  Same partial blocks; launch_wgrad routes there.
bool wgrad_fewch_shape(int C, int H, int W, int K, int R, int S, int pad, int pool);
bool wgrad_fewch_applies(const WgradArgs &a, const WgradPlan &plan);
hipError_t launch_wgrad_fewch(const WgradArgs &a, const WgradPlan &plan, hipStream_t stream);
hipError_t launch_wgrad(const WgradArgs &a, const WgradPlan &plan, hipStream_t stream);

// dw = scale * (sum(pos partials) - sum(neg partials)); optional in-place theta += step * dw.
struct WgradReduceArgs {
  const float *pos = nullptr;  // partial buffer of the positive phase
  const float *neg = nullptr;  // nullable: partial buffer of the negative phase (same plan)
  float scale = 1.0f;
  float *dw = nullptr;         // nullable
  float *db = nullptr;         // nullable
  float *w_update = nullptr;   // nullable: w_update += step * dw
  float *b_update = nullptr;   // nullable
  float step = 0.0f;
  float *w_vel = nullptr, *b_vel = nullptr;   // nullable: momentum buffers of the filters and biases
  float mu = 0.0f, w_decay = 0.0f;            // momentum; weight decay (filters only)
  int C = 0, K = 0, R = 0, S = 0;
};
hipError_t launch_wgrad_reduce(const WgradReduceArgs &a, const WgradPlan &plan, hipStream_t stream);

// ---------------------------------------------------------------------------------------
// Dense layers: C[M][N] (+)= A * B with arbitrary element strides, fp32 MFMA.
// ---------------------------------------------------------------------------------------
struct GemmArgs {
  int M = 0, N = 0, Kdim = 0;
  const float *A = nullptr; long a_m = 0, a_k = 0;   // A(m,k) = A[m*a_m + k*a_k]
  const float *B = nullptr; long b_k = 0, b_n = 0;   // B(k,n) = B[k*b_k + n*b_n]
  float *Cout = nullptr; long c_m = 0, c_n = 0;      // nullable when only the update is wanted
  const float *bias = nullptr;                       // [N], added before act
  int act = ACT_IDENTITY;
  // optional factor applied last: C(m,n) *= act'(C_ref(m,n)), C_ref with the strides of Cout (dense
  // backward: the data gradient leaves as dz of the layer below, dz = dh * act'(h))
  const float *C_ref = nullptr; int c_ref_act = ACT_IDENTITY;
  float *update = nullptr; float step = 0.0f;        // nullable: update(m,n) += step * C(m,n), same strides as Cout
  float *vel = nullptr; float mu = 0.0f, decay = 0.0f; // nullable momentum buffer of `update` (see update_param)
  int split_k = 1;
  float *partial = nullptr;                          // split_k * M * N floats when split_k > 1
  // split_k > 1 only: leave the partials as they are; the consumer adds them (in split order,
  // then the bias) itself.  Only for an identity epilogue without update.
  bool defer_reduce = false;
  // split_k <= 1 only: take the small-product kernel although the product is larger than
  // gemm_is_small() allows (see gemm_prefers_small)
  bool small_form = false;
  // Softmax + cross-entropy in the epilogue (only where gemm_fuses_softmax() says so: every row of
  // logits lies inside one 16-column tile): Cout receives the logits, sm_dz (strides of Cout)
  // (softmax - onehot(label)) * sm_scale, sm_rowloss[m] = -ln softmax[label].
  const int *sm_labels = nullptr;
  float *sm_dz = nullptr, *sm_rowloss = nullptr;
  float sm_scale = 1.0f;
};
int gemm_pick_split_k(int M, int N, int Kdim);
hipError_t launch_gemm(const GemmArgs &a, hipStream_t stream);
// Two products that do not depend on each other, in one launch where their forms allow it.
hipError_t launch_gemm_pair(const GemmArgs &a, const GemmArgs &b, hipStream_t stream);
// Small products (the dense layers of the MNIST/CIFAR-sized networks) take a kernel built for a
// short latency chain instead: 32 x 32 tiles, the k range split between the wavefronts of a
// workgroup, no split-K partials (gemm_pick_split_k returns 1 for them).  launch_gemm routes there.
bool gemm_is_small(int M, int N, int Kdim);
// Data-gradient products (A contiguous along k, B along n) of up to 2^28 multiply-adds are still
// faster there than as a split-K product with its reduction launch behind it (measured on the
// 128 x 2048 x 1000 product of the 1000-class layer: 18 against 21 us); the forward and
// weight-gradient forms of that size are not.
bool gemm_prefers_small(const GemmArgs &a);
bool gemm_fuses_softmax(int M, int N, int Kdim);
hipError_t launch_gemm_small(const GemmArgs &a, hipStream_t stream);

// Column sums out[n] = sum_m A(m,n) of a row-major [M][N] array; optional update.
hipError_t launch_colsum(const float *A, int M, int N, float *out,
                         float *update, float step, float *vel, float mu, hipStream_t stream);

// Softmax cross-entropy over rows; loss = mean; dlogits = (p - onehot)/B.  rowloss: B floats scratch.
// With partial != NULL the logits are first formed from split_k partial products [z][B][classes]
// plus bias (what the deferred split-K reduction would have written) and stored to `logits`.
hipError_t launch_softmax_ce(float *logits, const int *labels, int B, int classes, float *loss,
                             float *dlogits, float *rowloss, const float *partial, int split_k, const float *bias,
                             hipStream_t stream);

// prob[n][j] = softmax(logits[n][:])[j] with the row maximum subtracted (inference output).
hipError_t launch_softmax_prob(const float *logits, int B, int classes, float *prob, hipStream_t stream);

// CRBM visible statistics: dc[ch] = scale * sum(v0 - v1), mse = mean((v0-v1)^2); scratch: 2 * nblocks floats.
size_t visible_stats_scratch_floats(int N, int C, int HW);
hipError_t launch_visible_stats(const float *v0, const float *v1, int N, int C, int HW, float scale,
                                float *dc, float *mse, float *c_update, float step, float *scratch,
                                hipStream_t stream);

hipError_t launch_copy(const float *src, float *dst, size_t count, hipStream_t stream);

// Fully-connected RBM step, element-wise parts: Bernoulli states 1[u < p]; the two phases' hidden
// probabilities stacked as [scale * h0p; -scale * h1p] (2 * count floats); visible statistics
// dc[i] = scale * sum_n (v0 - v1)[n][i], mse = mean((v0 - v1)^2) with rbm_visible_scratch_floats(nv) floats of scratch.
hipError_t launch_bernoulli(const float *p, const float *u, float *states, size_t count, hipStream_t stream);
hipError_t launch_rbm_stack(const float *h0p, const float *h1p, float scale, float *stacked, size_t count, hipStream_t stream);
size_t rbm_visible_scratch_floats(int nv);
hipError_t launch_rbm_visible_stats(const float *v0, const float *v1, int B, int nv, float scale, float *dc, float *mse,
                                    float *c_update, float step, float *scratch, hipStream_t stream);

// ---------------------------------------------------------------------------------------
// Closing kernel of a training step: the reductions that nothing later in the step waits for
// (filter-gradient reductions with their updates, dense bias gradients, the mean loss) run as
// jobs of ONE launch instead of one tiny dependent kernel each.
// ---------------------------------------------------------------------------------------
struct StepTail {
  static constexpr int kMaxReduce = 8, kMaxColsum = 4;
  int n_reduce = 0, n_colsum = 0;
  struct Reduce { WgradReduceArgs a; WgradPlan plan; } reduce[kMaxReduce];
  struct Colsum { const float *A; int M, N; float *out, *update; float step; float *vel; float mu; } colsum[kMaxColsum];
  const float *rowloss = nullptr; int rows = 0; float *loss = nullptr;   // optional: *loss = mean(rowloss)
};
hipError_t launch_step_tail(const StepTail &t, hipStream_t stream);

}  // namespace dllk
