// Element-wise companions of the fully-connected RBM's CD-1 step (Section II: RBM trained with
// Contrastive Divergence); the matrix products themselves run in the GEMM kernels.
#include "dll_internal.h"
#include "small_bodies.h"

namespace dllk {
namespace {

constexpr int kThreads = 256;

// states[e] = 1[u[e] < p[e]]
__global__ __launch_bounds__(kThreads) void bernoulli_kernel(const float *p, const float *u, float *states, size_t count) {
  for (size_t e = (size_t)blockIdx.x * kThreads + threadIdx.x; e < count; e += (size_t)gridDim.x * kThreads)
    states[e] = u[e] < p[e] ? 1.0f : 0.0f;
}

// The two phases' hidden probabilities stacked along the batch axis with the step's signs and
// its 1/B folded in, so that ONE product over 2B rows yields (positive - negative) / B:
//   stacked[n][j] = scale * h0p[n][j],  stacked[B + n][j] = -scale * h1p[n][j]
__global__ __launch_bounds__(kThreads) void rbm_stack_kernel(const float *h0p, const float *h1p, float scale, float *stacked,
                                                            size_t count) {
  for (size_t e = (size_t)blockIdx.x * kThreads + threadIdx.x; e < count; e += (size_t)gridDim.x * kThreads) {
    stacked[e] = scale * h0p[e];
    stacked[count + e] = -scale * h1p[e];
  }
}

// 32 visible units per workgroup, 8 row slices each: dc[i] = scale * sum_n (v0 - v1)[n][i] (slices
// added in a fixed order, so the result does not depend on the launch), the optional bias update,
// and the workgroup's sum of squared differences.
constexpr int kVisCols = 32, kVisSlices = kThreads / kVisCols;
__global__ __launch_bounds__(kThreads) void rbm_visible_kernel(const float *v0, const float *v1, int B, int nv, float scale,
                                                              float *dc, float *c_update, float step, float *sq_partial) {
  __shared__ float sh[kThreads];
  __shared__ float part[kVisSlices][kVisCols + 1];
  const int col = threadIdx.x % kVisCols, slice = threadIdx.x / kVisCols;
  const int i = blockIdx.x * kVisCols + col;
  float s = 0.0f, q = 0.0f;
  if (i < nv) {
    for (int n = slice; n < B; n += kVisSlices) {
      const float d = v0[(size_t)n * nv + i] - v1[(size_t)n * nv + i];
      s += d;
      q += d * d;
    }
  }
  part[slice][col] = s;
  __syncthreads();
  if (slice == 0 && i < nv) {
    float t = 0.0f;
#pragma unroll
    for (int k = 0; k < kVisSlices; ++k) t += part[k][col];
    const float g = scale * t;
    if (dc) dc[i] = g;
    if (c_update) c_update[i] += step * g;
  }
  q = block_reduce(q, sh, false);
  if (threadIdx.x == 0) sq_partial[blockIdx.x] = q;
}

__global__ void rbm_mse_kernel(const float *sq_partial, int blocks, double count, float *mse) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double s = 0.0;
  for (int b = 0; b < blocks; ++b) s += (double)sq_partial[b];
  *mse = (float)(s / count);
}

unsigned grid_for(size_t count) {
  size_t blocks = (count + kThreads - 1) / kThreads;
  return (unsigned)(blocks > 4096 ? 4096 : blocks);
}

}  // namespace

hipError_t launch_bernoulli(const float *p, const float *u, float *states, size_t count, hipStream_t stream) {
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(bernoulli_kernel, dim3(grid_for(count)), dim3(kThreads), 0, stream, p, u, states, count);
  return hipGetLastError();
}

hipError_t launch_rbm_stack(const float *h0p, const float *h1p, float scale, float *stacked, size_t count,
                            hipStream_t stream) {
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(rbm_stack_kernel, dim3(grid_for(count)), dim3(kThreads), 0, stream, h0p, h1p, scale, stacked, count);
  return hipGetLastError();
}

size_t rbm_visible_scratch_floats(int nv) { return (size_t)(nv + kVisCols - 1) / kVisCols; }

hipError_t launch_rbm_visible_stats(const float *v0, const float *v1, int B, int nv, float scale, float *dc, float *mse,
                                    float *c_update, float step, float *scratch, hipStream_t stream) {
  const int blocks = (nv + kVisCols - 1) / kVisCols;
  hipLaunchKernelGGL(rbm_visible_kernel, dim3(blocks), dim3(kThreads), 0, stream, v0, v1, B, nv, scale, dc, c_update, step,
                     scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !mse) return e;
  hipLaunchKernelGGL(rbm_mse_kernel, dim3(1), dim3(64), 0, stream, scratch, blocks, (double)B * nv, mse);
  return hipGetLastError();
}

}  // namespace dllk
