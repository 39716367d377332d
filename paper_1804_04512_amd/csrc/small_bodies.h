// Bodies of the small reduction kernels, shared by their stand-alone launches (gemm.hip) and by
// the training step's closing kernel (conv_wgrad.hip), which runs all of a step's deferred
// reductions in one launch.  One workgroup of 256 threads per call; `blk` is the workgroup's
// index inside its job.
#pragma once

#include "dll_internal.h"

namespace dllk {

constexpr int kSmallThreads = 256;
constexpr int kColsumCols = 16, kColsumSlices = kSmallThreads / kColsumCols;

// out[n] = sum_m A[m][n]: 16 columns per workgroup, 16 row slices added in a fixed order
// (small inputs: many short independent load chains beat few long ones).
__device__ __forceinline__ void colsum_block(const float *A, int M, int N, float *out, float *update, float step, float *vel,
                                             float mu, int blk) {
  __shared__ float part[kColsumSlices][kColsumCols + 1];
  const int col = threadIdx.x % kColsumCols, slice = threadIdx.x / kColsumCols;
  const int n = blk * kColsumCols + col;
  float s = 0.0f;
  if (n < N) {
#pragma unroll 4
    for (int m = slice; m < M; m += kColsumSlices) s += A[(long)m * N + n];
  }
  part[slice][col] = s;
  __syncthreads();
  if (slice == 0 && n < N) {
    float q[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      q[g] = 0.0f;
#pragma unroll
      for (int i = 0; i < kColsumSlices / 4; ++i) q[g] += part[g * (kColsumSlices / 4) + i][col];
    }
    s = (q[0] + q[1]) + (q[2] + q[3]);
    if (out) out[n] = s;
    if (update) update_param(update + n, vel ? vel + n : nullptr, s, step, mu, 0.0f);
  }
}

// Sum or maximum over the workgroup's 256 threads, the same value in every thread: lane exchanges
// inside a wavefront (a butterfly, so every lane adds the same pairs in the same order), then the
// four wavefronts' results in wavefront order.  Two barriers instead of the nine of a tree in LDS,
// which were most of what the small row kernels spent.  sh: at least 4 floats, free again on return.
__device__ __forceinline__ float block_reduce(float v, float *sh, bool is_max) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float w = __shfl_xor(v, o);
    v = is_max ? fmaxf(v, w) : v + w;
  }
  const int tid = threadIdx.x;
  if ((tid & 63) == 0) sh[tid >> 6] = v;
  __syncthreads();
  float r = sh[0];
#pragma unroll
  for (int w = 1; w < kSmallThreads / 64; ++w) r = is_max ? fmaxf(r, sh[w]) : r + sh[w];
  __syncthreads();
  return r;
}

// *out = mean of v[0 .. count)
__device__ __forceinline__ void mean_block(const float *v, int count, float *out) {
  __shared__ float sh[kSmallThreads];
  float s = 0.0f;
  for (int j = threadIdx.x; j < count; j += kSmallThreads) s += v[j];
  s = block_reduce(s, sh, false);
  if (threadIdx.x == 0) *out = s / (float)count;
}

}  // namespace dllk
