// Dense-layer matrix products on fp32 MFMA (v_mfma_f32_16x16x4_f32), gfx950.
//
// Section II-A of the paper: the forward pass of a fully-connected layer over a minibatch is
// one matrix product, the backward pass one with the transposed weights, the gradient one
// more.  A single kernel serves all three through element strides:
//   C(m,n) = sum_k A(m,k) * B(k,n),   A(m,k) = A[m*a_m + k*a_k],  B(k,n) = B[k*b_k + n*b_n]
// with an optional act'(.) factor on A (dzh = dh * act'(h)), bias + activation, split-K with
// a fixed-order second pass, and an optional in-place parameter update C_upd += step * C.
// Workgroup tile 64 x 64 x 32, four wavefronts of 32 x 32 each.
#include "dll_internal.h"

namespace dllk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int BM = 64, BN = 64, BK = 32;
constexpr int LDS_TILE = 64 * 80;   // floats per operand tile, covers both layouts (64*34 and 32*80)

struct GemmParams {
  GemmArgs a;
  int k_per_split;   // multiple of BK
};

__device__ __forceinline__ float act_apply(int act, float z) {
  if (act == ACT_SIGMOID) return 1.0f / (1.0f + expf(-z));
  if (act == ACT_RELU) return z > 0.0f ? z : 0.0f;
  return z;
}
__device__ __forceinline__ float act_deriv(int act, float out) {
  if (act == ACT_SIGMOID) return out * (1.0f - out);
  if (act == ACT_RELU) return out > 0.0f ? 1.0f : 0.0f;
  return 1.0f;
}

// Stage a 64 (x) by 32 (k) operand tile.  k-contiguous sources go to LDS as [x][34] (lanes
// run along k), x-contiguous ones as [k][80] (lanes run along x): both are conflict-free for
// the staging writes and for the MFMA operand reads.
__device__ __forceinline__ void stage_tile(float *dst, const float *src, const float *src_out, int act,
                                           long sx, long sk, int x0, int k0, int X, int Kend, bool kcontig) {
  const int tid = threadIdx.x;
  if (kcontig) {
    const int k = tid & 31, xb = tid >> 5;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int x = xb + it * 8;
      float v = 0.0f;
      if (x0 + x < X && k0 + k < Kend) {
        const long o = (long)(x0 + x) * sx + (long)(k0 + k) * sk;
        v = src[o];
        if (src_out) v *= act_deriv(act, src_out[o]);
      }
      dst[x * 34 + k] = v;
    }
  } else {
    const int x = tid & 63, kb = tid >> 6;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int k = kb + it * 4;
      float v = 0.0f;
      if (x0 + x < X && k0 + k < Kend) {
        const long o = (long)(x0 + x) * sx + (long)(k0 + k) * sk;
        v = src[o];
        if (src_out) v *= act_deriv(act, src_out[o]);
      }
      dst[k * 80 + x] = v;
    }
  }
}

__global__ __launch_bounds__(kThreads) void gemm_kernel(const GemmParams p) {
  __shared__ float As[LDS_TILE];
  __shared__ float Bs[LDS_TILE];
  const GemmArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int kbeg = blockIdx.z * p.k_per_split;
  const int kend = min(a.Kdim, kbeg + p.k_per_split);
  const bool a_kc = (a.a_k == 1), b_kc = (a.b_k == 1);
  const int alx = a_kc ? 34 : 1, alk = a_kc ? 1 : 80;
  const int blx = b_kc ? 34 : 1, blk = b_kc ? 1 : 80;
  const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;

  floatx4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  for (int k0 = kbeg; k0 < kend; k0 += BK) {
    __syncthreads();
    stage_tile(As, a.A, a.A_out, a.a_act, a.a_m, a.a_k, m0, k0, a.M, kend, a_kc);
    stage_tile(Bs, a.B, nullptr, 0, a.b_n, a.b_k, n0, k0, a.N, kend, b_kc);
    __syncthreads();
#pragma unroll
    for (int s = 0; s < BK / 4; ++s) {
      float af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) af[i] = As[(wm + i * 16 + i16) * alx + (4 * s + kq) * alk];
#pragma unroll
      for (int j = 0; j < 2; ++j) bf[j] = Bs[(wn + j * 16 + i16) * blx + (4 * s + kq) * blk];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
  }

  // lane holds C(m = 4*kq + v, n = i16) of each 16x16 tile
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + wn + j * 16 + i16;
      if (n >= a.N) continue;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int m = m0 + wm + i * 16 + 4 * kq + v;
        if (m >= a.M) continue;
        float c = acc[i][j][v];
        if (a.split_k > 1) {
          a.partial[((long)blockIdx.z * a.M + m) * a.N + n] = c;
        } else {
          if (a.bias) c += a.bias[n];
          c = act_apply(a.act, c);
          const long o = (long)m * a.c_m + (long)n * a.c_n;
          if (a.Cout) a.Cout[o] = c;
          if (a.update) a.update[o] += a.step * c;
        }
      }
    }
}

__global__ __launch_bounds__(kThreads) void gemm_splitk_reduce_kernel(const GemmArgs a) {
  const long total = (long)a.M * a.N;
  for (long e = (long)blockIdx.x * kThreads + threadIdx.x; e < total; e += (long)gridDim.x * kThreads) {
    const int m = (int)(e / a.N), n = (int)(e - (long)m * a.N);
    float c = 0.0f;
    for (int z = 0; z < a.split_k; ++z) c += a.partial[(long)z * total + e];
    if (a.bias) c += a.bias[n];
    c = act_apply(a.act, c);
    const long o = (long)m * a.c_m + (long)n * a.c_n;
    if (a.Cout) a.Cout[o] = c;
    if (a.update) a.update[o] += a.step * c;
  }
}

// out[n] = sum_m A[m][n] * act'(Aout[m][n]);  one thread per column, fixed order.
__global__ __launch_bounds__(kThreads) void colsum_kernel(const float *A, const float *A_out, int act, int M, int N,
                                                         float *out, float *update, float step) {
  const int n = blockIdx.x * kThreads + threadIdx.x;
  if (n >= N) return;
  float s = 0.0f;
  for (int m = 0; m < M; ++m) {
    float v = A[(long)m * N + n];
    if (A_out) v *= act_deriv(act, A_out[(long)m * N + n]);
    s += v;
  }
  if (out) out[n] = s;
  if (update) update[n] += step * s;
}

__device__ __forceinline__ float block_reduce(float v, float *sh, bool is_max) {
  const int tid = threadIdx.x;
  sh[tid] = v;
  __syncthreads();
  for (int s = kThreads / 2; s > 0; s >>= 1) {
    if (tid < s) sh[tid] = is_max ? fmaxf(sh[tid], sh[tid + s]) : sh[tid] + sh[tid + s];
    __syncthreads();
  }
  const float r = sh[0];
  __syncthreads();
  return r;
}

// One workgroup per sample: p = softmax(logits) with the row maximum subtracted,
// rowloss = -ln p[label], dlogits = (p - onehot) / B.
__global__ __launch_bounds__(kThreads) void softmax_ce_kernel(const float *logits, const int *labels, int B, int classes,
                                                             float *dlogits, float *rowloss) {
  __shared__ float sh[kThreads];
  const int n = blockIdx.x, tid = threadIdx.x;
  const float *row = logits + (long)n * classes;
  float m = -INFINITY;
  for (int j = tid; j < classes; j += kThreads) m = fmaxf(m, row[j]);
  m = block_reduce(m, sh, true);
  float s = 0.0f;
  for (int j = tid; j < classes; j += kThreads) s += expf(row[j] - m);
  s = block_reduce(s, sh, false);
  const int label = labels[n];
  const float inv = 1.0f / s, invB = 1.0f / (float)B;
  for (int j = tid; j < classes; j += kThreads) {
    const float pj = expf(row[j] - m) * inv;
    dlogits[(long)n * classes + j] = (pj - (j == label ? 1.0f : 0.0f)) * invB;
  }
  if (tid == 0) rowloss[n] = -(row[label] - m - logf(s));
}

__global__ __launch_bounds__(kThreads) void mean_kernel(const float *v, int count, float *out) {
  __shared__ float sh[kThreads];
  float s = 0.0f;
  for (int j = threadIdx.x; j < count; j += kThreads) s += v[j];
  s = block_reduce(s, sh, false);
  if (threadIdx.x == 0) *out = s / (float)count;
}

constexpr int kStatBlocks = 32;

// scratch[ch][b] = sum over the block's slice of (v0 - v1); scratch[C*32 + ch*32 + b] = sum of squares
__global__ __launch_bounds__(kThreads) void visible_stats_kernel(const float *v0, const float *v1, int N, int C, int HW,
                                                                float *scratch) {
  __shared__ float sh[kThreads];
  const int ch = blockIdx.y, b = blockIdx.x;
  const long per = (long)N * HW;
  float s = 0.0f, q = 0.0f;
  for (long e = (long)b * kThreads + threadIdx.x; e < per; e += (long)kStatBlocks * kThreads) {
    const long nn = e / HW, r = e - nn * HW;
    const long o = (nn * C + ch) * HW + r;
    const float d = v0[o] - v1[o];
    s += d;
    q += d * d;
  }
  s = block_reduce(s, sh, false);
  q = block_reduce(q, sh, false);
  if (threadIdx.x == 0) {
    scratch[ch * kStatBlocks + b] = s;
    scratch[(C + ch) * kStatBlocks + b] = q;
  }
}

__global__ void visible_stats_final_kernel(const float *scratch, int N, int C, int HW, float scale, float *dc, float *mse,
                                           float *c_update, float step) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double sq = 0.0;
  for (int ch = 0; ch < C; ++ch) {
    double s = 0.0;
    for (int b = 0; b < kStatBlocks; ++b) {
      s += (double)scratch[ch * kStatBlocks + b];
      sq += (double)scratch[(C + ch) * kStatBlocks + b];
    }
    const float g = (float)(s * (double)scale);
    if (dc) dc[ch] = g;
    if (c_update) c_update[ch] += step * g;
  }
  if (mse) *mse = (float)(sq / ((double)N * C * HW));
}

__global__ __launch_bounds__(kThreads) void copy_kernel(const float *src, float *dst, size_t count) {
  for (size_t e = (size_t)blockIdx.x * kThreads + threadIdx.x; e < count; e += (size_t)gridDim.x * kThreads) dst[e] = src[e];
}

}  // namespace

int gemm_pick_split_k(int M, int N, int Kdim) {
  const long tiles = (long)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const int ksteps = (Kdim + BK - 1) / BK;
  int split = 1;
  while (tiles * split < 512 && split * 2 <= ksteps && split < 64) split *= 2;
  return split;
}

hipError_t launch_gemm(const GemmArgs &a, hipStream_t stream) {
  GemmParams p;
  p.a = a;
  if (p.a.split_k < 1) p.a.split_k = 1;
  const int ksteps = (a.Kdim + BK - 1) / BK;
  p.k_per_split = ((ksteps + p.a.split_k - 1) / p.a.split_k) * BK;
  dim3 grid((a.N + BN - 1) / BN, (a.M + BM - 1) / BM, p.a.split_k);
  hipLaunchKernelGGL(gemm_kernel, grid, dim3(kThreads), 0, stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (p.a.split_k > 1) {
    const long total = (long)a.M * a.N;
    long blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(gemm_splitk_reduce_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, p.a);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_colsum(const float *A, const float *A_out, int a_act, int M, int N, float *out, float *update,
                         float step, hipStream_t stream) {
  hipLaunchKernelGGL(colsum_kernel, dim3((N + kThreads - 1) / kThreads), dim3(kThreads), 0, stream, A, A_out, a_act, M, N,
                     out, update, step);
  return hipGetLastError();
}

hipError_t launch_softmax_ce(const float *logits, const int *labels, int B, int classes, float *loss, float *dlogits,
                             float *rowloss, hipStream_t stream) {
  hipLaunchKernelGGL(softmax_ce_kernel, dim3(B), dim3(kThreads), 0, stream, logits, labels, B, classes, dlogits, rowloss);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(kThreads), 0, stream, rowloss, B, loss);
  return hipGetLastError();
}

size_t visible_stats_scratch_floats(int, int C, int) { return (size_t)2 * C * kStatBlocks; }

hipError_t launch_visible_stats(const float *v0, const float *v1, int N, int C, int HW, float scale, float *dc, float *mse,
                                float *c_update, float step, float *scratch, hipStream_t stream) {
  hipLaunchKernelGGL(visible_stats_kernel, dim3(kStatBlocks, C), dim3(kThreads), 0, stream, v0, v1, N, C, HW, scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(visible_stats_final_kernel, dim3(1), dim3(64), 0, stream, scratch, N, C, HW, scale, dc, mse, c_update,
                     step);
  return hipGetLastError();
}

hipError_t launch_copy(const float *src, float *dst, size_t count, hipStream_t stream) {
  size_t blocks = (count + kThreads - 1) / kThreads;
  if (blocks > 4096) blocks = 4096;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, src, dst, count);
  return hipGetLastError();
}

}  // namespace dllk
