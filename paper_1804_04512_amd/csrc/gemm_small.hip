// fp32 MFMA matrix product for SMALL problems: the dense layers of the paper's MNIST and CIFAR
// networks and of the fully-connected RBM (Sections II-A, IV, V: a few hundred units, batch 100).
//
// Such a product cannot fill the chip; what it costs is a chain of latencies (launch, first
// loads, one LDS round trip and one barrier per k-tile, a split-K reduction launch).  This kernel
// shortens the chain instead of raising the rate:
//   * 32 x 32 or, for the smallest products, 16 x 16 output tile per workgroup (many more workgroups
//     than the 128 x 64 tiles of the big kernel, far fewer products with padding);
//   * the four wavefronts split the k range BETWEEN them and each multiplies the whole tile, so
//     there is no LDS staging and no barrier inside the k loop at all: every lane loads its
//     MFMA fragments straight from global memory, the next three k-tiles' loads in flight while
//     the current one is multiplied.  Inside a k-tile of 32, the lane with k-quarter kq owns the 8
//     consecutive k values 8*kq .. 8*kq+7 of both operands (any assignment works as long as both
//     operands use the same one), which makes a k-contiguous operand two 16-byte loads per row;
//   * the partial tiles meet in LDS once, are added in wavefront order (results do not depend
//     on timing), and one wavefront per 16 x 16 quarter of the tile finishes it: bias, activation,
//     act' of a reference tensor, store and/or fused parameter update.  No split-K partials in
//     global memory, no reduction launch.
// Every global load is issued unconditionally from a clamped address; nothing is masked before
// the multiplication needs it.
#include "dll_internal.h"

namespace dllk {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int KT = 32;    // k-tile

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

struct SmallParams {
  GemmArgs a;
  int a_vec, b_vec;   // k-contiguous operand with aligned rows of whole 16-byte groups
};

// One operand's fragments of a k-tile: frag[t][s] = X(x0 + 16 t + i16, k0 + 8 kq + s), X(x, k) = src[x * sx + k * sk].
// Nothing here depends on a loaded value, so all loads of a k-tile stay in flight until the
// multiplication needs them.  Rows past the operand's end re-read its last row: they only feed
// output rows/columns that are never stored.  A k past the end re-reads k = 0 (a finite value);
// `zero_tail` (uniform; set for ONE operand of the k-tile that overhangs Kdim) then clears those
// entries, so that their products vanish.
template <bool KC, int Q>
__device__ __forceinline__ void load_frags(float (&frag)[Q][8], const float *src, long sx, long sk, int x0, int X, int k0,
                                           int Kdim, int i16, int kq, bool vec, bool zero_tail) {
  const int k = k0 + 8 * kq;
#pragma unroll
  for (int t = 0; t < Q; ++t) {
    const long base = (long)min(x0 + 16 * t + i16, X - 1) * sx;
    if (KC && vec) {   // uniform: rows are whole aligned 16-byte groups, so a group is entirely in or out of range
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int kk = k + 4 * h;
        const float4 v = *reinterpret_cast<const float4 *>(src + base + (kk < Kdim ? kk : 0));
        frag[t][4 * h + 0] = v.x; frag[t][4 * h + 1] = v.y; frag[t][4 * h + 2] = v.z; frag[t][4 * h + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int s = 0; s < 8; ++s) frag[t][s] = src[base + (long)(k + s < Kdim ? k + s : 0) * sk];
    }
  }
  if (zero_tail) {
#pragma unroll
    for (int t = 0; t < Q; ++t)
#pragma unroll
      for (int s = 0; s < 8; ++s)
        if (k + s >= Kdim) frag[t][s] = 0.0f;
  }
}

// Q = 2: 32 x 32 tile (four 16 x 16 quarters); Q = 1: 16 x 16 tile, for products whose 32 x 32 tiles
// would occupy a small part of the chip with long k loops
template <bool A_KC, bool B_KC, int WAVES, int Q>
__global__ __launch_bounds__(WAVES * 64) void gemm_small_kernel(const SmallParams p) {
  constexpr int TS = 16 * Q;
  __shared__ __attribute__((aligned(16))) float red[WAVES][Q * Q][64][4];   // [wavefront][quarter][lane][4]
  const GemmArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
  const int nkt = (a.Kdim + KT - 1) / KT;

  floatx4 acc[Q][Q];   // [m quarter][n quarter]; lane holds C(m = i16, n = 4 kq + v)
#pragma unroll
  for (int i = 0; i < Q; ++i)
#pragma unroll
    for (int j = 0; j < Q; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  float afA[Q][8], bfA[Q][8], afB[Q][8], bfB[Q][8], afC[Q][8], bfC[Q][8], afD[Q][8], bfD[Q][8];
  auto load_tile = [&](int kt, float (&af)[Q][8], float (&bf)[Q][8]) __attribute__((always_inline)) {
    load_frags<A_KC, Q>(af, a.A, a.a_m, a.a_k, m0, a.M, kt * KT, a.Kdim, i16, kq, p.a_vec != 0, false);
    load_frags<B_KC, Q>(bf, a.B, a.b_n, a.b_k, n0, a.N, kt * KT, a.Kdim, i16, kq, p.b_vec != 0, kt * KT + KT > a.Kdim);
  };
  auto multiply = [&](const float (&af)[Q][8], const float (&bf)[Q][8]) __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int i = 0; i < Q; ++i)
#pragma unroll
        for (int j = 0; j < Q; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(bf[j][s], af[i][s], acc[i][j], 0, 0, 0);
  };
  // this wavefront's k-tiles: wave, wave + WAVES, ...; four register sets, so that three k-tiles'
  // loads are in flight while one is multiplied: with a handful of workgroups on the whole chip
  // (a batch-by-64 product over a long k) the loop runs at memory latency divided by that depth
  if (wave < nkt) {
    // (uniform conditions: a wavefront with one k-tile issues one k-tile's loads)
    load_tile(wave, afA, bfA);
    if (wave + WAVES < nkt) load_tile(wave + WAVES, afB, bfB);
    if (wave + 2 * WAVES < nkt) load_tile(wave + 2 * WAVES, afC, bfC);
    for (int kt = wave; kt < nkt; kt += 4 * WAVES) {
      if (kt + 3 * WAVES < nkt) load_tile(kt + 3 * WAVES, afD, bfD);
      __builtin_amdgcn_sched_barrier(0);
      multiply(afA, bfA);
      __builtin_amdgcn_sched_barrier(0);
      if (kt + 4 * WAVES < nkt) load_tile(kt + 4 * WAVES, afA, bfA);
      __builtin_amdgcn_sched_barrier(0);
      if (kt + WAVES < nkt) multiply(afB, bfB);
      __builtin_amdgcn_sched_barrier(0);
      if (kt + 5 * WAVES < nkt) load_tile(kt + 5 * WAVES, afB, bfB);
      __builtin_amdgcn_sched_barrier(0);
      if (kt + 2 * WAVES < nkt) multiply(afC, bfC);
      __builtin_amdgcn_sched_barrier(0);
      if (kt + 6 * WAVES < nkt) load_tile(kt + 6 * WAVES, afC, bfC);
      __builtin_amdgcn_sched_barrier(0);
      if (kt + 3 * WAVES < nkt) multiply(afD, bfD);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- the partial tiles meet in LDS
#pragma unroll
  for (int i = 0; i < Q; ++i)
#pragma unroll
    for (int j = 0; j < Q; ++j)
      *reinterpret_cast<float4 *>(&red[wave][Q * i + j][lane][0]) = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
  __syncthreads();
  if (wave >= Q * Q) return;
  // ---- wavefront w < Q * Q finishes quarter w: rows m0 + 16 (w / Q) .., columns n0 + 16 (w % Q) ..
  const int m = m0 + 16 * (wave / Q) + i16, n = n0 + 16 * (wave % Q) + 4 * kq;
  float c[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int w = 0; w < WAVES; ++w) {   // wavefront order, whatever finished first
    const float4 t = *reinterpret_cast<const float4 *>(&red[w][wave][lane][0]);
    c[0] += t.x; c[1] += t.y; c[2] += t.z; c[3] += t.w;
  }
  // everything the epilogue reads, in one batch of clamped loads
  const bool min_ = m < a.M;
  bool ok[4];
  long o[4];
  float bv[4], rv[4], uv[4], vv[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    ok[v] = min_ && n + v < a.N;
    o[v] = ok[v] ? (long)m * a.c_m + (long)(n + v) * a.c_n : 0;
    bv[v] = a.bias ? a.bias[n + v < a.N ? n + v : 0] : 0.0f;
    rv[v] = a.C_ref ? a.C_ref[o[v]] : 0.0f;
    uv[v] = a.update ? a.update[o[v]] : 0.0f;
    vv[v] = a.vel ? a.vel[o[v]] : 0.0f;
  }
  if (Q == 1 && a.sm_labels) {
    // Softmax + cross-entropy on the finished logits: a row's 16 columns sit in the four lanes
    // i16, i16 + 16, i16 + 32, i16 + 48 (four columns each), so two exchanges complete a row.
    // Columns past N count as -inf / 0; rows past M compute on clamped data and store nothing.
    const int label = a.sm_labels[min(m, a.M - 1)];
    float z[4], mx = -INFINITY;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      z[v] = c[v] + bv[v];
      if (n + v < a.N) mx = fmaxf(mx, z[v]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float e[4], sum = 0.0f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      e[v] = n + v < a.N ? expf(z[v] - mx) : 0.0f;
      sum += e[v];
    }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      if (!ok[v]) continue;
      if (a.Cout) a.Cout[o[v]] = z[v];
      a.sm_dz[o[v]] = (e[v] * inv - (n + v == label ? 1.0f : 0.0f)) * a.sm_scale;
      if (n + v == label) a.sm_rowloss[m] = -(z[v] - mx - logf(sum));
    }
    return;
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    c[v] = act_apply(a.act, c[v] + bv[v]);
    if (a.C_ref) c[v] *= act_deriv(a.c_ref_act, rv[v]);
    if (!ok[v]) continue;
    if (a.Cout) a.Cout[o[v]] = c[v];
    if (a.update) {
      update_param(&uv[v], a.vel ? &vv[v] : nullptr, c[v], a.step, a.mu, a.decay);
      a.update[o[v]] = uv[v];
      if (a.vel) a.vel[o[v]] = vv[v];
    }
  }
}

}  // namespace

// Products below this many multiply-adds run here; above it the chip can be filled and the
// persistent kernel's rate matters more than the latency chain.
bool gemm_is_small(int M, int N, int Kdim) { return (long)M * N * Kdim <= (1L << 27); }

bool gemm_prefers_small(const GemmArgs &a) {
  if (gemm_is_small(a.M, a.N, a.Kdim)) return true;
  return a.a_k == 1 && a.b_n == 1 && !a.update && !a.sm_labels && (long)a.M * a.N * a.Kdim <= (1L << 28);
}

// Tiles of 16 x 16 (the launcher's choice below for this size) hold whole rows of up to 16 logits.
bool gemm_fuses_softmax(int M, int N, int Kdim) { return gemm_is_small(M, N, Kdim) && N <= 16 && (M + 31) / 32 <= 512; }

hipError_t launch_gemm_small(const GemmArgs &a, hipStream_t stream) {
  if (a.sm_labels && (!gemm_fuses_softmax(a.M, a.N, a.Kdim) || !a.sm_dz || !a.sm_rowloss || a.act != ACT_IDENTITY || a.update ||
                      a.C_ref))
    return hipErrorInvalidValue;
  SmallParams p;
  p.a = a;
  p.a.split_k = 1;
  auto al16 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
  const bool a_kc = a.a_k == 1, b_kc = a.b_k == 1;
  p.a_vec = a_kc && al16(a.A) && a.a_m % 4 == 0 && a.Kdim % 4 == 0;
  p.b_vec = b_kc && al16(a.B) && a.b_n % 4 == 0 && a.Kdim % 4 == 0;
  // 16 x 16 tiles while 32 x 32 ones would number at most two per CU: four times the workgroups, a
  // quarter of the multiplications per wavefront (measured faster for every product of the small
  // workloads, whatever its k)
  const long tiles32 = (long)((a.N + 31) / 32) * ((a.M + 31) / 32);
  const bool fine = tiles32 <= 512;
  const int TS = fine ? 16 : 32;
  const dim3 grid((a.N + TS - 1) / TS, (a.M + TS - 1) / TS);
  // (eight wavefronts per workgroup, sharing the k range in eighths, measured slower at every size tried)
#define DLL_SMALL(AK, BK_)                                                                                         \
  do {                                                                                                             \
    if (fine) hipLaunchKernelGGL((gemm_small_kernel<AK, BK_, 4, 1>), grid, dim3(256), 0, stream, p);               \
    else hipLaunchKernelGGL((gemm_small_kernel<AK, BK_, 4, 2>), grid, dim3(256), 0, stream, p);                    \
  } while (0)
  if (a_kc && b_kc) DLL_SMALL(true, true);
  else if (a_kc) DLL_SMALL(true, false);
  else if (b_kc) DLL_SMALL(false, true);
  else DLL_SMALL(false, false);
#undef DLL_SMALL
  return hipGetLastError();
}

}  // namespace dllk
