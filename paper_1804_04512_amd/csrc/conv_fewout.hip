// Forward-form convolution with very few output channels (Kout <= 3) on fp32 MFMA.
//
// The case: the CRBM's visible reconstruction (Section II: the full convolution of the hidden
// states with the filters, K hidden maps -> one or three visible maps) and the backward-data pass
// into a grey-scale or RGB input (Section II-A).  With output channels on the MFMA N axis, as in
// the general engine, 15 of 16 columns would multiply zeros.  Here the N axis carries 16
// neighbouring output COLUMNS instead, and the filter enters as a banded (Toeplitz) operand:
//   out[i, j0+jj] = sum_{c,r,t} win[c][i+r][t] * B[(c,r,t)][jj],   B[(c,r,t)][jj] = wgt[c][r][t-jj] (0 <= t-jj < S)
// with win the source window of the tile (16+R-1 rows, 16+S-1 columns, zero outside the image).
// M = 16 output rows, N = 16 output columns, K = (channel, filter row, window column): S of every
// 16+S-1 products are real, e.g. 9/24 for 9x9 filters instead of 1/16.  B fragments are read from
// the compact filter rows in LDS (each row padded with zeros on both sides), so the banded matrix
// is never stored.
//
// One workgroup = one 16x16 output tile of one image, all (<= 3) output channels.  Source
// channels are staged in rounds of kRch; inside a round each of the four wavefronts multiplies
// its own kRch/4 channels, and the four partial tiles are added in a fixed order at the end.
#include "dll_internal.h"

namespace dllk {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kRch = 8;            // source channels per staging round
constexpr int kRsx = 34;           // LDS row stride of the window: 2 mod 32 -> conflict-free A reads
constexpr int kSteps = 8;          // MFMA steps a window row can have (window <= 32 columns: S <= 17)
constexpr int kRoww = 15 + 4 * kSteps + 1;   // filter row: 15 zeros, the taps, zeros up to the last column a lane reads
constexpr int kStage = 4;          // staging loads per thread and batch

struct FewoutParams {
  ConvEngineArgs a;
  int tiles_x, tiles_y;
  int rows;        // window rows = 16 + R - 1
  int winp;        // window columns staged = 4 * wsteps >= 16 + S - 1
  int wsteps;
  int rounds;
};

__device__ __forceinline__ float act_apply(int act, float z) {
  if (act == ACT_SIGMOID) return 1.0f / (1.0f + expf(-z));
  if (act == ACT_RELU) return z > 0.0f ? z : 0.0f;
  return z;
}

template <int KO>
__global__ __launch_bounds__(kThreads) void conv_fewout_kernel(const FewoutParams p) {
  extern __shared__ float lds[];
  const ConvEngineArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int psx = p.rows * kRsx;
  float *xs = lds;                    // [kRch][rows][kRsx]
  float *wf = xs + kRch * psx;        // [KO][kRch][R][kRoww]
  const int bid = blockIdx.x;
  const int tx = bid % p.tiles_x, ty = (bid / p.tiles_x) % p.tiles_y, n = bid / (p.tiles_x * p.tiles_y);
  const int i0 = ty * 16, j0 = tx * 16;
  const int RSf = a.R * a.S;
  const bool need_y = a.src_dz && a.src_act != ACT_IDENTITY;

  // the zero borders of the filter rows are written once; the rounds rewrite the taps only
  for (int e = tid; e < KO * kRch * a.R * kRoww; e += kThreads) wf[e] = 0.0f;

  floatx4 acc[KO];
#pragma unroll
  for (int c = 0; c < KO; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};

  for (int round = 0; round < p.rounds; ++round) {
    const int c0 = round * kRch;
    __syncthreads();   // the previous round's readers are done (first round: the zero fill is complete)
    // Staging works in batches: all addresses, then all loads, unconditionally and from clamped
    // addresses (element 0 stands in for padding and for channels that do not exist), then the
    // selects and the LDS stores; a load behind a per-lane branch would be waited for on its own.
    // ---- filter taps of the round's channels: wf[c][cl][r][15 + s]
    {
      const int total = KO * kRch * RSf;
      for (int e0 = tid; e0 < total; e0 += kStage * kThreads) {
        float v[kStage];
        bool ok[kStage];
        int dst[kStage];
#pragma unroll
        for (int u = 0; u < kStage; ++u) {
          const int e = min(e0 + u * kThreads, total - 1);
          const int s = e % a.S, q = e / a.S;
          const int r = q % a.R, q2 = q / a.R;
          const int cl = q2 % kRch, c = q2 / kRch;
          const int ci = c0 + cl;
          ok[u] = ci < a.Cin;
          const int o = a.w_flip ? ((ci * a.Kout + c) * a.R + (a.R - 1 - r)) * a.S + (a.S - 1 - s)
                                 : ((c * a.Cin + ci) * a.R + r) * a.S + s;
          v[u] = a.w[ok[u] ? o : 0];
          dst[u] = ((c * kRch + cl) * a.R + r) * kRoww + 15 + s;
        }
#pragma unroll
        for (int u = 0; u < kStage; ++u)
          if (e0 + u * kThreads < total) wf[dst[u]] = ok[u] ? v[u] : 0.0f;
      }
    }
    // ---- source window of the round's channels: xs[cl][y][x] = srcpad(c0 + cl, i0 - pad + y, j0 - pad + x)
    {
      const int total = kRch * p.rows * p.winp;
      for (int e0 = tid; e0 < total; e0 += kStage * kThreads) {
        float gv[kStage], yv[kStage];
        bool ok[kStage];
        int dst[kStage];
#pragma unroll
        for (int u = 0; u < kStage; ++u) {
          const int e = min(e0 + u * kThreads, total - 1);
          const int x = e % p.winp, q = e / p.winp;
          const int y = q % p.rows, cl = q / p.rows;
          const int gi = i0 - a.pad_h + y, gj = j0 - a.pad_w + x, ci = c0 + cl;
          ok[u] = ci < a.Cin && gi >= 0 && gi < a.Hin && gj >= 0 && gj < a.Win;
          const int o = ok[u] ? ((n * a.Cin + ci) * a.Hin + gi) * a.Win + gj : 0;
          gv[u] = a.src[o];
          yv[u] = need_y ? a.src_y[o] : 0.0f;
          dst[u] = cl * psx + y * kRsx + x;
        }
#pragma unroll
        for (int u = 0; u < kStage; ++u) {
          if (e0 + u * kThreads >= total) continue;
          float v = gv[u];
          if (need_y) {   // dz = dy * act'(y), from the layer output
            if (a.src_act == ACT_SIGMOID) v *= yv[u] * (1.0f - yv[u]);
            else v = yv[u] > 0.0f ? v : 0.0f;
          }
          xs[dst[u]] = ok[u] ? v : 0.0f;
        }
      }
    }
    __syncthreads();
    // ---- MFMA over (channel, filter row) pairs of this wavefront's channels; the fragments of the
    // next pair are read from LDS while the current pair is multiplied.  A: lane (row i16, k = kq)
    // reads window column 4*step + kq of row i16 + r; B: lane (column i16, k = kq) reads tap
    // 4*step + kq - i16 of the padded filter row (zero outside the S taps).
    {
      constexpr int CPW = kRch / 4;   // channels per wavefront
      const int npairs = CPW * a.R;
      float afA[kSteps], afB[kSteps], bfA[KO][kSteps], bfB[KO][kSteps];
      auto load_pair = [&](int cc, int r, float (&af)[kSteps], float (&bf)[KO][kSteps]) __attribute__((always_inline)) {
        const int cl = wave * CPW + cc;
        const float *ap = xs + cl * psx + (i16 + r) * kRsx + kq;
#pragma unroll
        for (int st = 0; st < kSteps; ++st) af[st] = ap[4 * st];
#pragma unroll
        for (int c = 0; c < KO; ++c) {
          const float *bp = wf + ((c * kRch + cl) * a.R + r) * kRoww + 15 + kq - i16;
#pragma unroll
          for (int st = 0; st < kSteps; ++st) bf[c][st] = bp[4 * st];
        }
      };
      auto mfma_pair = [&](const float (&af)[kSteps], const float (&bf)[KO][kSteps]) __attribute__((always_inline)) {
#pragma unroll
        for (int st = 0; st < kSteps; ++st) {
          if (st < p.wsteps) {
#pragma unroll
            for (int c = 0; c < KO; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[st], bf[c][st], acc[c], 0, 0, 0);
          }
        }
      };
      int cc = 0, r = 0;   // the pair whose fragments are loaded next
      auto advance = [&]() __attribute__((always_inline)) {
        if (++r == a.R) { r = 0; ++cc; }
        if (cc == CPW) { cc = CPW - 1; r = a.R - 1; }   // past the end: re-read the last pair (not multiplied)
      };
      load_pair(cc, r, afA, bfA);
      advance();
      for (int t = 0; t < npairs; t += 2) {
        load_pair(cc, r, afB, bfB);
        advance();
        __builtin_amdgcn_sched_barrier(0);
        mfma_pair(afA, bfA);
        __builtin_amdgcn_sched_barrier(0);
        load_pair(cc, r, afA, bfA);
        advance();
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < npairs) mfma_pair(afB, bfB);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  // ---- the four wavefronts' partial tiles, added in wavefront order, then bias, activation, store.
  // Lane holds D[row 4*kq + v][column i16].
  __syncthreads();
  float *red = lds;   // [wave][KO][lane][4]
#pragma unroll
  for (int c = 0; c < KO; ++c)
    *reinterpret_cast<float4 *>(red + ((wave * KO + c) * 64 + lane) * 4) = make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int c = 0; c < KO; ++c) {
      float4 s = *reinterpret_cast<const float4 *>(red + ((0 * KO + c) * 64 + lane) * 4);
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        const float4 t = *reinterpret_cast<const float4 *>(red + ((w * KO + c) * 64 + lane) * 4);
        s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
      }
      const float bv = a.bias ? a.bias[c] : 0.0f;
      const float sv[4] = {s.x, s.y, s.z, s.w};
      const int oj = j0 + i16;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int oi = i0 + 4 * kq + v;
        if (oi < a.Hout && oj < a.Wout) a.out[((n * a.Kout + c) * a.Hout + oi) * a.Wout + oj] = act_apply(a.act, sv[v] + bv);
      }
    }
  }
}

size_t fewout_lds_bytes(const ConvEngineArgs &a, int rows) {
  const size_t stage = sizeof(float) * ((size_t)kRch * rows * kRsx + (size_t)a.Kout * kRch * a.R * kRoww);
  const size_t red = sizeof(float) * 4 * (size_t)a.Kout * 64 * 4;
  return stage > red ? stage : red;
}

}  // namespace

bool conv_fewout_applies(const ConvEngineArgs &a) {
  if (a.Kout > 3 || a.pool != 1 || a.sample || a.out_pool) return false;
  if (a.act != ACT_IDENTITY && a.act != ACT_SIGMOID && a.act != ACT_RELU) return false;
  if (a.src_dz && (a.src_pool != 1 || (a.src_act != ACT_IDENTITY && a.src_act != ACT_SIGMOID && a.src_act != ACT_RELU))) return false;
  if (16 + a.S - 1 > 4 * kSteps) return false;
  return fewout_lds_bytes(a, 16 + a.R - 1) <= 64 * 1024;
}

hipError_t launch_conv_fewout(const ConvEngineArgs &a, hipStream_t stream) {
  FewoutParams p;
  p.a = a;
  p.tiles_x = (a.Wout + 15) / 16;
  p.tiles_y = (a.Hout + 15) / 16;
  p.rows = 16 + a.R - 1;
  p.wsteps = (16 + a.S - 1 + 3) / 4;
  p.winp = 4 * p.wsteps;
  p.rounds = (a.Cin + kRch - 1) / kRch;
  const long blocks = (long)a.N * p.tiles_x * p.tiles_y;
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = fewout_lds_bytes(a, p.rows);
  const dim3 grid((unsigned)blocks);
  switch (a.Kout) {
    case 1: hipLaunchKernelGGL(conv_fewout_kernel<1>, grid, dim3(kThreads), lds, stream, p); break;
    case 2: hipLaunchKernelGGL(conv_fewout_kernel<2>, grid, dim3(kThreads), lds, stream, p); break;
    case 3: hipLaunchKernelGGL(conv_fewout_kernel<3>, grid, dim3(kThreads), lds, stream, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace dllk
