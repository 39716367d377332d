// Filter gradient of a convolution layer on fp32 MFMA (v_mfma_f32_16x16x4_f32), gfx950.
//
//   dw[k,c,r,s] = sum_{n,i,j} dz[n,k,i,j] * xpad[n,c,i+r,j+s],   db[k] = sum_{n,i,j} dz[n,k,i,j]
//
// The contraction runs over pixels, so pixels sit on the MFMA K axis (4 neighbouring
// columns per instruction), filters on M and the (channel, tap) pairs of a channel chunk on
// N.  A workgroup walks over image tiles of 32 x TH output pixels: it stages the halo tile of
// x and the tile of dz = unpool(dy) * act'(y) (formed on the fly, never stored in HBM) in LDS
// and keeps its K x taps partial sums in accumulator registers across all its tiles.  Every
// wavefront finally writes its partial block; a second kernel adds the blocks in a fixed
// order (no float atomics: the result is bit-identical from run to run) and can apply the
// parameter update in the same pass.
#include "dll_internal.h"

namespace dllk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kTileW = 32;

struct WgradParams {
  WgradArgs a;
  int Ho, Wo;
  int CC, nchunks, G;
  int rows, cols, RS, PS;  // x halo tile in LDS
  int PSZ;                 // dz plane stride in LDS (row stride is 32)
  int tiles_x, tiles_y, items;
  int kgroups;
  long db_offset;
  long group_stride;       // floats between filter groups in the dw partial area
};

__device__ __forceinline__ float dz_value(const WgradArgs &a, int Ho, int Wo, int n, int k, int i, int j) {
  int o;
  if (a.pool == 2) {
    o = ((n * a.K + k) * (Ho >> 1) + (i >> 1)) * (Wo >> 1) + (j >> 1);
    if (a.idx[o] != (unsigned char)(((i & 1) << 1) | (j & 1))) return 0.0f;
  } else {
    o = ((n * a.K + k) * Ho + i) * Wo + j;
  }
  float g = a.dy[o];
  if (a.act == ACT_SIGMOID) {
    const float v = a.y[o];
    g *= v * (1.0f - v);
  } else if (a.act == ACT_RELU) {
    if (!(a.y[o] > 0.0f)) g = 0.0f;
  }
  return g;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// grid: x = G * nchunks, y = filter groups of MTF*16
template <int MTF, int NTT, int TH>
__global__ __launch_bounds__(kThreads) void wgrad_kernel(const WgradParams p) {
  extern __shared__ float lds[];
  const WgradArgs &a = p.a;
  float *xs = lds;                 // [CC][PS]
  float *dzs = xs + p.CC * p.PS;   // [MTF*16 (clipped to K)][PSZ]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int gidx = blockIdx.x % p.G, chunk = blockIdx.x / p.G;
  const int k0 = blockIdx.y * (MTF * 16);
  const int kcount = min(MTF * 16, a.K - k0);   // filters this group really has
  const int c0 = chunk * p.CC;
  const int RSf = a.R * a.S;
  constexpr int PLANE = TH * kTileW;
  constexpr int ITS_PER_K = PLANE / kThreads;   // staging iterations per filter plane
  constexpr int RW = TH / 4;                    // rows per wave

  floatx4 acc[MTF][NTT];
#pragma unroll
  for (int mf = 0; mf < MTF; ++mf)
#pragma unroll
    for (int nt = 0; nt < NTT; ++nt) acc[mf][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  float dbacc[MTF * 16];
#pragma unroll
  for (int k = 0; k < MTF * 16; ++k) dbacc[k] = 0.0f;

  // B operand: lane's tap of N-tile nt -> offset inside the halo tile
  int tapoff[NTT];
#pragma unroll
  for (int nt = 0; nt < NTT; ++nt) {
    const int tap = nt * 16 + i16;
    const int cl = tap / RSf, rs = tap - cl * RSf;
    const int r = rs / a.S, s = rs - r * a.S;
    tapoff[nt] = (cl < p.CC) ? cl * p.PS + r * p.RS + s : 0;
  }
  // A operand: lane's filter plane of M-tile mf (clipped: surplus rows are never stored)
  int fplane[MTF];
#pragma unroll
  for (int mf = 0; mf < MTF; ++mf) fplane[mf] = min(mf * 16 + i16, kcount - 1) * p.PSZ;

  for (int item = gidx; item < p.items; item += p.G) {
    const int tx = item % p.tiles_x;
    const int ty = (item / p.tiles_x) % p.tiles_y;
    const int n = item / (p.tiles_x * p.tiles_y);
    const int oy0 = ty * TH, ox0 = tx * kTileW;
    __syncthreads();
    // ---- dz tile [kcount][TH][32]
#pragma unroll
    for (int it = 0; it < MTF * 16 * ITS_PER_K; ++it) {
      const int k = it / ITS_PER_K;   // compile-time
      if (k < kcount) {
        const int e = (it % ITS_PER_K) * kThreads + tid;
        const int col = e & 31, row = e >> 5;
        const int gi = oy0 + row, gj = ox0 + col;
        float v = 0.0f;
        if (gi < p.Ho && gj < p.Wo) v = dz_value(a, p.Ho, p.Wo, n, k0 + k, gi, gj);
        dzs[k * p.PSZ + e] = v;
        dbacc[k] += v;
      }
    }
    // ---- x halo tile [CC][rows][cols]
    {
      const int total = p.CC * p.rows * p.cols;
      int col = tid % p.cols;
      int q = tid / p.cols;
      int row = q % p.rows, cl = q / p.rows;
      const int dcol = kThreads % p.cols, dq = kThreads / p.cols;
      for (int e = tid; e < total; e += kThreads) {
        const int gi = oy0 - a.pad + row, gj = ox0 - a.pad + col, ci = c0 + cl;
        float v = 0.0f;
        if (ci < a.C && gi >= 0 && gi < a.H && gj >= 0 && gj < a.W)
          v = a.x[((n * a.C + ci) * a.H + gi) * a.W + gj];
        xs[cl * p.PS + row * p.RS + col] = v;
        col += dcol;
        row += dq;
        if (col >= p.cols) { col -= p.cols; ++row; }
        while (row >= p.rows) { row -= p.rows; ++cl; }
      }
    }
    __syncthreads();
    // ---- MFMA: 4 neighbouring pixels per step
#pragma unroll
    for (int rr = 0; rr < RW; ++rr) {
      const int row = wave * RW + rr;
      const float *za = dzs + row * kTileW + kq;
      const float *xb = xs + row * p.RS + kq;
#pragma unroll
      for (int cg = 0; cg < 8; ++cg) {
        float af[MTF], bf[NTT];
#pragma unroll
        for (int mf = 0; mf < MTF; ++mf) af[mf] = za[fplane[mf] + 4 * cg];
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt) bf[nt] = xb[tapoff[nt] + 4 * cg];
#pragma unroll
        for (int mf = 0; mf < MTF; ++mf)
#pragma unroll
          for (int nt = 0; nt < NTT; ++nt)
            acc[mf][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[mf], bf[nt], acc[mf][nt], 0, 0, 0);
      }
    }
  }

  // ---- per-wave partial block: [(chunk*G + g)*4 + wave][mf][nt][v][lane], per filter group
  {
    float *dst = a.partial + (long)blockIdx.y * p.group_stride +
                 ((long)(chunk * p.G + gidx) * 4 + wave) * (MTF * NTT * 256);
#pragma unroll
    for (int mf = 0; mf < MTF; ++mf)
#pragma unroll
      for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v) dst[((mf * NTT + nt) * 4 + v) * 64 + lane] = acc[mf][nt][v];
  }
  // ---- db partials: [wave-partial of chunk 0][K]
  if (chunk == 0) {
    float *dbp = a.partial + p.db_offset + ((long)gidx * 4 + wave) * a.K + k0;
#pragma unroll
    for (int k = 0; k < MTF * 16; ++k) {
      const float s = wave_sum(dbacc[k]);
      if (lane == 0 && k < kcount) dbp[k] = s;
    }
  }
}

// One workgroup per 16 outputs (consecutive taps of one filter); 16 slices of the partial
// list are summed in parallel in double, then combined in a fixed order.
__global__ __launch_bounds__(kThreads) void wgrad_reduce_kernel(const WgradReduceArgs a, const WgradPlan plan,
                                                               int kgroups, long group_stride, int ndw) {
  __shared__ double red[16][17];
  const int tid = threadIdx.x, o16 = tid & 15, slice = tid >> 4;
  const int RSf = a.R * a.S;
  const int blk = blockIdx.x;
  const int nblk_dw = (ndw + 15) / 16;
  double sum = 0.0;
  int out_index = -1;
  if (blk < nblk_dw) {
    const int o = blk * 16 + o16;   // flat index into dw[K][C][R][S]
    if (o < ndw) {
      const int ko = o / (a.C * RSf), rem = o - ko * (a.C * RSf);
      const int ci = rem / RSf, rs = rem - ci * RSf;
      const int chunk = ci / plan.CC, cl = ci - chunk * plan.CC;
      const int tap = cl * RSf + rs;
      const int grp = ko / (plan.MTF * 16), m = ko - grp * (plan.MTF * 16);
      const int mf = m >> 4, lq = (m & 15) >> 2, v = m & 3;
      const int nt = tap >> 4, lane = lq * 16 + (tap & 15);
      const long within = ((long)(mf * plan.NTT + nt) * 4 + v) * 64 + lane;
      const long blockf = (long)plan.MTF * plan.NTT * 256;
      const long base = (long)grp * group_stride + (long)chunk * plan.n_partials * blockf + within;
      for (int pidx = slice; pidx < plan.n_partials; pidx += 16) {
        double t = (double)a.pos[base + pidx * blockf];
        if (a.neg) t -= (double)a.neg[base + pidx * blockf];
        sum += t;
      }
      out_index = o;
    }
  } else {
    const int k = (blk - nblk_dw) * 16 + o16;
    if (k < a.K) {
      for (int pidx = slice; pidx < plan.n_partials; pidx += 16) {
        double t = (double)a.pos[plan.db_offset + (long)pidx * a.K + k];
        if (a.neg) t -= (double)a.neg[plan.db_offset + (long)pidx * a.K + k];
        sum += t;
      }
      out_index = k;
    }
  }
  red[slice][o16] = sum;
  __syncthreads();
  if (slice == 0 && out_index >= 0) {
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < 16; ++q) s += red[q][o16];
    const float gval = (float)(s * (double)a.scale);
    if (blk < nblk_dw) {
      if (a.dw) a.dw[out_index] = gval;
      if (a.w_update) a.w_update[out_index] += a.step * gval;
    } else {
      if (a.db) a.db[out_index] = gval;
      if (a.b_update) a.b_update[out_index] += a.step * gval;
    }
  }
}

inline int round_up_mod(int v, int m, int r) {
  int x = v - (v % m) + r;
  if (x < v) x += m;
  return x;
}

const int kNttChoices[] = {2, 5, 7, 9};

inline int pick_ntt(int tiles) {
  for (int c : kNttChoices)
    if (tiles <= c) return c;
  return 0;
}

}  // namespace

bool plan_wgrad(int N, int C, int H, int W, int K, int R, int S, int pad, WgradPlan *plan) {
  const int Ho = H + 2 * pad - R + 1, Wo = W + 2 * pad - S + 1;
  const int RSf = R * S;
  // channels per chunk: minimise (chunks x tap tiles) with at most 9 tap tiles
  int best_cc = 0, best_cost = 0, best_ntt = 0;
  for (int cc = 1; cc <= (C < 16 ? C : 16); ++cc) {
    const int ntt = pick_ntt((cc * RSf + 15) / 16);
    if (!ntt) break;
    const int cost = ((C + cc - 1) / cc) * ntt;
    if (!best_cc || cost <= best_cost) { best_cc = cc; best_cost = cost; best_ntt = ntt; }
  }
  if (!best_cc) return false;
  plan->CC = best_cc;
  plan->NTT = best_ntt;
  plan->nchunks = (C + best_cc - 1) / best_cc;
  plan->TH = 8;
  const int rows = plan->TH + R - 1, cols = kTileW + S - 1;
  const int RS = round_up_mod(cols, 32, 6);
  const int PS = RS * rows;
  const int PSZ = plan->TH * kTileW + 2;
  int mtf = (K + 15) / 16;
  if (mtf > 3) mtf = 3;
  for (;; --mtf) {
    const int planes = K < mtf * 16 ? K : mtf * 16;
    plan->lds_bytes = sizeof(float) * ((size_t)best_cc * PS + (size_t)planes * PSZ);
    if (plan->lds_bytes <= 64 * 1024) break;
    if (mtf == 1) return false;
  }
  plan->MTF = mtf;
  const int tiles_x = (Wo + kTileW - 1) / kTileW, tiles_y = (Ho + plan->TH - 1) / plan->TH;
  const long items = (long)N * tiles_x * tiles_y;
  const int kgroups = (K + mtf * 16 - 1) / (mtf * 16);
  long G = 1024 / ((long)plan->nchunks * kgroups);
  if (G < 1) G = 1;
  if (G > items) G = items;
  plan->G = (int)G;
  plan->n_partials = 4 * plan->G;
  const size_t blockf = (size_t)mtf * plan->NTT * 256;
  const size_t group_stride = (size_t)plan->nchunks * plan->n_partials * blockf;
  plan->db_offset = group_stride * kgroups;
  plan->partial_floats = plan->db_offset + (size_t)plan->n_partials * K;
  return true;
}

namespace {
template <int MTF, int NTT>
hipError_t launch_wgrad_t(const WgradParams &p, const WgradPlan &plan, hipStream_t stream) {
  dim3 grid((unsigned)(plan.G * plan.nchunks), (unsigned)p.kgroups, 1);
  hipLaunchKernelGGL((wgrad_kernel<MTF, NTT, 8>), grid, dim3(kThreads), plan.lds_bytes, stream, p);
  return hipGetLastError();
}
template <int MTF>
hipError_t launch_wgrad_m(const WgradParams &p, const WgradPlan &plan, hipStream_t stream) {
  switch (plan.NTT) {
  case 2: return launch_wgrad_t<MTF, 2>(p, plan, stream);
  case 5: return launch_wgrad_t<MTF, 5>(p, plan, stream);
  case 7: return launch_wgrad_t<MTF, 7>(p, plan, stream);
  case 9: return launch_wgrad_t<MTF, 9>(p, plan, stream);
  default: return hipErrorInvalidValue;
  }
}
}  // namespace

hipError_t launch_wgrad(const WgradArgs &a, const WgradPlan &plan, hipStream_t stream) {
  WgradParams p;
  p.a = a;
  p.Ho = a.H + 2 * a.pad - a.R + 1;
  p.Wo = a.W + 2 * a.pad - a.S + 1;
  p.CC = plan.CC;
  p.nchunks = plan.nchunks;
  p.G = plan.G;
  p.rows = plan.TH + a.R - 1;
  p.cols = kTileW + a.S - 1;
  p.RS = round_up_mod(p.cols, 32, 6);
  p.PS = p.RS * p.rows;
  p.PSZ = plan.TH * kTileW + 2;
  p.tiles_x = (p.Wo + kTileW - 1) / kTileW;
  p.tiles_y = (p.Ho + plan.TH - 1) / plan.TH;
  p.items = a.N * p.tiles_x * p.tiles_y;
  p.kgroups = (a.K + plan.MTF * 16 - 1) / (plan.MTF * 16);
  p.db_offset = (long)plan.db_offset;
  p.group_stride = (long)plan.nchunks * plan.n_partials * ((long)plan.MTF * plan.NTT * 256);
  switch (plan.MTF) {
  case 1: return launch_wgrad_m<1>(p, plan, stream);
  case 2: return launch_wgrad_m<2>(p, plan, stream);
  case 3: return launch_wgrad_m<3>(p, plan, stream);
  default: return hipErrorInvalidValue;
  }
}

hipError_t launch_wgrad_reduce(const WgradReduceArgs &a, const WgradPlan &plan, hipStream_t stream) {
  const int ndw = a.K * a.C * a.R * a.S;
  const int kgroups = (a.K + plan.MTF * 16 - 1) / (plan.MTF * 16);
  const long group_stride = (long)plan.nchunks * plan.n_partials * ((long)plan.MTF * plan.NTT * 256);
  const int blocks = (ndw + 15) / 16 + (a.K + 15) / 16;
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(blocks), dim3(kThreads), 0, stream, a, plan, kgroups, group_stride, ndw);
  return hipGetLastError();
}

}  // namespace dllk
