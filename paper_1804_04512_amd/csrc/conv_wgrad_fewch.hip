// Filter gradient of a padded 3x3 layer with one to three input channels behind ReLU + 2x2 max
// pooling (the first layer of the image networks: RGB or grey-scale input, 16 filters), on fp32
// MFMA (v_mfma_f32_16x16x4_f32), gfx950.
//
//   dw[k,c,r,s] = sum_{n,i,j} dz[n,k,i,j] * xpad[n,c,i+r,j+s],   db[k] = sum_{n,i,j} dz[n,k,i,j]
//
// Filters sit on the MFMA M axis, the (channel, tap) pairs on N (27 of 32 columns for RGB).  dz has
// at most one non-zero per pooling window, so the sum over pixels is taken position by position:
// for each of the four window positions one instruction contracts over four WINDOWS, the
// filter-side operand of lane (filter, window) being the pooled gradient where the recorded
// position is that position and the unit is active, else zero: one compare and one select on
// values that come straight from global memory into registers (16 bytes per lane and 16 windows,
// every element loaded once); no tile of dz exists anywhere.  The image-side operand is read from
// LDS at (window + position + tap), an address that is a per-lane constant plus an instruction
// immediate.  Column 27 of the second tap tile multiplies by a row of ones, so the bias gradient
// falls out of the same products.
// Every wavefront works alone on a strip of 32 windows (64 pixels) that it walks downwards, with
// its own four-row ring of image rows in LDS (two new rows per window row, requested one window
// row ahead); the four wavefronts of a workgroup take neighbouring strips, so a workgroup reads
// whole stretches of image rows.  No workgroup barrier until the final, fixed-order sum of the
// wavefronts' accumulators; partial blocks have the direct kernel's layout.
#include "dll_internal.h"

#include <type_traits>

namespace dllk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kWin = 32;                 // windows per strip row
constexpr int kRS = 100;                 // LDS row: image column x0 sits at LDS column 4; 4 (mod 32) banks apart
constexpr int kPS = 4 * kRS;             // channel plane of four row slots: 16 (mod 32) banks apart
constexpr int kOnes = 3 * kPS;           // a row of ones (the bias-gradient column) ...
constexpr int kZeros = kOnes + 72;       // ... and a row of zeros (tap columns the layer does not have)
constexpr int kWaveFloats = kZeros + 72;
constexpr unsigned kOob = 0x80000000u;

struct FewchParams {
  WgradArgs a;
  int Hp, Wp;
  int xsegs, xgroups;  // 64-pixel strips per row; groups of four neighbouring strips
  int rg, rgroups;     // window rows per work item, row groups per image
  int items;           // work items of a workgroup: N * rgroups * xgroups
  int G;
  long db_offset;
  unsigned x_bytes, dy_bytes;
};

__global__ __launch_bounds__(kThreads, 4) void wgrad_fewch_kernel(const FewchParams p) {
  extern __shared__ float lds[];
  const WgradArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int gidx = blockIdx.x;
  float *xs = lds + wave * kWaveFloats;

  const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.dy), 0, (int)p.dy_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_idx = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(a.idx), 0, (int)(p.dy_bytes >> 2), 0x00020000);

  for (int e = lane; e < 72; e += 64) { xs[kOnes + e] = 1.0f; xs[kZeros + e] = 0.0f; }

  // ---- image-side operand: lane (tap column i16 of tile nt, window 4kq + e of a group of 16) reads, for
  // window position (pa, pb), x[c][2wy - 1 + pa + r][2wx - 1 + pb + s]; rows pa + r of the window's 4x4
  // patch live in the ring's slots, which alternate with the parity of the window row.  pb, e and
  // the group are instruction immediates.
  int offB[2][2][2];   // [tap tile][pa][parity]
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int tap = nt * 16 + i16;
    const int c = tap / 9, rs9 = tap - 9 * c, r = rs9 / 3, s = rs9 - 3 * r;
#pragma unroll
    for (int pa = 0; pa < 2; ++pa)
#pragma unroll
      for (int sp = 0; sp < 2; ++sp) {
        const int i = pa + r;
        const int slot = i < 2 ? 2 * sp + i : 2 * (sp ^ 1) + (i - 2);
        offB[nt][pa][sp] = (tap < 9 * a.C ? c * kPS + slot * kRS + 3 + s : (tap == 27 ? kOnes : kZeros)) + 8 * kq;
      }
  }

  // ---- staging slots of a pair of image rows: (channel, row of the pair, aligned 16-byte group) and
  // (channel, row, left or right neighbour column); offsets are fixed per work item
  int xlo[2], xpl[2], xcol[2];
  bool xr1[2], xin[2];
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int s = lane + 64 * it;
    const int ch = s >> 5, rr = (s >> 4) & 1, j = s & 15;
    xin[it] = ch < a.C;
    xr1[it] = rr == 1;
    xpl[it] = (ch * a.H + rr) * a.W + 4 * j;
    xcol[it] = 4 * j;
    xlo[it] = ch * kPS + rr * kRS + 4 + 4 * j;
  }
  const int h_ch = lane >> 2, h_rr = (lane >> 1) & 1, h_side = lane & 1;
  const bool h_in = h_ch < a.C;
  const int hpl = (h_ch * a.H + h_rr) * a.W + (h_side ? 64 : -1);
  const int hlo = (h_in ? h_ch : 0) * kPS + h_rr * kRS + (h_side ? 68 : 3);

  floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
  float4 xa[2], xb[2];
  float ha = 0.0f, hb = 0.0f;
  float4 dyc[2], dyn[2];       // pooled gradients of the lane's windows 16j + 4kq .. + 3 of a strip row (j = 0, 1)
  unsigned idc[2], idn[2];     // and their pooling bytes
  unsigned xv[2], hv = kOob, dv = kOob, iv = kOob;
  bool dok[2] = {false, false};   // the lane's two 16-byte groups lie inside the pooled row

  auto item_setup = [&](int n, int x0, int wx0, int wy0) {
    const int base = (n * a.C * a.H + (2 * wy0 - 1)) * a.W + x0;
#pragma unroll
    for (int it = 0; it < 2; ++it) xv[it] = (xin[it] && x0 + xcol[it] < a.W) ? 4u * (unsigned)(base + xpl[it]) : kOob;
    const int hc = x0 + (h_side ? 64 : -1);
    hv = (h_in && x0 < a.W && (unsigned)hc < (unsigned)a.W) ? 4u * (unsigned)(base + hpl) : kOob;
    const unsigned e = (unsigned)(((n * a.K + i16) * p.Hp + wy0) * p.Wp + wx0 + 4 * kq);
    dv = 4u * e;
    iv = e;
    dok[0] = i16 < a.K && wx0 + 4 * kq < p.Wp;
    dok[1] = i16 < a.K && wx0 + 16 + 4 * kq < p.Wp;
  };
  // rows 2P-1 and 2P -> registers; dP = P - wy0 of the item (added to the lanes' offsets: the range
  // check of a buffer load looks at the vector offset on its own)
  auto load_pair = [&](int P, int dP, float4 (&xr)[2], float &xh) {
    const unsigned down = (unsigned)(8 * a.W) * (unsigned)dP;
    const bool top = P == 0, bot = 2 * P >= a.H;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      unsigned off = xv[it] + down;
      if (top || bot) off = (xr1[it] ? bot : top) ? kOob : off;
      const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs_x, (int)off, 0, 0));
      xr[it] = make_float4(v[0], v[1], v[2], v[3]);
    }
    unsigned off = hv + down;
    if (top || bot) off = (h_rr ? bot : top) ? kOob : off;
    xh = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_x, (int)off, 0, 0));
  };
  auto store_pair = [&](int slotpair, const float4 (&xr)[2], float xh) {
    float *dst = xs + slotpair * 2 * kRS;
#pragma unroll
    for (int it = 0; it < 2; ++it)
      if (xin[it]) *reinterpret_cast<float4 *>(dst + xlo[it]) = xr[it];
    if (h_in) dst[hlo] = xh;
  };
  // pooled gradients and pooling bytes of window row wy0 + dB: the lane's filter, its eight windows
  auto load_dy = [&](int dB, float4 (&g)[2], unsigned (&f)[2]) {
    const unsigned down = (unsigned)p.Wp * (unsigned)dB;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs_dy, (int)(dok[j] ? dv + 4u * down + 64u * j : kOob), 0, 0));
      g[j] = make_float4(v[0], v[1], v[2], v[3]);
      f[j] = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(rs_idx, (int)(dok[j] ? iv + down + 16u * j : kOob), 0, 0);
    }
  };

  // ---- one window row: eight steps of four windows (one per K lane) x four positions x two tap tiles.
  // The image-side fragments of a step are read while the step before it is multiplied (scheduling
  // barriers keep that order).
  auto window_row = [&](auto spc) {
    constexpr int SP = decltype(spc)::value;
    const float *bp[2][2] = {{xs + offB[0][0][SP], xs + offB[0][1][SP]}, {xs + offB[1][0][SP], xs + offB[1][1][SP]}};
    float fr[2][4][2];   // [buffer][position][tap tile]
    auto read_step = [&](auto tc) {
      constexpr int t = decltype(tc)::value, j = t >> 2, e = t & 3;
#pragma unroll
      for (int pos = 0; pos < 4; ++pos)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) fr[t & 1][pos][nt] = bp[nt][pos >> 1][(pos & 1) + 32 * j + 2 * e];
    };
    auto step = [&](auto tc) {
      constexpr int t = decltype(tc)::value, j = t >> 2, e = t & 3;
      if constexpr (t < 7) read_step(std::integral_constant<int, t + 1>{});
      __builtin_amdgcn_sched_barrier(0);
      const float gv = e == 0 ? dyc[j].x : (e == 1 ? dyc[j].y : (e == 2 ? dyc[j].z : dyc[j].w));
      const unsigned where = (idc[j] >> (8 * e)) & 7u;   // recorded position, 4 and above: inactive unit
#pragma unroll
      for (int pos = 0; pos < 4; ++pos) {
        const float av = where == (unsigned)pos ? gv : 0.0f;
        acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av, fr[t & 1][pos][0], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av, fr[t & 1][pos][1], acc1, 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    read_step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 0>{}); step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{}); step(std::integral_constant<int, 3>{});
    step(std::integral_constant<int, 4>{}); step(std::integral_constant<int, 5>{});
    step(std::integral_constant<int, 6>{}); step(std::integral_constant<int, 7>{});
  };

  // ---- work items: (image, group of window rows, group of four neighbouring strips), one strip per
  // wavefront; the rows and gradients an item starts with are requested during the last window row
  // of the item before it
  auto begin_item = [&](int item, int &wy1) {
    const int xg = item % p.xgroups;
    const int rgrp = (item / p.xgroups) % p.rgroups;
    const int n = item / (p.xgroups * p.rgroups);
    const int xseg = xg * 4 + wave;
    const int wy0 = rgrp * p.rg;
    item_setup(n, xseg * 64, xseg * kWin, wy0);
    wy1 = xseg < p.xsegs ? min(wy0 + p.rg, p.Hp) : wy0;
    return wy0;
  };
  auto request_item = [&](int item) {
    int wy1;
    const int wy0 = begin_item(item, wy1);
    if (wy1 > wy0) {
      load_pair(wy0, 0, xa, ha);
      load_pair(wy0 + 1, 1, xb, hb);
      load_dy(0, dyn, idn);
    }
  };
  if (gidx < p.items) request_item(gidx);
  for (int item = gidx; item < p.items; item += p.G) {
    int wy1;
    const int wy0 = begin_item(item, wy1);
    if (wy1 > wy0) store_pair(wy0 & 1, xa, ha);
    for (int wy = wy0; wy < wy1; ++wy) {
      dyc[0] = dyn[0]; dyc[1] = dyn[1]; idc[0] = idn[0]; idc[1] = idn[1];
      if (wy == wy0) store_pair((wy + 1) & 1, xb, hb);
      else store_pair((wy + 1) & 1, xa, ha);
      if (wy + 1 < wy1) {
        load_pair(wy + 2, wy + 2 - wy0, xa, ha);   // in flight during this window row's products
        load_dy(wy + 1 - wy0, dyn, idn);
      } else if (item + p.G < p.items) {
        request_item(item + p.G);
      }
      if (wy & 1) window_row(std::integral_constant<int, 1>{});
      else window_row(std::integral_constant<int, 0>{});
    }
    if (wy1 == wy0 && item + p.G < p.items) request_item(item + p.G);
  }

  // ---- the four wavefronts' accumulators are added in wavefront order; the block leaves in the
  // direct kernel's layout [tap tile][v][lane]; column 27 of the second tile is the bias gradient
  float *blk = lds;   // [wavefront][512], over the rings
  __syncthreads();
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    blk[wave * 512 + v * 64 + lane] = acc0[v];
    blk[wave * 512 + 256 + v * 64 + lane] = acc1[v];
  }
  __syncthreads();
  if (tid < 128) {
    float4 sum = *reinterpret_cast<const float4 *>(blk + 4 * tid);
#pragma unroll
    for (int w2 = 1; w2 < 4; ++w2) {
      const float4 o = *reinterpret_cast<const float4 *>(blk + w2 * 512 + 4 * tid);
      sum.x += o.x; sum.y += o.y; sum.z += o.z; sum.w += o.w;
    }
    *reinterpret_cast<float4 *>(a.partial + (long)gidx * 512 + 4 * tid) = sum;
    // element (filter 4kq'+v, tap 27) sits at float 256 + 64v + 16kq' + 11: component w of thread 64 + 16v + 4kq' + 2
    if (tid >= 64 && (tid & 3) == 2) {
      const int v = (tid - 64) >> 4, kq2 = ((tid - 64) >> 2) & 3, k = 4 * kq2 + v;
      if (k < a.K) a.partial[p.db_offset + (long)gidx * a.K + k] = sum.w;
    }
  }
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

}  // namespace

bool wgrad_fewch_shape(int C, int H, int W, int K, int R, int S, int pad, int pool) {
  return R == 3 && S == 3 && pad == 1 && pool == 2 && C <= 3 && K <= 16 && W % 8 == 0 && H % 2 == 0;
}

bool wgrad_fewch_applies(const WgradArgs &a, const WgradPlan &plan) {
  if (!wgrad_fewch_shape(a.C, a.H, a.W, a.K, a.R, a.S, a.pad, a.pool)) return false;
  if (a.act != ACT_RELU_FLAGGED || !a.idx || a.W >= (1 << 17)) return false;
  if (plan.MTF != 1 || plan.NTT != 2 || plan.CC != a.C || plan.nchunks != 1) return false;
  if (!aligned16(a.x) || !aligned16(a.dy) || (reinterpret_cast<uintptr_t>(a.idx) & 3u)) return false;
  const long limit = (1L << 31) - (1L << 24);
  return 4L * a.N * a.C * a.H * a.W < limit && 4L * a.N * a.K * (a.H / 2) * (a.W / 2) < limit;
}

hipError_t launch_wgrad_fewch(const WgradArgs &a, const WgradPlan &plan, hipStream_t stream) {
  if (!wgrad_fewch_applies(a, plan)) return hipErrorInvalidValue;
  FewchParams p;
  p.a = a;
  p.Hp = a.H / 2;
  p.Wp = a.W / 2;
  p.xsegs = (a.W + 63) / 64;
  p.xgroups = (p.xsegs + 3) / 4;
  p.G = plan.G;
  p.db_offset = (long)plan.db_offset;
  p.x_bytes = (unsigned)(4L * a.N * a.C * a.H * a.W);
  p.dy_bytes = (unsigned)(4L * a.N * a.K * p.Hp * p.Wp);
  // window rows per work item: the longest strip that still leaves every workgroup an item
  p.rg = 2;
  for (int rg = 16; rg >= 2; rg /= 2) {
    const long items = (long)a.N * p.xgroups * ((p.Hp + rg - 1) / rg);
    if (items >= p.G || rg == 2) { p.rg = rg; break; }
  }
  p.rgroups = (p.Hp + p.rg - 1) / p.rg;
  const long items = (long)a.N * p.xgroups * p.rgroups;
  if (items > 0x7fffffffL) return hipErrorInvalidValue;
  p.items = (int)items;
  const size_t lds = sizeof(float) * 4 * kWaveFloats;
  hipLaunchKernelGGL(wgrad_fewch_kernel, dim3((unsigned)p.G), dim3(kThreads), lds, stream, p);
  return hipGetLastError();
}

}  // namespace dllk
