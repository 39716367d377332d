// Forward pass of a padded 3x3 layer with one to three input channels and at most 16 filters,
// bias + ReLU + 2x2 max pooling fused (the first layer of the image networks, Section VI), on fp32
// MFMA (v_mfma_f32_16x16x4_f32), gfx950.
//
//   y[n,k,u,v] = max over the 2x2 window of relu(b[k] + sum_{c,r,s} xpad[n,c,2u+a+r,2v+b+s] * w[k,c,r,s])
//
// Pixels sit on the MFMA M axis (an M-tile is four pooling windows x four window positions, so a
// lane's four accumulator registers are one window: maximum, position, bias and ReLU are
// register-local), filters on N, the 27 (channel, tap) products of an RGB layer on K as seven steps
// in the filter's own order.  The filter-side fragments never change and stay in registers; the
// image-side fragment is one LDS read per instruction at a per-lane constant plus an immediate.
// Every wavefront works alone on a strip of 32 windows (64 pixels) that it walks downwards with
// its own four-row ring of image rows in LDS (two new rows per window row, requested one window
// row ahead); the four wavefronts of a workgroup take neighbouring strips, so a workgroup reads and
// writes whole stretches of rows: a lane stores eight neighbouring pooled values of its filter (two
// 16-byte stores) and their eight pooling bytes.  No workgroup barrier anywhere.
#include "dll_internal.h"

#include <type_traits>

namespace dllk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kWin = 32;                 // windows per strip row
constexpr int kRS = 100;                 // LDS row: image column x0 sits at LDS column 4
constexpr int kPS = 4 * kRS;             // channel plane of four row slots
constexpr int kZeros = 3 * kPS;          // a row of zeros: the K slots beyond the layer's (channel, tap) pairs
constexpr int kWaveFloats = kZeros + 72;
constexpr unsigned kOob = 0x80000000u;

struct FwdFewchParams {
  ConvEngineArgs a;
  int Hp, Wp;
  int xsegs, xgroups;  // 64-pixel strips per row; groups of four neighbouring strips
  int rg, rgroups;     // window rows per work item, row groups per image
  int items, G;
  unsigned x_bytes, y_bytes;
};

template <bool IDX>
__global__ __launch_bounds__(kThreads, 3) void conv_fwd_fewch_kernel(const FwdFewchParams p) {
  extern __shared__ float lds[];
  const ConvEngineArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int gidx = blockIdx.x;
  const int C = a.Cin, K = a.Kout, H = a.Hin, W = a.Win;
  float *xs = lds + wave * kWaveFloats;

  const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.src), 0, (int)p.x_bytes, 0x00020000);
  // Outputs leave through range-checked buffer stores: a lane with nothing to store gets an
  // out-of-range offset, so every window row issues the same number of stores and the wait for the
  // next rows' loads (which were requested before them) need not wait for the stores as well.
  const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, (int)p.y_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_i = __builtin_amdgcn_make_buffer_rsrc(IDX ? a.out_idx : reinterpret_cast<unsigned char *>(a.out), 0, (int)(p.y_bytes >> 2), 0x00020000);
  for (int e = lane; e < 72; e += 64) xs[kZeros + e] = 0.0f;

  // ---- image-side operand: lane (pixel i16 of an M-tile = window i16 / 4, position i16 % 4 = 2pa + pb;
  // K slot kq) reads, in step t, x[c][2wy - 1 + pa + r][2wx - 1 + pb + s] for (c, r, s) = pair 4t + kq.
  // M-tile mt of the lane's window group holds window 8 * (i16 / 4) + mt of the strip, so that the
  // lane that ends up with a window's results (accumulator rows 4kq + v) owns eight neighbours.
  const int wl = i16 >> 2, pa = (i16 >> 1) & 1, pb = i16 & 1;
  int offA[7][2];
  float wB[7];
#pragma unroll
  for (int t = 0; t < 7; ++t) {
    const int k = 4 * t + kq;
    const int c = k / 9, rs9 = k - 9 * c, r = rs9 / 3, s = rs9 - 3 * r;
    const bool real = k < 9 * C;
#pragma unroll
    for (int sp = 0; sp < 2; ++sp) {
      const int i = pa + r;
      const int slot = i < 2 ? 2 * sp + i : 2 * (sp ^ 1) + (i - 2);
      offA[t][sp] = (real ? c * kPS + slot * kRS + 3 + pb + s : kZeros) + 16 * wl;
    }
    wB[t] = (real && i16 < K) ? a.w[i16 * 9 * C + k] : 0.0f;   // filter i16, pair k in the filter's own order
  }
  const float bias = (a.bias && i16 < K) ? a.bias[i16] : 0.0f;

  // ---- staging slots of a pair of image rows (as in the first layer's filter-gradient kernel)
  int xlo[2], xpl[2], xcol[2];
  bool xr1[2], xin[2];
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int s = lane + 64 * it;
    const int ch = s >> 5, rr = (s >> 4) & 1, j = s & 15;
    xin[it] = ch < C;
    xr1[it] = rr == 1;
    xpl[it] = (ch * H + rr) * W + 4 * j;
    xcol[it] = 4 * j;
    xlo[it] = ch * kPS + rr * kRS + 4 + 4 * j;
  }
  const int h_ch = lane >> 2, h_rr = (lane >> 1) & 1, h_side = lane & 1;
  const bool h_in = h_ch < C;
  const int hpl = (h_ch * H + h_rr) * W + (h_side ? 64 : -1);
  const int hlo = (h_in ? h_ch : 0) * kPS + h_rr * kRS + (h_side ? 68 : 3);

  floatx4 acc[8];
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
  float4 xa[2], xb[2];
  float ha = 0.0f, hb = 0.0f;
  unsigned xv[2], hv = kOob;
  unsigned out0 = 0;    // element offset of the lane's first pooled output of the item's first window row
  bool ok0 = false, ok1 = false;   // the lane's two groups of four windows lie inside the pooled row

  auto item_setup = [&](int n, int x0, int wx0, int wy0) {
    const int base = (n * C * H + (2 * wy0 - 1)) * W + x0;
#pragma unroll
    for (int it = 0; it < 2; ++it) xv[it] = (xin[it] && x0 + xcol[it] < W) ? 4u * (unsigned)(base + xpl[it]) : kOob;
    const int hc = x0 + (h_side ? 64 : -1);
    hv = (h_in && x0 < W && (unsigned)hc < (unsigned)W) ? 4u * (unsigned)(base + hpl) : kOob;
    out0 = (unsigned)(((n * K + i16) * p.Hp + wy0) * p.Wp + wx0 + 8 * kq);
    ok0 = i16 < K && wx0 + 8 * kq < p.Wp;
    ok1 = i16 < K && wx0 + 8 * kq + 4 < p.Wp;
  };
  auto load_pair = [&](int P, int dP, float4 (&xr)[2], float &xh) {
    const unsigned down = (unsigned)(8 * W) * (unsigned)dP;
    const bool top = P == 0, bot = 2 * P >= H;
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

  // ---- one window row: seven K steps x eight M-tiles; the fragments of a step are read while the
  // step before it is multiplied (scheduling barriers keep that order); then the epilogue
  auto window_row = [&](auto spc, int dW) {
    constexpr int SP = decltype(spc)::value;
    float fr[2][8];
    auto read_step = [&](auto tc) {
      constexpr int t = decltype(tc)::value;
      const float *ap = xs + offA[t][SP];
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) fr[t & 1][mt] = ap[2 * mt];
    };
    auto step = [&](auto tc) {
      constexpr int t = decltype(tc)::value;
      if constexpr (t < 6) read_step(std::integral_constant<int, t + 1>{});
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mt = 0; mt < 8; ++mt)   // the first step starts from zero: no clearing of the accumulators between window rows
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(fr[t & 1][mt], wB[t], t == 0 ? floatx4{0.f, 0.f, 0.f, 0.f} : acc[mt], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    };
    read_step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 0>{}); step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{}); step(std::integral_constant<int, 3>{});
    step(std::integral_constant<int, 4>{}); step(std::integral_constant<int, 5>{});
    step(std::integral_constant<int, 6>{});
    // the lane's eight windows (filter i16, windows 8kq .. 8kq + 7 of the strip): first maximum in the
    // order (0,0), (0,1), (1,0), (1,1); bias and ReLU commute with the maximum
    float yv[8];
    unsigned ib[2] = {0u, 0u};
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      const floatx4 z = acc[mt];
      float m = z[0];
      unsigned arg = 0;
      if (z[1] > m) { m = z[1]; arg = 1; }
      if (z[2] > m) { m = z[2]; arg = 2; }
      if (z[3] > m) { m = z[3]; arg = 3; }
      const float y = fmaxf(m + bias, 0.0f);
      yv[mt] = y;
      ib[mt >> 2] |= (arg | (y > 0.0f ? 0u : (unsigned)kIdxInactive)) << (8 * (mt & 3));
    }
    const unsigned o = out0 + (unsigned)dW * (unsigned)p.Wp;
    const floatx4 y0 = {yv[0], yv[1], yv[2], yv[3]}, y1 = {yv[4], yv[5], yv[6], yv[7]};
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((ext_vector_type(4))) unsigned, y0), rs_y, (int)(ok0 ? 4u * o : kOob), 0, 0);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((ext_vector_type(4))) unsigned, y1), rs_y, (int)(ok1 ? 4u * o + 16u : kOob), 0, 0);
    if (IDX) {
      __builtin_amdgcn_raw_buffer_store_b32(ib[0], rs_i, (int)(ok0 ? o : kOob), 0, 0);
      __builtin_amdgcn_raw_buffer_store_b32(ib[1], rs_i, (int)(ok1 ? o + 4u : kOob), 0, 0);
    }
  };

  // ---- work items: (image, group of window rows, group of four neighbouring strips), one strip per
  // wavefront; the rows an item starts with are requested during the last window row of the item before
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
    }
  };
  if (gidx < p.items) request_item(gidx);
  for (int item = gidx; item < p.items; item += p.G) {
    int wy1;
    const int wy0 = begin_item(item, wy1);
    // what the epilogue needs of this item survives the request for the next one (which re-runs item_setup)
    const unsigned my_out0 = out0;
    const bool my_ok0 = ok0, my_ok1 = ok1;
    if (wy1 > wy0) store_pair(wy0 & 1, xa, ha);
    for (int wy = wy0; wy < wy1; ++wy) {
      if (wy == wy0) store_pair((wy + 1) & 1, xb, hb);
      else store_pair((wy + 1) & 1, xa, ha);
      if (wy + 1 < wy1) load_pair(wy + 2, wy + 2 - wy0, xa, ha);   // in flight during this window row's products
      else if (item + p.G < p.items) request_item(item + p.G);
      out0 = my_out0; ok0 = my_ok0; ok1 = my_ok1;
      if (wy & 1) window_row(std::integral_constant<int, 1>{}, wy - wy0);
      else window_row(std::integral_constant<int, 0>{}, wy - wy0);
    }
    if (wy1 == wy0 && item + p.G < p.items) request_item(item + p.G);
  }
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

}  // namespace

bool conv_fwd_fewch_applies(const ConvEngineArgs &a) {
  if (a.src_dz || a.w_flip || a.R != 3 || a.S != 3 || a.pad_h != 1 || a.pad_w != 1) return false;
  if (a.Cin > 3 || a.Kout > 16 || a.act != ACT_RELU || a.pool != 2) return false;
  if (a.Hout != a.Hin || a.Wout != a.Win || a.Win % 8 != 0 || a.Hin % 2 != 0 || a.Win >= (1 << 17)) return false;
  if (a.uniform || a.sample || a.out_pool) return false;
  if (!aligned16(a.src) || !aligned16(a.out) || (a.out_idx && (reinterpret_cast<uintptr_t>(a.out_idx) & 3u))) return false;
  const long limit = (1L << 31) - (1L << 24);
  return 4L * a.N * a.Cin * a.Hin * a.Win < limit && 4L * a.N * a.Kout * (a.Hin / 2) * (a.Win / 2) < limit;
}

hipError_t launch_conv_fwd_fewch(const ConvEngineArgs &a, hipStream_t stream) {
  if (!conv_fwd_fewch_applies(a)) return hipErrorInvalidValue;
  FwdFewchParams p;
  p.a = a;
  p.Hp = a.Hin / 2;
  p.Wp = a.Win / 2;
  p.xsegs = (a.Win + 63) / 64;
  p.xgroups = (p.xsegs + 3) / 4;
  p.x_bytes = (unsigned)(4L * a.N * a.Cin * a.Hin * a.Win);
  p.y_bytes = (unsigned)(4L * a.N * a.Kout * p.Hp * p.Wp);
  const long resident = 3L * chip().cus;   // three workgroups per compute unit (registers)
  // window rows per work item: the longest strip that still leaves every resident workgroup an item
  p.rg = 2;
  for (int rg = 16; rg >= 2; rg /= 2) {
    const long items = (long)a.N * p.xgroups * ((p.Hp + rg - 1) / rg);
    if (items >= resident || rg == 2) { p.rg = rg; break; }
  }
  p.rgroups = (p.Hp + p.rg - 1) / p.rg;
  const long items = (long)a.N * p.xgroups * p.rgroups;
  if (items <= 0 || items > 0x7fffffffL) return hipErrorInvalidValue;
  p.items = (int)items;
  p.G = (int)(items < resident ? items : resident);
  const size_t lds = sizeof(float) * 4 * kWaveFloats;
  if (a.out_idx) hipLaunchKernelGGL(conv_fwd_fewch_kernel<true>, dim3((unsigned)p.G), dim3(kThreads), lds, stream, p);
  else hipLaunchKernelGGL(conv_fwd_fewch_kernel<false>, dim3((unsigned)p.G), dim3(kThreads), lds, stream, p);
  return hipGetLastError();
}

}  // namespace dllk
