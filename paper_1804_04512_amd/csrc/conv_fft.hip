// Full convolution through the Fourier transform (Section II-A names this route for the backward
// pass: image and filter padded to the output size, transformed, multiplied point by point,
// transformed back; an image's transform is computed once and serves every filter).
//
//   dx[n,c] = crop_pad( sum_k  dz[n,k] (*) w[k,c] ),   (*) = true (filter-flipping) full convolution
//
// which is exactly the backward-data sum  dx[n,c,i,j] = sum_{k,r,s} dz[n,k,i+pad-r,j+pad-s] w[k,c,r,s].
// Here the padded size is the next power of two (at most 64 x 64, so a whole complex image fits in
// LDS): no wrap-around reaches the part that is kept.
//
//   fft2_forward_kernel    one workgroup per real image (a dz map, formed on the fly from the pooled
//                          gradient, the pooling bytes and the layer output exactly as the other
//                          backward kernels do, or a filter slice): rows, then columns, radix-2
//                          decimation in frequency, natural order in, bit-reversed order out;
//   fft2_product_inverse_kernel   one workgroup per (image n, channel c): sum over k of the
//                          products of the two spectra (both in the same bit-reversed order, so
//                          no reordering pass exists anywhere), then columns and rows back by
//                          decimation in time (bit-reversed in, natural out), scaled, cropped.
// The filters are real, so convolving is linear over the complex numbers with real coefficients:
// two images n, n+1 of the batch ride through all three stages as ONE complex signal
// dz[n] + i dz[n+1], and the real and imaginary parts of the result are dx[n] and dx[n+1].  That
// halves the image transforms, the products and the inverse transforms.
// All arithmetic is fp32; the result differs from the direct sum by rounding only (a few 1e-7 of
// the largest output).
#include "dll_internal.h"

namespace dllk {
namespace {

constexpr int kFftThreads = 256;
constexpr int kMaxLog = 6;                 // padded sides up to 64
constexpr int kTw = 1 << (kMaxLog - 1);    // twiddles exp(-2 pi i t / 64), t < 32

__device__ __forceinline__ float2 cmul(float2 a, float2 b) { return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x); }

__device__ __forceinline__ void make_twiddles(float2 *tw) {
  if (threadIdx.x < kTw) {
    float s, c;
    sincospif(-(float)threadIdx.x / (float)kTw, &s, &c);   // exp(-i pi t / 32) = exp(-2 pi i t / 64)
    tw[threadIdx.x] = make_float2(c, s);
  }
}

// One radix-2 pass over every line of the image along one axis.  `stride` separates consecutive
// elements of a line, `lstride` consecutive lines; consecutive threads take consecutive lines when
// the lines run down the columns (stride = PW), consecutive butterflies of a line otherwise.
// DIF (forward): a' = a + b, b' = (a - b) w.   DIT (inverse): t = b conj(w), a' = a + t, b' = a - t.
template <bool INVERSE>
__device__ __forceinline__ void fft_pass(float2 *buf, const float2 *tw, int len_log, int lines, int stride, int lstride,
                                         bool lines_fast, int stage) {
  const int half = 1 << (len_log - 1);
  const int span = INVERSE ? (1 << stage) : (half >> stage);
  const int total = lines * half;
  for (int b = threadIdx.x; b < total; b += kFftThreads) {
    const int line = lines_fast ? b % lines : b / half;
    const int q = lines_fast ? b / lines : b % half;
    const int group = q / span, j = q - group * span;
    const int i0 = line * lstride + (group * 2 * span + j) * stride, i1 = i0 + span * stride;
    float2 w = tw[j * (kTw / span)];
    const float2 a = buf[i0], c = buf[i1];
    if (INVERSE) {
      w.y = -w.y;
      const float2 t = cmul(c, w);
      buf[i0] = make_float2(a.x + t.x, a.y + t.y);
      buf[i1] = make_float2(a.x - t.x, a.y - t.y);
    } else {
      buf[i0] = make_float2(a.x + c.x, a.y + c.y);
      buf[i1] = cmul(make_float2(a.x - c.x, a.y - c.y), w);
    }
  }
  __syncthreads();
}

struct FftFwdArgs {
  const float *src;            // plain images [count][H][W], or dy of a layer
  const float *src_y;          // layer output (same shape as dy) where act' needs it
  const unsigned char *src_idx;
  int src_dz, src_act, src_pool;
  int count, H, W;             // real image size before padding (a dz map: pre-pool size)
  int pair_stride;             // > 0: workgroup g packs images g' and g' + pair_stride (the same filter map of
                               // two neighbouring batch images) as real and imaginary part; count = images given,
                               // planes = maps per batch image
  int planes;
  int lph, lpw;                // log2 of the padded sides
  float2 *out;                 // [count][PH * PW], bit-reversed order
};

__device__ __forceinline__ float act_deriv(int act, float out) {
  if (act == ACT_SIGMOID) return out * (1.0f - out);
  if (act == ACT_RELU) return out > 0.0f ? 1.0f : 0.0f;
  return 1.0f;
}

// dz = unpool(dy) * act'(y) at pre-pool position (i, j) of image `img`
__device__ __forceinline__ float fft_src_value(const FftFwdArgs &a, int img, int i, int j) {
  if (!a.src_dz) return a.src[((long)img * a.H + i) * a.W + j];
  long o;
  if (a.src_pool == 2) {
    o = ((long)img * (a.H >> 1) + (i >> 1)) * (a.W >> 1) + (j >> 1);
    const unsigned char f = a.src_idx[o];
    if ((f & kIdxPosMask) != (unsigned char)(((i & 1) << 1) | (j & 1))) return 0.0f;
    if (a.src_act == ACT_RELU_FLAGGED) return (f & kIdxInactive) ? 0.0f : a.src[o];
  } else {
    o = ((long)img * a.H + i) * a.W + j;
  }
  float g = a.src[o];
  if (a.src_act == ACT_SIGMOID || a.src_act == ACT_RELU) g *= act_deriv(a.src_act, a.src_y[o]);
  return g;
}

__global__ __launch_bounds__(kFftThreads) void fft2_forward_kernel(const FftFwdArgs a) {
  extern __shared__ float2 fbuf[];   // [PH * PW] + twiddles
  const int PH = 1 << a.lph, PW = 1 << a.lpw, F = PH * PW;
  float2 *tw = fbuf + F;
  // packed: workgroup (pair p, plane k) takes images (2p, k) and (2p + 1, k) of [N][planes]
  int img = blockIdx.x, img2 = -1;
  if (a.pair_stride > 0) {
    const int p = blockIdx.x / a.planes, k = blockIdx.x - p * a.planes;
    img = 2 * p * a.planes + k;
    img2 = img + a.pair_stride < a.count ? img + a.pair_stride : -1;
  }
  make_twiddles(tw);
  for (int e = threadIdx.x; e < F; e += kFftThreads) {
    const int i = e >> a.lpw, j = e & (PW - 1);
    const bool in = i < a.H && j < a.W;
    const float v = in ? fft_src_value(a, img, i, j) : 0.0f;
    const float v2 = (in && img2 >= 0) ? fft_src_value(a, img2, i, j) : 0.0f;
    fbuf[e] = make_float2(v, v2);
  }
  __syncthreads();
  for (int s = 0; s < a.lpw; ++s) fft_pass<false>(fbuf, tw, a.lpw, PH, 1, PW, false, s);   // along the rows
  for (int s = 0; s < a.lph; ++s) fft_pass<false>(fbuf, tw, a.lph, PW, PW, 1, true, s);    // down the columns
  float2 *dst = a.out + (long)blockIdx.x * F;
  for (int e = threadIdx.x; e < F; e += kFftThreads) dst[e] = fbuf[e];
}

struct FftInvArgs {
  const float2 *xf;   // [ceil(N/2)][K][F]: batch images 2p (real part) and 2p + 1 (imaginary part)
  const float2 *wf;   // [K][C][F]
  int N, K, C;
  int lph, lpw;
  int H, W, off;      // output size and the crop offset (the layer's padding)
  float *out;         // [N][C][H][W]
};

// PT pairs of batch images x CT channels per workgroup: every spectrum entry that is loaded serves
// PT (a filter's) or CT (an image's) products, which is what the product stage is bound by.
template <int PT, int CT>
__global__ __launch_bounds__(kFftThreads) void fft2_product_inverse_kernel(const FftInvArgs a) {
  extern __shared__ float2 fbuf[];
  const int PH = 1 << a.lph, PW = 1 << a.lpw, F = PH * PW;
  float2 *tw = fbuf + F;
  const int c0 = blockIdx.x * CT, pr0 = blockIdx.y * PT;
  const int pairs = (a.N + 1) / 2;
  make_twiddles(tw);
  constexpr int kSlots = (1 << (2 * kMaxLog)) / kFftThreads;   // 16 spectrum entries per thread at 64 x 64
  constexpr int kBatch = PT * CT > 1 ? kSlots / 2 : kSlots;    // entries whose loads are in flight together
  float2 acc[PT][CT][kSlots];
#pragma unroll
  for (int i = 0; i < PT; ++i)
#pragma unroll
    for (int j = 0; j < CT; ++j)
#pragma unroll
      for (int q = 0; q < kSlots; ++q) acc[i][j][q] = make_float2(0.0f, 0.0f);
  // surplus rows and columns of the last tiles re-read the last pair / channel and are never stored
  const float2 *xp[PT], *wp[CT];
#pragma unroll
  for (int i = 0; i < PT; ++i) xp[i] = a.xf + (long)min(pr0 + i, pairs - 1) * a.K * F;
#pragma unroll
  for (int j = 0; j < CT; ++j) wp[j] = a.wf + (long)min(c0 + j, a.C - 1) * F;
  for (int k = 0; k < a.K; ++k) {
#pragma unroll
    for (int h = 0; h < kSlots / kBatch; ++h) {
      // loads first, products after: entries past F re-read entry 0 and are never stored
      float2 xv[PT][kBatch], wv[CT][kBatch];
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        const int e = threadIdx.x + (h * kBatch + q) * kFftThreads;
        const int ec = e < F ? e : 0;
#pragma unroll
        for (int i = 0; i < PT; ++i) xv[i][q] = xp[i][(long)k * F + ec];
#pragma unroll
        for (int j = 0; j < CT; ++j) wv[j][q] = wp[j][(long)k * a.C * F + ec];
      }
#pragma unroll
      for (int q = 0; q < kBatch; ++q)
#pragma unroll
        for (int i = 0; i < PT; ++i)
#pragma unroll
          for (int j = 0; j < CT; ++j) {
            const float2 p = cmul(xv[i][q], wv[j][q]);
            acc[i][j][h * kBatch + q].x += p.x;
            acc[i][j][h * kBatch + q].y += p.y;
          }
    }
  }
  const float scale = 1.0f / (float)F;
  const long next = (long)a.C * a.H * a.W;   // the pair's second image
#pragma unroll
  for (int i = 0; i < PT; ++i)
#pragma unroll
    for (int j = 0; j < CT; ++j) {
      const int pr = pr0 + i, c = c0 + j, n = 2 * pr;
      if (pr >= pairs || c >= a.C) continue;   // uniform over the workgroup
#pragma unroll
      for (int q = 0; q < kSlots; ++q) {
        const int e = threadIdx.x + q * kFftThreads;
        if (e < F) fbuf[e] = acc[i][j][q];
      }
      __syncthreads();
      for (int s = 0; s < a.lph; ++s) fft_pass<true>(fbuf, tw, a.lph, PW, PW, 1, true, s);    // columns back
      for (int s = 0; s < a.lpw; ++s) fft_pass<true>(fbuf, tw, a.lpw, PH, 1, PW, false, s);   // rows back
      float *dst = a.out + ((long)n * a.C + c) * a.H * a.W;
      const bool two = n + 1 < a.N;
      for (int e = threadIdx.x; e < a.H * a.W; e += kFftThreads) {
        const int r = e / a.W, col = e - r * a.W;
        const float2 v = fbuf[((r + a.off) << a.lpw) + col + a.off];
        dst[e] = v.x * scale;
        if (two) dst[e + next] = v.y * scale;
      }
      __syncthreads();   // the image is read out before the next one overwrites it
    }
}

int log2_ceil(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

}  // namespace

bool conv_fft_plan(int Ho, int Wo, int R, int S, int *lph, int *lpw) {
  const int fh = Ho + R - 1, fw = Wo + S - 1;   // size of the full convolution
  if (fh < 1 || fw < 1 || fh > (1 << kMaxLog) || fw > (1 << kMaxLog)) return false;
  int a = log2_ceil(fh), b = log2_ceil(fw);
  if (a < 1) a = 1;
  if (b < 1) b = 1;
  *lph = a; *lpw = b;
  return true;
}

hipError_t launch_conv_full_fft(const ConvFftArgs &g, hipStream_t stream) {
  int lph, lpw;
  if (!conv_fft_plan(g.Ho, g.Wo, g.R, g.S, &lph, &lpw)) return hipErrorInvalidValue;
  const int F = 1 << (lph + lpw);
  const size_t lds = (size_t)(F + kTw) * sizeof(float2);
  FftFwdArgs x;
  x.src = g.dy; x.src_y = g.y; x.src_idx = g.idx;
  x.src_dz = 1; x.src_act = g.act; x.src_pool = g.pool;
  x.count = g.N * g.K; x.H = g.Ho; x.W = g.Wo; x.lph = lph; x.lpw = lpw;
  x.pair_stride = g.K; x.planes = g.K;
  x.out = g.xf;
  const int pairs = (g.N + 1) / 2;
  hipLaunchKernelGGL(fft2_forward_kernel, dim3(pairs * g.K), dim3(kFftThreads), lds, stream, x);
  FftFwdArgs f;
  f.src = g.w; f.src_y = nullptr; f.src_idx = nullptr;
  f.src_dz = 0; f.src_act = ACT_IDENTITY; f.src_pool = 1;
  f.count = g.K * g.C; f.H = g.R; f.W = g.S; f.lph = lph; f.lpw = lpw;
  f.pair_stride = 0; f.planes = 1;
  f.out = g.wf;
  hipLaunchKernelGGL(fft2_forward_kernel, dim3(f.count), dim3(kFftThreads), lds, stream, f);
  FftInvArgs v;
  v.xf = g.xf; v.wf = g.wf; v.N = g.N; v.K = g.K; v.C = g.C; v.lph = lph; v.lpw = lpw;
  v.H = g.H; v.W = g.W; v.off = g.pad; v.out = g.dx;
  // 2 x 2 tiles once there is enough work to fill the chip with them
  if ((long)pairs * g.C >= 4L * chip().cus)
    hipLaunchKernelGGL((fft2_product_inverse_kernel<2, 2>), dim3((g.C + 1) / 2, (pairs + 1) / 2), dim3(kFftThreads), lds, stream, v);
  else
    hipLaunchKernelGGL((fft2_product_inverse_kernel<1, 1>), dim3(g.C, pairs), dim3(kFftThreads), lds, stream, v);
  return hipGetLastError();
}

}  // namespace dllk
