// Filter gradient of the padded 3x3 layers with 16 or 32 channels in and out behind ReLU + 2x2 max
// pooling in the minimal-filtering form F(3x3, 2x2): kernel entry and launcher (the kernel's body, with
// the description of the method, is in conv_wgrad_wino_body.h).
#include "conv_wgrad_wino_body.h"

namespace dllk {

namespace {

using namespace wgw;

template <int KT, int CT>
__global__ __launch_bounds__(kThreads, 2) void wgrad_wino_kernel(const WinoWgradParams p) {
  extern __shared__ float lds[];
  wgrad_wino_body<KT, CT>(p, lds, blockIdx.x);
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

}  // namespace

bool wgrad_wino_shape(int C, int H, int W, int K, int R, int S, int pad, int pool) {
  return R == 3 && S == 3 && pad == 1 && pool == 2 && (C == 16 || C == 32) && (K == 16 || K == 32) && W % 8 == 0 && H % 2 == 0;
}

bool wgrad_wino_applies(const WgradArgs &a, const WgradPlan &plan) {
  if (!wgrad_wino_shape(a.C, a.H, a.W, a.K, a.R, a.S, a.pad, a.pool)) return false;
  if (a.act != ACT_RELU_FLAGGED || !a.idx || a.W >= (1 << 17)) return false;
  if (plan.MTF * 16 != a.K || plan.NTT != 9 || plan.CC != 16 || plan.nchunks * 16 != a.C) return false;
  if (!aligned16(a.x) || !aligned16(a.dy) || (reinterpret_cast<uintptr_t>(a.idx) & 3u)) return false;
  const long limit = (1L << 31) - (1L << 24);
  return 4L * a.N * a.C * a.H * a.W < limit && 4L * a.N * a.K * (a.H / 2) * (a.W / 2) < limit;
}

hipError_t launch_wgrad_wino(const WgradArgs &a, const WgradPlan &plan, hipStream_t stream) {
  if (!wgrad_wino_applies(a, plan)) return hipErrorInvalidValue;
  WinoWgradParams p;
  if (!fill_wino_wgrad_params(a, plan, p)) return hipErrorInvalidValue;
  const int KT = a.K / 16, CT = a.C / 16;
  const size_t lds = kWinoWgradLdsBytes;
  const dim3 grid((unsigned)p.G), block(kThreads);
  if (KT == 1 && CT == 1) hipLaunchKernelGGL((wgrad_wino_kernel<1, 1>), grid, block, lds, stream, p);
  else if (KT == 2 && CT == 1) hipLaunchKernelGGL((wgrad_wino_kernel<2, 1>), grid, block, lds, stream, p);
  else if (KT == 1 && CT == 2) hipLaunchKernelGGL((wgrad_wino_kernel<1, 2>), grid, block, lds, stream, p);
  else hipLaunchKernelGGL((wgrad_wino_kernel<2, 2>), grid, block, lds, stream, p);
  return hipGetLastError();
}

}  // namespace dllk
