// C ABI of the library: argument validation, workspace carving and the launch sequences of
// the single-layer calls, the CRBM CD-1 step and the CNN training step.  No kernel lives
// here and nothing is allocated: all scratch comes from the caller's workspace.
#include "../../include/dll_conv.h"
#include "dll_internal.h"

#include <stdint.h>

#include <mutex>
#include <utility>
#include <vector>

using namespace dllk;

namespace dllk {

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_chip_mutex;
ChipInfo g_chip[kMaxDevices];
bool g_chip_known[kMaxDevices];
std::vector<std::pair<int, const void *>> g_large_lds_done;
}  // namespace

// Asked once per device.  The library is built for gfx950 only; where no device answers (a
// workspace query on a machine without a GPU) the MI355X's published figures stand in: 256 compute
// units, 160 KB of LDS per compute unit.
const ChipInfo &chip() {
  static const ChipInfo mi355x{256, (size_t)160 * 1024};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return mi355x;
  }
  std::lock_guard<std::mutex> lock(g_chip_mutex);
  if (!g_chip_known[dev]) {
    int cus = 0, lds = 0;
    ChipInfo info = mi355x;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) info.cus = cus;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) == hipSuccess && lds >= 64 * 1024)
      info.lds_bytes = (size_t)lds;
    (void)hipGetLastError();
    g_chip[dev] = info;
    g_chip_known[dev] = true;
  }
  return g_chip[dev];
}

hipError_t allow_large_lds(const void *kernel, size_t lds_bytes) {
  if (lds_bytes <= 64 * 1024) return hipSuccess;
  const size_t limit = chip().lds_bytes;
  if (lds_bytes > limit) return hipErrorInvalidValue;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(g_chip_mutex);
  for (const auto &d : g_large_lds_done)
    if (d.first == dev && d.second == kernel) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)limit);
  if (e == hipSuccess) g_large_lds_done.emplace_back(dev, kernel);
  return e;
}

}  // namespace dllk

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Carver {
  char *base;
  size_t size, used;
  Carver(void *ws, size_t bytes) : base(static_cast<char *>(ws)), size(bytes), used(0) {}
  void *take(size_t bytes) {
    void *p = base ? base + used : nullptr;
    used += align_up(bytes);
    return p;
  }
  float *floats(size_t n) { return static_cast<float *>(take(n * sizeof(float))); }
};

inline int out_h(const dll_conv_desc *d) { return d->H + 2 * d->pad - d->R + 1; }
inline int out_w(const dll_conv_desc *d) { return d->W + 2 * d->pad - d->S + 1; }
inline size_t y_count(const dll_conv_desc *d) {
  return (size_t)d->N * d->K * (out_h(d) / d->pool) * (out_w(d) / d->pool);
}
inline size_t x_count(const dll_conv_desc *d) { return (size_t)d->N * d->C * d->H * d->W; }

dll_status check_desc(const dll_conv_desc *d, bool check_act_pool = true, bool check_taps = true) {
  if (!d) return DLL_ERR_NULL;
  if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0) return DLL_ERR_SHAPE;
  if (d->pad < 0 || d->pad > d->R - 1 || d->pad > d->S - 1) return DLL_ERR_SHAPE;
  const int Ho = out_h(d), Wo = out_w(d);
  if (Ho <= 0 || Wo <= 0) return DLL_ERR_SHAPE;
  if (check_act_pool) {
    if (d->act < DLL_ACT_IDENTITY || d->act > DLL_ACT_RELU) return DLL_ERR_UNSUPPORTED;
    if (d->pool != 1 && d->pool != 2) return DLL_ERR_UNSUPPORTED;
    if (d->pool == 2 && ((Ho & 1) || (Wo & 1))) return DLL_ERR_SHAPE;
  }
  const size_t lim = (size_t)1 << 31;
  if ((size_t)d->N * d->C * d->H * d->W >= lim || (size_t)d->N * d->K * Ho * Wo >= lim ||
      (size_t)d->K * d->C * d->R * d->S >= lim)
    return DLL_ERR_UNSUPPORTED;
  if (check_taps && d->R * d->S > 144) return DLL_ERR_UNSUPPORTED;  // filter-gradient kernel: at most 9 tap tiles per channel
  return DLL_OK;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

dll_status check_ws(const void *ws, size_t have, size_t need) {
  if (need == 0) return DLL_OK;
  if (!ws) return DLL_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & (kAlign - 1)) return DLL_ERR_WORKSPACE;
  return have >= need ? DLL_OK : DLL_ERR_WORKSPACE;
}

inline dll_status dev(hipError_t e) { return e == hipSuccess ? DLL_OK : DLL_ERR_DEVICE; }

ConvEngineArgs fwd_args(const dll_conv_desc *d, const float *x, const float *w, const float *bias, float *y,
                        unsigned char *idx) {
  ConvEngineArgs a;
  a.src = x;
  a.N = d->N; a.Cin = d->C; a.Hin = d->H; a.Win = d->W;
  a.w = w; a.w_flip = 0;
  a.Kout = d->K; a.R = d->R; a.S = d->S; a.pad_h = d->pad; a.pad_w = d->pad;
  a.Hout = out_h(d); a.Wout = out_w(d);
  a.bias = bias; a.act = d->act; a.pool = d->pool;
  a.out = y; a.out_idx = idx;
  return a;
}

// A pooled ReLU layer's backward passes may run without the layer output: the forward pass
// left the unit's activity in the pooling index.
inline bool flagged_relu(const dll_conv_desc *d, const float *y) {
  return !y && d->act == DLL_ACT_RELU && d->pool == 2;
}
inline bool output_required(const dll_conv_desc *d) {
  return d->act != DLL_ACT_IDENTITY && !(d->act == DLL_ACT_RELU && d->pool == 2);
}

// Backward-data as a forward-form convolution of dz (K channels at Ho x Wo) with the
// rotated, transposed filters on an input padded by R-1-pad (Section II-A's identity).
ConvEngineArgs bwd_args(const dll_conv_desc *d, const float *dy, const float *y, const unsigned char *idx,
                        const float *w, float *dx) {
  ConvEngineArgs a;
  a.src = dy; a.src_y = y; a.src_idx = idx;
  a.src_dz = 1; a.src_act = flagged_relu(d, y) ? ACT_RELU_FLAGGED : d->act; a.src_pool = d->pool;
  a.N = d->N; a.Cin = d->K; a.Hin = out_h(d); a.Win = out_w(d);
  a.w = w; a.w_flip = 1;
  a.Kout = d->C; a.R = d->R; a.S = d->S; a.pad_h = d->R - 1 - d->pad; a.pad_w = d->S - 1 - d->pad;
  a.Hout = d->H; a.Wout = d->W;
  a.act = ACT_IDENTITY; a.pool = 1;
  a.out = dx;
  return a;
}

WgradArgs wgrad_args(const dll_conv_desc *d, const float *x, const float *dy, const float *y,
                     const unsigned char *idx, float *partial) {
  WgradArgs a;
  a.x = x; a.dy = dy; a.y = y; a.idx = idx;
  a.act = flagged_relu(d, y) ? ACT_RELU_FLAGGED : d->act; a.pool = d->pool;
  a.N = d->N; a.C = d->C; a.H = d->H; a.W = d->W; a.K = d->K; a.R = d->R; a.S = d->S; a.pad = d->pad;
  a.partial = partial;
  return a;
}

bool plan_for(const dll_conv_desc *d, WgradPlan *plan) {
  return plan_wgrad(d->N, d->C, d->H, d->W, d->K, d->R, d->S, d->pad, d->pool, plan);
}

}  // namespace

extern "C" {

const char *dll_status_string(dll_status s) {
  switch (s) {
  case DLL_OK: return "ok";
  case DLL_ERR_NULL: return "required pointer is NULL";
  case DLL_ERR_SHAPE: return "invalid shape or aliasing";
  case DLL_ERR_UNSUPPORTED: return "unsupported configuration";
  case DLL_ERR_WORKSPACE: return "workspace too small or misaligned";
  case DLL_ERR_DEVICE: return "device launch failed";
  case DLL_ERR_SCRATCH_LIMIT: return "layer needs more scratch than the built-in array of the no-allocation entry point holds";
  }
  return "unknown status";
}

size_t dll_conv_workspace_bytes(const dll_conv_desc *d) {
  if (check_desc(d) != DLL_OK) return 0;
  WgradPlan plan;
  if (!plan_for(d, &plan)) return 0;
  return align_up(plan.partial_floats * sizeof(float));
}

dll_status dll_conv_valid_fwd(const dll_conv_desc *d, const float *x, const float *w, const float *bias, float *y,
                              unsigned char *pool_idx, void *ws, size_t ws_bytes, void *stream) {
  (void)ws; (void)ws_bytes;
  dll_status st = check_desc(d);
  if (st != DLL_OK) return st;
  if (!x || !w || !y || (d->pool == 2 && !pool_idx)) return DLL_ERR_NULL;
  if ((const float *)y == x || (const float *)y == w) return DLL_ERR_SHAPE;
  if (misaligned(x) || misaligned(w) || misaligned(y) || misaligned(pool_idx)) return DLL_ERR_SHAPE;
  return dev(launch_conv_engine(fwd_args(d, x, w, bias, y, pool_idx), static_cast<hipStream_t>(stream)));
}

dll_status dll_conv_full_bwd(const dll_conv_desc *d, const float *dy, const float *y, const unsigned char *pool_idx,
                             const float *w, float *dx, void *ws, size_t ws_bytes, void *stream) {
  (void)ws; (void)ws_bytes;
  dll_status st = check_desc(d);
  if (st != DLL_OK) return st;
  if (!dy || !w || !dx || (output_required(d) && !y) || (d->pool == 2 && !pool_idx)) return DLL_ERR_NULL;
  if ((const float *)dx == dy || (const float *)dx == y || (const float *)dx == w) return DLL_ERR_SHAPE;
  if (misaligned(dy) || misaligned(y) || misaligned(w) || misaligned(dx) || misaligned(pool_idx)) return DLL_ERR_SHAPE;
  return dev(launch_conv_engine(bwd_args(d, dy, y, pool_idx, w, dx), static_cast<hipStream_t>(stream)));
}

size_t dll_conv_full_fft_workspace_bytes(const dll_conv_desc *d) {
  if (check_desc(d, true, false) != DLL_OK) return 0;
  int lph, lpw;
  if (!conv_fft_plan(out_h(d), out_w(d), d->R, d->S, &lph, &lpw)) return 0;
  const size_t F = (size_t)1 << (lph + lpw);
  Carver c(nullptr, 0);
  c.take((size_t)((d->N + 1) / 2) * d->K * F * sizeof(float2));   // two batch images per complex image
  c.take((size_t)d->K * d->C * F * sizeof(float2));
  return c.used;
}

dll_status dll_conv_full_bwd_fft(const dll_conv_desc *d, const float *dy, const float *y, const unsigned char *pool_idx,
                                 const float *w, float *dx, void *ws, size_t ws_bytes, void *stream) {
  dll_status st = check_desc(d, true, false);   // any filter size the transform can hold
  if (st != DLL_OK) return st;
  if (!dy || !w || !dx || (output_required(d) && !y) || (d->pool == 2 && !pool_idx)) return DLL_ERR_NULL;
  if ((const float *)dx == dy || (const float *)dx == y || (const float *)dx == w) return DLL_ERR_SHAPE;
  int lph, lpw;
  if (!conv_fft_plan(out_h(d), out_w(d), d->R, d->S, &lph, &lpw)) return DLL_ERR_UNSUPPORTED;
  st = check_ws(ws, ws_bytes, dll_conv_full_fft_workspace_bytes(d));
  if (st != DLL_OK) return st;
  const size_t F = (size_t)1 << (lph + lpw);
  Carver c(ws, ws_bytes);
  ConvFftArgs a;
  a.dy = dy; a.y = y; a.idx = pool_idx;
  a.act = flagged_relu(d, y) ? ACT_RELU_FLAGGED : d->act; a.pool = d->pool;
  a.N = d->N; a.K = d->K; a.C = d->C; a.Ho = out_h(d); a.Wo = out_w(d); a.R = d->R; a.S = d->S;
  a.H = d->H; a.W = d->W; a.pad = d->pad;
  a.w = w; a.dx = dx;
  a.xf = static_cast<float2 *>(c.take((size_t)((d->N + 1) / 2) * d->K * F * sizeof(float2)));
  a.wf = static_cast<float2 *>(c.take((size_t)d->K * d->C * F * sizeof(float2)));
  return dev(launch_conv_full_fft(a, static_cast<hipStream_t>(stream)));
}

dll_status dll_conv_valid_wgrad_partial(const dll_conv_desc *d, const float *x, const float *dy, const float *y,
                                        const unsigned char *pool_idx, void *ws, size_t ws_bytes, void *stream) {
  dll_status st = check_desc(d);
  if (st != DLL_OK) return st;
  if (!x || !dy || (output_required(d) && !y) || (d->pool == 2 && !pool_idx)) return DLL_ERR_NULL;
  if (misaligned(x) || misaligned(dy) || misaligned(y)) return DLL_ERR_SHAPE;
  WgradPlan plan;
  if (!plan_for(d, &plan)) return DLL_ERR_UNSUPPORTED;
  st = check_ws(ws, ws_bytes, align_up(plan.partial_floats * sizeof(float)));
  if (st != DLL_OK) return st;
  return dev(launch_wgrad(wgrad_args(d, x, dy, y, pool_idx, static_cast<float *>(ws)), plan, static_cast<hipStream_t>(stream)));
}

dll_status dll_conv_valid_wgrad_finish(const dll_conv_desc *d, float *dw, float *dbias, const void *ws, size_t ws_bytes,
                                       void *stream) {
  dll_status st = check_desc(d);
  if (st != DLL_OK) return st;
  if (!dw) return DLL_ERR_NULL;
  if (misaligned(dw)) return DLL_ERR_SHAPE;
  WgradPlan plan;
  if (!plan_for(d, &plan)) return DLL_ERR_UNSUPPORTED;
  st = check_ws(ws, ws_bytes, align_up(plan.partial_floats * sizeof(float)));
  if (st != DLL_OK) return st;
  if (static_cast<const void *>(dw) == ws) return DLL_ERR_SHAPE;
  WgradReduceArgs r;
  r.pos = static_cast<const float *>(ws); r.scale = 1.0f; r.dw = dw; r.db = dbias;
  r.C = d->C; r.K = d->K; r.R = d->R; r.S = d->S;
  return dev(launch_wgrad_reduce(r, plan, static_cast<hipStream_t>(stream)));
}

dll_status dll_conv_valid_wgrad(const dll_conv_desc *d, const float *x, const float *dy, const float *y,
                                const unsigned char *pool_idx, float *dw, float *dbias, void *ws, size_t ws_bytes,
                                void *stream) {
  dll_status st = check_desc(d);
  if (st != DLL_OK) return st;
  if (!x || !dy || !dw || (output_required(d) && !y) || (d->pool == 2 && !pool_idx)) return DLL_ERR_NULL;
  if ((const float *)dw == x || (const float *)dw == dy || (const float *)dw == y) return DLL_ERR_SHAPE;
  if (misaligned(dw)) return DLL_ERR_SHAPE;
  st = dll_conv_valid_wgrad_partial(d, x, dy, y, pool_idx, ws, ws_bytes, stream);
  if (st != DLL_OK) return st;
  return dll_conv_valid_wgrad_finish(d, dw, dbias, ws, ws_bytes, stream);
}

// ---- the filter gradient for callers that cannot allocate: same kernels, the partial sums live in
// a file-scope device array instead of a caller workspace.  Every GPU the library runs on holds its
// own copy of the array (at its own address) until the process ends.
}  // extern "C"

namespace {
constexpr size_t kScratchBytes = DLL_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
std::mutex g_scratch_mutex;
void *g_scratch_ptr[64];   // per device: the array's device address, asked of the runtime once

// The array's name is a host-side stand-in for the symbol, not a device address: host code only
// ever uses the address the runtime returns for the current device.
dll_status scratch_of_current_device(void **out) {
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) return DLL_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return DLL_ERR_DEVICE;
    }
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return DLL_OK;
}
}  // namespace

extern "C" {

dll_status dll_conv_valid_wgrad_noalloc(const dll_conv_desc *d, const float *x, const float *dy, const float *y,
                                        const unsigned char *pool_idx, float *dw, float *dbias, void *stream) {
  dll_status st = check_desc(d);
  if (st != DLL_OK) return st;
  WgradPlan plan;
  if (!plan_for(d, &plan)) return DLL_ERR_UNSUPPORTED;
  if (align_up(plan.partial_floats * sizeof(float)) > kScratchBytes) return DLL_ERR_SCRATCH_LIMIT;
  void *ptr = nullptr;
  st = scratch_of_current_device(&ptr);
  if (st != DLL_OK) return st;
  // every partial sum the reduction reads is written by the first kernel of this call: nothing in
  // the array has to start at zero, and what an earlier (larger) call left behind is never read
  return dll_conv_valid_wgrad(d, x, dy, y, pool_idx, dw, dbias, ptr, kScratchBytes, stream);
}

size_t dll_crbm_workspace_bytes(const dll_conv_desc *d) {
  if (check_desc(d, false) != DLL_OK) return 0;
  WgradPlan plan;
  if (!plan_for(d, &plan)) return 0;
  dll_conv_desc t = *d;
  t.pool = 1;
  Carver c(nullptr, 0);
  c.floats(y_count(&t)); c.floats(y_count(&t)); c.floats(y_count(&t));  // h0p, h0s, h1p
  c.floats(x_count(&t));                                                // v1
  c.floats(plan.partial_floats); c.floats(plan.partial_floats);
  c.floats(visible_stats_scratch_floats(d->N, d->C, d->H * d->W));
  return c.used;
}

dll_status dll_crbm_cd1_step_units(const dll_conv_desc *din, int visible, int hidden_pool, const float *v0, float *W,
                                   float *b_hid, float *c_vis, const float *uniform, const float *h0_sample_in, float lr,
                                   float *dW, float *db, float *dc, float *h0_prob, float *h0_sample, float *pool_prob,
                                   float *v1, float *h1_prob, float *recon_mse, void *ws, size_t ws_bytes, void *stream) {
  dll_status st = check_desc(din, false);
  if (st != DLL_OK) return st;
  if (!v0 || !W || !b_hid || !c_vis || !dW || !db || !dc || (!uniform && !h0_sample_in)) return DLL_ERR_NULL;
  if (dW == W || db == b_hid || dc == c_vis || (const float *)v1 == v0) return DLL_ERR_SHAPE;
  if ((visible != DLL_VISIBLE_BINARY && visible != DLL_VISIBLE_GAUSSIAN) || (hidden_pool != 1 && hidden_pool != 2))
    return DLL_ERR_SHAPE;
  dll_conv_desc d = *din;
  d.act = DLL_ACT_SIGMOID;
  d.pool = 1;
  const bool pmp = hidden_pool == 2;
  if (pmp && ((out_h(&d) & 1) || (out_w(&d) & 1))) return DLL_ERR_SHAPE;
  if (pool_prob && !pmp) return DLL_ERR_SHAPE;
  if (misaligned(v0) || misaligned(W) || misaligned(uniform) || misaligned(h0_sample_in) || misaligned(dW) ||
      misaligned(h0_prob) || misaligned(h0_sample) || misaligned(v1) || misaligned(h1_prob) || misaligned(pool_prob))
    return DLL_ERR_SHAPE;
  WgradPlan plan;
  if (!plan_for(&d, &plan)) return DLL_ERR_UNSUPPORTED;
  st = check_ws(ws, ws_bytes, dll_crbm_workspace_bytes(din));
  if (st != DLL_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  Carver c(ws, ws_bytes);
  const size_t nh = y_count(&d), nv = x_count(&d);
  float *h0p_ws = c.floats(nh), *h0s_ws = c.floats(nh), *h1p_ws = c.floats(nh), *v1_ws = c.floats(nv);
  float *part_pos = c.floats(plan.partial_floats), *part_neg = c.floats(plan.partial_floats);
  float *stats = c.floats(visible_stats_scratch_floats(d.N, d.C, d.H * d.W));
  float *h0p = h0_prob ? h0_prob : h0p_ws;
  float *h0s = h0_sample ? h0_sample : h0s_ws;
  float *h1p = h1_prob ? h1_prob : h1p_ws;
  float *v1p = v1 ? v1 : v1_ws;
  const int hid_act = pmp ? ACT_PMP : ACT_SIGMOID;

  // positive phase: hidden probabilities (+ the sampled states in the same epilogue)
  ConvEngineArgs f0 = fwd_args(&d, v0, W, b_hid, h0p, nullptr);
  f0.act = hid_act;
  f0.out_pool = pool_prob;
  if (!h0_sample_in) { f0.uniform = uniform; f0.sample = h0s; }
  if ((st = dev(launch_conv_engine(f0, s))) != DLL_OK) return st;
  const float *hs = h0s;
  if (h0_sample_in) {
    hs = h0_sample_in;
    if (h0_sample && (st = dev(launch_copy(h0_sample_in, h0_sample, nh, s))) != DLL_OK) return st;
  }
  // reconstruction: full convolution of the states, + c, then the visible unit's mean
  ConvEngineArgs rec = bwd_args(&d, hs, nullptr, nullptr, W, v1p);
  rec.src_dz = 0;
  rec.bias = c_vis;
  rec.act = visible == DLL_VISIBLE_BINARY ? ACT_SIGMOID : ACT_IDENTITY;
  if ((st = dev(launch_conv_engine(rec, s))) != DLL_OK) return st;
  // negative phase hidden probabilities
  ConvEngineArgs f1 = fwd_args(&d, v1p, W, b_hid, h1p, nullptr);
  f1.act = hid_act;
  if ((st = dev(launch_conv_engine(f1, s))) != DLL_OK) return st;
  // statistics: filter gradients with dz := hidden probabilities
  dll_conv_desc di = d;
  di.act = DLL_ACT_IDENTITY;
  if ((st = dev(launch_wgrad(wgrad_args(&di, v0, h0p, nullptr, nullptr, part_pos), plan, s))) != DLL_OK) return st;
  if ((st = dev(launch_wgrad(wgrad_args(&di, v1p, h1p, nullptr, nullptr, part_neg), plan, s))) != DLL_OK) return st;
  const float invB = 1.0f / (float)d.N;
  WgradReduceArgs r;
  r.pos = part_pos; r.neg = part_neg; r.scale = invB; r.dw = dW; r.db = db;
  r.C = d.C; r.K = d.K; r.R = d.R; r.S = d.S;
  if (lr != 0.0f) { r.w_update = W; r.b_update = b_hid; r.step = lr; }
  if ((st = dev(launch_wgrad_reduce(r, plan, s))) != DLL_OK) return st;
  return dev(launch_visible_stats(v0, v1p, d.N, d.C, d.H * d.W, invB, dc, recon_mse, lr != 0.0f ? c_vis : nullptr, lr,
                                  stats, s));
}

dll_status dll_crbm_cd1_step(const dll_conv_desc *d, const float *v0, float *W, float *b_hid, float *c_vis,
                             const float *uniform, const float *h0_sample_in, float lr, float *dW, float *db, float *dc,
                             float *h0_prob, float *h0_sample, float *v1, float *h1_prob, float *recon_mse, void *ws,
                             size_t ws_bytes, void *stream) {
  return dll_crbm_cd1_step_units(d, DLL_VISIBLE_BINARY, 1, v0, W, b_hid, c_vis, uniform, h0_sample_in, lr, dW, db, dc,
                                 h0_prob, h0_sample, nullptr, v1, h1_prob, recon_mse, ws, ws_bytes, stream);
}

namespace {
// split-K partial area the three batch-by-units products of the RBM step need at most
size_t rbm_partial_floats(int B, int nv, int nh) {
  const size_t a = (size_t)gemm_pick_split_k(B, nh, nv) * B * nh, b = (size_t)gemm_pick_split_k(B, nv, nh) * B * nv;
  return a > b ? a : b;
}
bool rbm_sizes_ok(int B, int nv, int nh) {
  return B > 0 && nv > 0 && nh > 0 && (size_t)nv * nh < ((size_t)1 << 31) && (size_t)2 * B * nv < ((size_t)1 << 31) &&
         (size_t)2 * B * nh < ((size_t)1 << 31);
}
}  // namespace

size_t dll_rbm_workspace_bytes(int batch, int n_vis, int n_hid) {
  if (!rbm_sizes_ok(batch, n_vis, n_hid)) return 0;
  const size_t nH = (size_t)batch * n_hid, nV = (size_t)batch * n_vis;
  Carver c(nullptr, 0);
  c.floats(nH); c.floats(nH); c.floats(nH);      // h0p, h0s, h1p
  c.floats(2 * nH); c.floats(2 * nV);            // stacked hidden probabilities, stacked visibles
  c.floats(rbm_partial_floats(batch, n_vis, n_hid));
  c.floats(rbm_visible_scratch_floats(n_vis));
  return c.used;
}

dll_status dll_rbm_cd1_step(int batch, int n_vis, int n_hid, int visible, const float *v0, float *W, float *b_hid,
                            float *c_vis, const float *uniform, const float *h0_sample_in, float lr, float *dW, float *db,
                            float *dc, float *h0_prob, float *h0_sample, float *v1, float *h1_prob, float *recon_mse,
                            void *ws, size_t ws_bytes, void *stream) {
  if (batch <= 0 || n_vis <= 0 || n_hid <= 0) return DLL_ERR_SHAPE;
  if (!rbm_sizes_ok(batch, n_vis, n_hid)) return DLL_ERR_UNSUPPORTED;
  if (visible != DLL_VISIBLE_BINARY && visible != DLL_VISIBLE_GAUSSIAN) return DLL_ERR_SHAPE;
  if (!v0 || !W || !b_hid || !c_vis || !dW || !db || !dc || (!uniform && !h0_sample_in)) return DLL_ERR_NULL;
  if (dW == W || db == b_hid || dc == c_vis || (const float *)v1 == v0) return DLL_ERR_SHAPE;
  if (misaligned(v0) || misaligned(W) || misaligned(uniform) || misaligned(h0_sample_in) || misaligned(dW) ||
      misaligned(h0_prob) || misaligned(h0_sample) || misaligned(v1) || misaligned(h1_prob))
    return DLL_ERR_SHAPE;
  dll_status st = check_ws(ws, ws_bytes, dll_rbm_workspace_bytes(batch, n_vis, n_hid));
  if (st != DLL_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int B = batch, nv = n_vis, nh = n_hid;
  const size_t nH = (size_t)B * nh, nV = (size_t)B * nv;
  Carver c(ws, ws_bytes);
  float *h0p_ws = c.floats(nH), *h0s_ws = c.floats(nH), *h1p_ws = c.floats(nH);
  float *hstack = c.floats(2 * nH), *vstack = c.floats(2 * nV);
  float *partial = c.floats(rbm_partial_floats(B, nv, nh));
  float *stats = c.floats(rbm_visible_scratch_floats(nv));
  float *h0p = h0_prob ? h0_prob : h0p_ws;
  float *h0s = h0_sample ? h0_sample : h0s_ws;
  float *h1p = h1_prob ? h1_prob : h1p_ws;
  float *v1p = vstack + nV;   // the reconstruction is produced in place as the lower half of the stack

  // hidden probabilities of a visible batch: sigmoid(b_hid + v W^T)
  auto hidden = [&](const float *v, float *out) {
    GemmArgs g;
    g.M = B; g.N = nh; g.Kdim = nv;
    g.A = v; g.a_m = nv; g.a_k = 1;
    g.B = W; g.b_k = 1; g.b_n = nv;
    g.bias = b_hid; g.act = ACT_SIGMOID;
    g.Cout = out; g.c_m = nh; g.c_n = 1;
    g.split_k = gemm_pick_split_k(g.M, g.N, g.Kdim);
    g.partial = partial;
    return dev(launch_gemm(g, s));
  };
  if ((st = hidden(v0, h0p)) != DLL_OK) return st;
  const float *hs = h0s;
  if (h0_sample_in) {
    hs = h0_sample_in;
    if (h0_sample && (st = dev(launch_copy(h0_sample_in, h0_sample, nH, s))) != DLL_OK) return st;
  } else if ((st = dev(launch_bernoulli(h0p, uniform, h0s, nH, s))) != DLL_OK) {
    return st;
  }
  {
    // reconstruction: c_vis + h0s W, then the visible unit's mean
    GemmArgs g;
    g.M = B; g.N = nv; g.Kdim = nh;
    g.A = hs; g.a_m = nh; g.a_k = 1;
    g.B = W; g.b_k = nv; g.b_n = 1;
    g.bias = c_vis; g.act = visible == DLL_VISIBLE_BINARY ? ACT_SIGMOID : ACT_IDENTITY;
    g.Cout = v1p; g.c_m = nv; g.c_n = 1;
    g.split_k = gemm_pick_split_k(g.M, g.N, g.Kdim);
    g.partial = partial;
    if ((st = dev(launch_gemm(g, s))) != DLL_OK) return st;
  }
  if ((st = hidden(v1p, h1p)) != DLL_OK) return st;
  if (v1 && (st = dev(launch_copy(v1p, v1, nV, s))) != DLL_OK) return st;
  // statistics: with the phases stacked along the batch axis (signs and 1/B folded into the hidden
  // half), dW is ONE product over 2B rows and db one column sum; the updates ride in their epilogues
  const float invB = 1.0f / (float)B;
  if ((st = dev(launch_copy(v0, vstack, nV, s))) != DLL_OK) return st;
  if ((st = dev(launch_rbm_stack(h0p, h1p, invB, hstack, nH, s))) != DLL_OK) return st;
  if ((st = dev(launch_rbm_visible_stats(v0, v1p, B, nv, invB, dc, recon_mse, lr != 0.0f ? c_vis : nullptr, lr, stats, s))) !=
      DLL_OK)
    return st;
  if ((st = dev(launch_colsum(hstack, 2 * B, nh, db, lr != 0.0f ? b_hid : nullptr, lr, nullptr, 0.0f, s))) != DLL_OK) return st;
  GemmArgs g;
  g.M = nh; g.N = nv; g.Kdim = 2 * B;
  g.A = hstack; g.a_m = 1; g.a_k = nh;
  g.B = vstack; g.b_k = nv; g.b_n = 1;
  g.Cout = dW; g.c_m = nv; g.c_n = 1;
  if (lr != 0.0f) { g.update = W; g.step = lr; }
  g.split_k = 1;
  return dev(launch_gemm(g, s));
}

}  // extern "C"

// ---------------------------------------------------------------------------------------
// CNN training step
// ---------------------------------------------------------------------------------------
namespace {

struct NetLayout {
  size_t total = 0;
  size_t gmax = 0;       // floats of the largest gradient tensor passed between layers
  size_t partial = 0;    // floats of the largest partial-sum area
  int B = 0;
};

dll_status check_net(const dll_net_desc *net, NetLayout *lay) {
  if (!net || !net->dense || (net->n_conv > 0 && !net->conv)) return DLL_ERR_NULL;
  if (net->n_conv < 0 || net->n_dense < 1 || net->classes < 1) return DLL_ERR_SHAPE;
  // a network without convolution layers is fully connected: its batch size is given, and its
  // input rows are as long as the first dense layer's input
  const int B = net->n_conv > 0 ? net->conv[0].N : net->batch;
  if (B < 1) return DLL_ERR_SHAPE;
  size_t feat = net->n_conv > 0 ? 0 : (size_t)(net->dense[0].in > 0 ? net->dense[0].in : 0), gmax = 0, partial = 0;
  for (int l = 0; l < net->n_conv; ++l) {
    const dll_conv_desc *d = &net->conv[l];
    dll_status st = check_desc(d);
    if (st != DLL_OK) return st;
    if (d->N != B) return DLL_ERR_SHAPE;
    if (l > 0) {
      const dll_conv_desc *q = &net->conv[l - 1];
      if (d->C != q->K || d->H != out_h(q) / q->pool || d->W != out_w(q) / q->pool) return DLL_ERR_SHAPE;
          if (x_count(d) > gmax) gmax = x_count(d);
    }
    if (y_count(d) > gmax) gmax = y_count(d);
    WgradPlan plan;
    if (!plan_for(d, &plan)) return DLL_ERR_UNSUPPORTED;
    feat = y_count(d) / B;
  }
  for (int q = 0; q < net->n_dense; ++q) {
    const dll_dense_desc *dd = &net->dense[q];
    if (dd->in <= 0 || dd->out <= 0) return DLL_ERR_SHAPE;
    if ((size_t)dd->in != feat) return DLL_ERR_SHAPE;
    if (q < net->n_dense - 1 && (dd->act < DLL_ACT_IDENTITY || dd->act > DLL_ACT_RELU)) return DLL_ERR_UNSUPPORTED;
    if ((size_t)dd->in * dd->out >= ((size_t)1 << 31)) return DLL_ERR_UNSUPPORTED;
    const size_t gi = (size_t)B * dd->in, go = (size_t)B * dd->out;
    if (gi > gmax) gmax = gi;
    if (go > gmax) gmax = go;
    size_t p;
    p = (size_t)gemm_pick_split_k(B, dd->out, dd->in) * B * dd->out;      // forward
    if (p > partial) partial = p;
    p = (size_t)gemm_pick_split_k(B, dd->in, dd->out) * B * dd->in;       // backward data
    if (p > partial) partial = p;
    feat = dd->out;
  }
  if ((int)feat != net->classes) return DLL_ERR_SHAPE;
  lay->gmax = gmax;
  lay->partial = partial;
  lay->B = B;
  return DLL_OK;
}

struct NetBuffers {
  float *act[64];
  unsigned char *idx[32];
  float *gbuf[2];
  float *rowloss;
  float *partial;        // split-K partials of the dense products
  float *cpartial[32];   // per conv layer: filter-gradient partial blocks (reduced by the step's closing kernel)
  float *dz[32];         // per dense layer: dz of that layer (kept until the closing kernel sums the bias gradients)
};

size_t carve_net(const dll_net_desc *net, const NetLayout &lay, void *ws, NetBuffers *nb) {
  Carver c(ws, 0);
  const int L = net->n_conv, D = net->n_dense;
  for (int l = 0; l < L; ++l) {
    nb->act[l + 1] = c.floats(y_count(&net->conv[l]));
    nb->idx[l] = static_cast<unsigned char *>(c.take(y_count(&net->conv[l])));
  }
  for (int q = 0; q < D; ++q) nb->act[L + q + 1] = c.floats((size_t)lay.B * net->dense[q].out);
  nb->gbuf[0] = c.floats(lay.gmax);
  nb->gbuf[1] = c.floats(lay.gmax);
  nb->rowloss = c.floats(lay.B);
  nb->partial = c.floats(lay.partial);
  for (int l = 0; l < L; ++l) {
    WgradPlan plan;
    nb->cpartial[l] = plan_for(&net->conv[l], &plan) ? c.floats(plan.partial_floats) : nullptr;
  }
  for (int q = 0; q < D; ++q) nb->dz[q] = c.floats((size_t)lay.B * net->dense[q].out);
  return c.used;
}

}  // namespace

extern "C" {

size_t dll_cnn_workspace_bytes(const dll_net_desc *net) {
  NetLayout lay;
  if (check_net(net, &lay) != DLL_OK) return 0;
  if (net->n_conv > 31 || net->n_conv + net->n_dense > 62) return 0;
  NetBuffers nb;
  return carve_net(net, lay, nullptr, &nb);
}

}  // extern "C"

namespace {

// One training step; `velocity` (nullable) switches the updates to momentum + weight decay.
dll_status run_cnn_step(const dll_net_desc *net, float *const *params, float *const *velocity, float *const *grads,
                        const float *x, const int *labels, float lr, float mu, float decay, float *loss, float *logits,
                        unsigned char *const *pool_idx, void *ws, size_t ws_bytes, void *stream) {
  NetLayout lay;
  dll_status st = check_net(net, &lay);
  if (st != DLL_OK) return st;
  const int L = net->n_conv, D = net->n_dense, B = lay.B;
  if (L > 31 || L + D > 62) return DLL_ERR_UNSUPPORTED;
  if (!params || !x || !labels || !loss) return DLL_ERR_NULL;
  for (int p = 0; p < 2 * (L + D); ++p) {
    if (!params[p]) return DLL_ERR_NULL;
    if (misaligned(params[p]) || (grads && misaligned(grads[p]))) return DLL_ERR_SHAPE;
    if (grads && grads[p] == params[p]) return DLL_ERR_SHAPE;
    if (velocity) {
      if (!velocity[p]) return DLL_ERR_NULL;
      if (misaligned(velocity[p]) || velocity[p] == params[p] || (grads && grads[p] == velocity[p])) return DLL_ERR_SHAPE;
    }
  }
  if (misaligned(x) || misaligned(logits)) return DLL_ERR_SHAPE;
  NetBuffers nb;
  const size_t need = carve_net(net, lay, ws, &nb);
  st = check_ws(ws, ws_bytes, need);
  if (st != DLL_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const float step = -lr;
  const bool upd = lr != 0.0f;

  for (int l = 0; l < L; ++l)
    if (pool_idx && pool_idx[l] && net->conv[l].pool == 2) {
      if (misaligned(pool_idx[l])) return DLL_ERR_SHAPE;
      nb.idx[l] = pool_idx[l];
    }

  // ---- forward
  nb.act[0] = const_cast<float *>(x);
  for (int l = 0; l < L; ++l) {
    const dll_conv_desc *d = &net->conv[l];
    st = dev(launch_conv_engine(fwd_args(d, nb.act[l], params[2 * l], params[2 * l + 1], nb.act[l + 1], nb.idx[l]), s));
    if (st != DLL_OK) return st;
  }
  if (logits) nb.act[L + D] = logits;
  int logits_split = 1;
  bool loss_fused = false;
  for (int q = 0; q < D; ++q) {
    const dll_dense_desc *dd = &net->dense[q];
    GemmArgs g;
    g.M = B; g.N = dd->out; g.Kdim = dd->in;
    g.A = nb.act[L + q]; g.a_m = dd->in; g.a_k = 1;
    g.B = params[2 * (L + q)]; g.b_k = 1; g.b_n = dd->in;
    g.bias = params[2 * (L + q) + 1];
    g.act = (q == D - 1) ? ACT_IDENTITY : dd->act;
    g.Cout = nb.act[L + q + 1]; g.c_m = dd->out; g.c_n = 1;
    g.split_k = gemm_pick_split_k(g.M, g.N, g.Kdim);
    g.partial = nb.partial;
    // the logits' split-K partials are added by the loss kernel, which reads them anyway
    if (q == D - 1 && g.split_k > 1) { g.defer_reduce = true; logits_split = g.split_k; }
    // few classes and a small product: the loss rides in the product's epilogue
    if (q == D - 1 && gemm_fuses_softmax(g.M, g.N, g.Kdim)) {
      g.sm_labels = labels; g.sm_dz = nb.dz[D - 1]; g.sm_rowloss = nb.rowloss; g.sm_scale = 1.0f / (float)B;
      loss_fused = true;
    }
    if ((st = dev(launch_gemm(g, s))) != DLL_OK) return st;
  }
  // ---- loss
  // Reductions that nothing later in the step waits for (filter-gradient reductions with the
  // filter updates, dense bias gradients, the mean loss) are collected as jobs of one closing
  // launch; a full job list is flushed on the spot, which keeps the order of the plain sequence.
  StepTail tail;
  auto flush_tail = [&]() -> dll_status {
    const dll_status r = dev(launch_step_tail(tail, s));
    tail = StepTail{};
    return r;
  };
  tail.rowloss = nb.rowloss; tail.rows = B; tail.loss = loss;
  if (!loss_fused) {
    st = dev(launch_softmax_ce(nb.act[L + D], labels, B, net->classes, nullptr, nb.dz[D - 1], nb.rowloss,
                               logits_split > 1 ? nb.partial : nullptr, logits_split, params[2 * (L + D - 1) + 1], s));
    if (st != DLL_OK) return st;
  }
  // ---- dense backward: data gradient first (old weights), then weight gradient + update
  GemmArgs pending;
  bool have_pending = false;
  for (int q = D - 1; q >= 0; --q) {
    const dll_dense_desc *dd = &net->dense[q];
    // dz[q] is dz of layer q: the loss kernel wrote it for the top layer, and each data-gradient
    // product below multiplies by the next lower layer's act' on its way out
    float *Wq = params[2 * (L + q)], *bq = params[2 * (L + q) + 1];
    float *gcur = nb.dz[q], *gnext = q > 0 ? nb.dz[q - 1] : nb.gbuf[0];
    GemmArgs g;
    g.M = B; g.N = dd->in; g.Kdim = dd->out;
    g.A = gcur; g.a_m = dd->out; g.a_k = 1;
    g.B = Wq; g.b_k = dd->in; g.b_n = 1;
    g.Cout = gnext; g.c_m = dd->in; g.c_n = 1;
    if (q > 0 && net->dense[q - 1].act != DLL_ACT_IDENTITY) { g.C_ref = nb.act[L + q]; g.c_ref_act = net->dense[q - 1].act; }
    g.split_k = gemm_pick_split_k(g.M, g.N, g.Kdim);
    g.partial = nb.partial;
    if (g.split_k > 1 && gemm_prefers_small(g)) { g.split_k = 1; g.small_form = true; }
    // the gradient with respect to the network input has no consumer
    if (q > 0 || L > 0)
      if ((st = dev(launch_gemm(g, s))) != DLL_OK) return st;
    GemmArgs h;
    h.M = dd->out; h.N = dd->in; h.Kdim = B;
    h.A = gcur; h.a_m = 1; h.a_k = dd->out;
    h.B = nb.act[L + q]; h.b_k = dd->in; h.b_n = 1;
    h.Cout = grads ? grads[2 * (L + q)] : nullptr; h.c_m = dd->in; h.c_n = 1;
    if (upd) {
      h.update = Wq; h.step = step;
      if (velocity) { h.vel = velocity[2 * (L + q)]; h.mu = mu; h.decay = decay; }
    }
    h.split_k = 1;
    // The weight-gradient product only has to be done before the step ends (nothing below reads the
    // updated weights: every data gradient is taken with the old ones, just above).  It waits for
    // the next layer's, and the two share a launch: the upper layers' products are too small to
    // fill the chip on their own.
    if (h.Cout || h.update) {
      if (have_pending) {
        if ((st = dev(launch_gemm_pair(h, pending, s))) != DLL_OK) return st;
        have_pending = false;
      } else {
        pending = h;
        have_pending = true;
      }
    }
    float *gb = grads ? grads[2 * (L + q) + 1] : nullptr;
    if (gb || upd) {
      if (tail.n_colsum == StepTail::kMaxColsum && (st = flush_tail()) != DLL_OK) return st;
      tail.colsum[tail.n_colsum++] = StepTail::Colsum{gcur, B, dd->out, gb, upd ? bq : nullptr, step,
                                                      (upd && velocity) ? velocity[2 * (L + q) + 1] : nullptr, mu};
    }
  }
  if (have_pending && (st = dev(launch_gemm(pending, s))) != DLL_OK) return st;
  // ---- convolution backward: filter-gradient partial sums, then the data gradient with the old filters;
  // the reduction of the partial sums and the filter update wait for the closing launch
  float *gcur = nb.gbuf[0], *gnext = nb.gbuf[1];
  for (int l = L - 1; l >= 0; --l) {
    const dll_conv_desc *d = &net->conv[l];
    // pooled ReLU layers: the forward pass above flagged the inactive units in idx, so the
    // backward passes do not read the layer output
    const float *yl = (d->act == DLL_ACT_RELU && d->pool == 2) ? nullptr : nb.act[l + 1];
    // The filter-gradient partial sums first: the layer's output gradient has just been written by the
    // layer above's data-gradient pass and is read back while the memory-side cache still holds it
    // (measured 0.6 % of the large-image step against the other order).  The filters change only in
    // the closing launch, so the data-gradient pass after it still sees the old ones.
    WgradPlan plan;
    if (!plan_for(d, &plan)) return DLL_ERR_UNSUPPORTED;
    const WgradArgs wa = wgrad_args(d, nb.act[l], gcur, yl, nb.idx[l], nb.cpartial[l]);
    bool shared = false;
    if (l > 0) {
      // the two passes do not depend on each other; where both are streaming kernels they share a launch
      // (the filter gradient then with half as many workgroups, hence a plan of its own - never more
      // partial blocks than the plan the workspace was sized with)
      const ConvEngineArgs ba = bwd_args(d, gcur, yl, nb.idx[l], params[2 * l], gnext);
      WgradPlan half;
      if (plan_wgrad(d->N, d->C, d->H, d->W, d->K, d->R, d->S, d->pad, d->pool, &half, true) &&
          half.partial_floats <= plan.partial_floats && wgrad_bwd_pair_applies(wa, half, ba)) {
        st = dev(launch_wgrad_bwd_pair(wa, half, ba, s));
        if (st != DLL_OK) return st;
        plan = half;
        shared = true;
      }
    }
    if (!shared) {
      st = dev(launch_wgrad(wa, plan, s));
      if (st != DLL_OK) return st;
      if (l > 0) {
        st = dev(launch_conv_engine(bwd_args(d, gcur, yl, nb.idx[l], params[2 * l], gnext), s));
        if (st != DLL_OK) return st;
      }
    }
    WgradReduceArgs r;
    r.pos = nb.cpartial[l]; r.scale = 1.0f;
    r.dw = grads ? grads[2 * l] : nullptr;
    r.db = grads ? grads[2 * l + 1] : nullptr;
    if (upd) {
      r.w_update = params[2 * l]; r.b_update = params[2 * l + 1]; r.step = step;
      if (velocity) { r.w_vel = velocity[2 * l]; r.b_vel = velocity[2 * l + 1]; r.mu = mu; r.w_decay = decay; }
    }
    r.C = d->C; r.K = d->K; r.R = d->R; r.S = d->S;
    if (tail.n_reduce == StepTail::kMaxReduce && (st = flush_tail()) != DLL_OK) return st;
    tail.reduce[tail.n_reduce].a = r;
    tail.reduce[tail.n_reduce].plan = plan;
    ++tail.n_reduce;
    float *t = gcur; gcur = gnext; gnext = t;
  }
  if ((st = flush_tail()) != DLL_OK) return st;
  return DLL_OK;
}

}  // namespace

extern "C" {

dll_status dll_cnn_train_step(const dll_net_desc *net, float *const *params, float *const *grads, const float *x,
                              const int *labels, float lr, float *loss, float *logits, unsigned char *const *pool_idx,
                              void *ws, size_t ws_bytes, void *stream) {
  return run_cnn_step(net, params, nullptr, grads, x, labels, lr, 0.0f, 0.0f, loss, logits, pool_idx, ws, ws_bytes, stream);
}

dll_status dll_cnn_train_step_momentum(const dll_net_desc *net, float *const *params, float *const *velocity,
                                       float *const *grads, const float *x, const int *labels, float lr, float momentum,
                                       float weight_decay, float *loss, float *logits, unsigned char *const *pool_idx,
                                       void *ws, size_t ws_bytes, void *stream) {
  if (!velocity) return DLL_ERR_NULL;
  if (!(momentum >= 0.0f) || !(weight_decay >= 0.0f)) return DLL_ERR_SHAPE;
  return run_cnn_step(net, params, velocity, grads, x, labels, lr, momentum, weight_decay, loss, logits, pool_idx, ws,
                      ws_bytes, stream);
}

size_t dll_cnn_forward_workspace_bytes(const dll_net_desc *net) {
  NetLayout lay;
  if (check_net(net, &lay) != DLL_OK) return 0;
  Carver c(nullptr, 0);
  c.floats(lay.gmax); c.floats(lay.gmax);
  c.floats(lay.partial);
  c.floats((size_t)lay.B * net->classes);
  return c.used;
}

dll_status dll_cnn_forward(const dll_net_desc *net, const float *const *params, const float *x, float *logits,
                           float *prob, void *ws, size_t ws_bytes, void *stream) {
  NetLayout lay;
  dll_status st = check_net(net, &lay);
  if (st != DLL_OK) return st;
  const int L = net->n_conv, D = net->n_dense, B = lay.B;
  if (!params || !x || (!logits && !prob)) return DLL_ERR_NULL;
  for (int p = 0; p < 2 * (L + D); ++p) {
    if (!params[p]) return DLL_ERR_NULL;
    if (misaligned(params[p])) return DLL_ERR_SHAPE;
  }
  if (misaligned(x) || misaligned(logits) || misaligned(prob)) return DLL_ERR_SHAPE;
  if (logits && logits == prob) return DLL_ERR_SHAPE;
  Carver c(ws, 0);
  float *buf[2] = {c.floats(lay.gmax), c.floats(lay.gmax)};
  float *partial = c.floats(lay.partial);
  float *own_logits = c.floats((size_t)B * net->classes);
  st = check_ws(ws, ws_bytes, c.used);
  if (st != DLL_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const float *cur = x;
  int flip = 0;
  for (int l = 0; l < L; ++l) {
    const dll_conv_desc *d = &net->conv[l];
    float *out = buf[flip];
    st = dev(launch_conv_engine(fwd_args(d, cur, params[2 * l], params[2 * l + 1], out, nullptr), s));
    if (st != DLL_OK) return st;
    cur = out;
    flip ^= 1;
  }
  float *lg = logits ? logits : own_logits;
  for (int q = 0; q < D; ++q) {
    const dll_dense_desc *dd = &net->dense[q];
    float *out = (q == D - 1) ? lg : buf[flip];
    GemmArgs g;
    g.M = B; g.N = dd->out; g.Kdim = dd->in;
    g.A = cur; g.a_m = dd->in; g.a_k = 1;
    g.B = params[2 * (L + q)]; g.b_k = 1; g.b_n = dd->in;
    g.bias = params[2 * (L + q) + 1];
    g.act = (q == D - 1) ? ACT_IDENTITY : dd->act;
    g.Cout = out; g.c_m = dd->out; g.c_n = 1;
    g.split_k = gemm_pick_split_k(g.M, g.N, g.Kdim);
    g.partial = partial;
    if ((st = dev(launch_gemm(g, s))) != DLL_OK) return st;
    cur = out;
    flip ^= 1;
  }
  if (prob && (st = dev(launch_softmax_prob(lg, B, net->classes, prob, s))) != DLL_OK) return st;
  return DLL_OK;
}

}  // extern "C"
