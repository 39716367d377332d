// Stand-alone probe (not part of the library): what this GPU gives to the two roofs the kernels
// are priced against.
//   * fp32 MFMA: a register-only loop of v_mfma_f32_16x16x4_f32 with eight independent
//     accumulators per wavefront, at 1, 2 and 4 wavefronts per SIMD;
//   * HBM: a 16-byte-per-lane copy of 1 GiB (read + write), a read-only sum and a write-only fill.
// Usage: bench_chip_probe   (prints one line per measurement, then one JSON line that bench.py reads:
//        the best MFMA rate, the three HBM rates, and what the runtime reports of the device)
// Built by __graft_entry__.build(); bench.py runs it as a child process when it is there.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef float floatx4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                  \
  do {                                                                            \
    hipError_t e_ = (x);                                                          \
    if (e_ != hipSuccess) {                                                       \
      fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                     \
      exit(1);                                                                    \
    }                                                                             \
  } while (0)

__global__ __launch_bounds__(256) void mfma_loop(float *out, int iters, float a0, float b0) {
  floatx4 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
  const float a = a0 + (float)threadIdx.x, b = b0;
  // 64 products per trip: with only eight, the loop's own branch shows (41 instead of 33 cycles per
  // product at one wavefront per SIMD)
  for (int it = 0; it < iters; it += 8) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += (acc[i][0] + acc[i][1]) + (acc[i][2] + acc[i][3]);
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void copy16(const float4 *src, float4 *dst, size_t n) {
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256) dst[e] = src[e];
}
__global__ __launch_bounds__(256) void read16(const float4 *src, float *out, size_t n) {
  float s = 0.f;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256) {
    const float4 v = src[e];
    s += (v.x + v.y) + (v.z + v.w);
  }
  if (s == 12345.678f) out[0] = s;   // keeps the loads alive; never true for the fill value used
}
__global__ __launch_bounds__(256) void fill16(float4 *dst, size_t n, float v) {
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256) dst[e] = make_float4(v, v, v, v);
}

template <typename F>
static float time_ms(F launch, int reps) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  launch();
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0));
  for (int r = 0; r < reps; ++r) launch();
  CHECK(hipEventRecord(e1));
  CHECK(hipEventSynchronize(e1));
  float ms = 0.f;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  CHECK(hipGetLastError());
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
  return ms / reps;
}

int main() {
  hipDeviceProp_t prop;
  CHECK(hipGetDeviceProperties(&prop, 0));
  printf("device %s  CUs %d  clock %d MHz\n", prop.name, prop.multiProcessorCount, prop.clockRate / 1000);
  const int cus = prop.multiProcessorCount;
  int lds_cu = 0, lds_block = 0;
  CHECK(hipDeviceGetAttribute(&lds_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, 0));
  CHECK(hipDeviceGetAttribute(&lds_block, hipDeviceAttributeMaxSharedMemoryPerBlock, 0));
  printf("LDS per compute unit %d bytes, per workgroup %d bytes; L2 %d bytes\n", lds_cu, lds_block, prop.l2CacheSize);
  double best_mfma = 0.0;

  float *out = nullptr;
  CHECK(hipMalloc(&out, (size_t)cus * 4 * 256 * sizeof(float)));
  const int iters = 20000;
  for (int wps = 1; wps <= 4; wps *= 2) {   // workgroups of four wavefronts: one per SIMD each
    const int blocks = cus * wps;
    const float ms = time_ms([&] { hipLaunchKernelGGL(mfma_loop, dim3(blocks), dim3(256), 0, 0, out, iters, 1.0f, 0.5f); }, 3);
    const double flop = (double)blocks * 4 * iters * 8 * 2048.0;
    printf("fp32 MFMA 16x16x4, registers only, %d wavefront(s) per SIMD: %.3f ms  %.1f TFLOP/s\n", wps, ms, flop / ms / 1e9);
    if (flop / ms / 1e9 > best_mfma) best_mfma = flop / ms / 1e9;
  }
  CHECK(hipFree(out));

  const size_t bytes = (size_t)1 << 30, n = bytes / sizeof(float4);
  float4 *src = nullptr, *dst = nullptr;
  float *sink = nullptr;
  CHECK(hipMalloc(&src, bytes));
  CHECK(hipMalloc(&dst, bytes));
  CHECK(hipMalloc(&sink, sizeof(float)));
  const int blocks = cus * 16;
  hipLaunchKernelGGL(fill16, dim3(blocks), dim3(256), 0, 0, src, n, 1.0f);
  CHECK(hipDeviceSynchronize());
  float ms = time_ms([&] { hipLaunchKernelGGL(copy16, dim3(blocks), dim3(256), 0, 0, (const float4 *)src, dst, n); }, 10);
  printf("HBM copy 1 GiB (read + write): %.3f ms  %.2f TB/s\n", ms, 2.0 * bytes / ms / 1e9);
  const double copy_tbs = 2.0 * bytes / ms / 1e9;
  ms = time_ms([&] { hipLaunchKernelGGL(read16, dim3(blocks), dim3(256), 0, 0, (const float4 *)src, sink, n); }, 10);
  printf("HBM read 1 GiB: %.3f ms  %.2f TB/s\n", ms, 1.0 * bytes / ms / 1e9);
  const double read_tbs = 1.0 * bytes / ms / 1e9;
  ms = time_ms([&] { hipLaunchKernelGGL(fill16, dim3(blocks), dim3(256), 0, 0, dst, n, 2.0f); }, 10);
  printf("HBM write 1 GiB: %.3f ms  %.2f TB/s\n", ms, 1.0 * bytes / ms / 1e9);
  const double write_tbs = 1.0 * bytes / ms / 1e9;
  printf("{\"mfma_f32_tflops\": %.2f, \"hbm_copy_gbps\": %.1f, \"hbm_read_gbps\": %.1f, \"hbm_write_gbps\": %.1f, "
         "\"cus\": %d, \"clock_mhz\": %d, \"lds_per_cu\": %d, \"lds_per_workgroup\": %d}\n",
         best_mfma, copy_tbs * 1e3, read_tbs * 1e3, write_tbs * 1e3, cus, prop.clockRate / 1000, lds_cu, lds_block);
  CHECK(hipFree(src));
  CHECK(hipFree(dst));
  CHECK(hipFree(sink));
  return 0;
}
