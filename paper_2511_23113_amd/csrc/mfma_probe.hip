// Sustained dense-MFMA rate of the chip, measured on the spot: context for the roofline.
// The published bf16 peak assumes 2.4 GHz; what a kernel can reach also depends on the clock the
// chip sustains under load, so the benchmark reports both the nominal and this measured ceiling.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>

#include "dbsp.h"
#include "dbsp_diag.h"
#include "plan.hpp"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Every wave issues `iters` x 8 independent v_mfma_f32_32x32x16_bf16 on four accumulators and
// nothing else; two waves per SIMD keep the matrix pipe full.  The operands are eight different
// register sets of pseudo-random values in [-2, 2) per lane (what the chip sustains depends on how
// many bits flip, so constant operands would flatter it).  Block 0 also reports the shader clock
// it ran at (core cycles over ticks of the 100 MHz constant clock).
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

__global__ __launch_bounds__(512) void mfma_probe_kernel(float* sink, uint64_t* clocks, int iters, uint32_t seed) {
  f32x16 acc[4];
  for (int a = 0; a < 4; ++a)
    for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;
  bf16x8 A[8], B[8];
#pragma unroll
  for (int m = 0; m < 8; ++m)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t ha = mix32(seed + (blockIdx.x * 512u + threadIdx.x) * 131u + m * 17u + i);
      const uint32_t hb = mix32(ha + 0x9e3779b9u);
      A[m][i] = (__bf16)(((int)(ha & 0xffff) - 32768) * (1.0f / 16384.0f));
      B[m][i] = (__bf16)(((int)(hb & 0xffff) - 32768) * (1.0f / 16384.0f));
    }
  const uint64_t c0 = clock64(), w0 = wall_clock64();
  float s = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 8; ++m) acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[m], B[m], acc[m & 3], 0, 0, 0);
    if ((it & 63) == 63) {   // keep the sums finite (a few moves per 512 MFMAs)
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) { s += acc[a][i]; acc[a][i] = 0.f; }
    }
  }
  const uint64_t c1 = clock64(), w1 = wall_clock64();
  for (int a = 0; a < 4; ++a)
    for (int i = 0; i < 16; ++i) s += acc[a][i];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clocks[0] = c1 - c0;
    clocks[1] = w1 - w0;
  }
}

}  // namespace

extern "C" int dbsp_mfma_probe(double* tflops, double* clock_ghz, void* stream) {
  if (!tflops) return dbsp_set_error(DBSP_EINVAL, "dbsp_mfma_probe: null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  int dev = 0;
  hipDeviceProp_t prop;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) { (void)hipGetLastError(); return dbsp_set_error(DBSP_EHIP, std::string("dbsp_mfma_probe: ") + hipGetErrorString(e)); }
  const int grid = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;   // one 8-wave workgroup per compute unit
  const int threads = 512, iters = 40000;
  float* sink = nullptr;
  uint64_t* clocks = nullptr;
  hipEvent_t a = nullptr, b = nullptr;
  auto cleanup = [&]() {
    if (sink) (void)hipFree(sink);
    if (clocks) (void)hipFree(clocks);
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
  };
  auto failed = [&](hipError_t err) {
    (void)hipGetLastError();
    cleanup();
    return dbsp_set_error(DBSP_EHIP, std::string("dbsp_mfma_probe: ") + hipGetErrorString(err));
  };
  if ((e = hipMalloc(&sink, sizeof(float) * (size_t)grid * threads)) != hipSuccess) return failed(e);
  if ((e = hipMalloc(&clocks, 2 * sizeof(uint64_t))) != hipSuccess) return failed(e);
  if ((e = hipEventCreate(&a)) != hipSuccess) return failed(e);
  if ((e = hipEventCreate(&b)) != hipSuccess) return failed(e);
  for (int rep = 0; rep < 3; ++rep)   // warm-up: clocks take a few tens of milliseconds to settle after idling
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(grid), dim3(threads), 0, st, sink, clocks, iters, 12345u + rep);
  if ((e = hipEventRecord(a, st)) != hipSuccess) return failed(e);
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(grid), dim3(threads), 0, st, sink, clocks, iters, 12345u);
  if ((e = hipGetLastError()) != hipSuccess) return failed(e);
  if ((e = hipEventRecord(b, st)) != hipSuccess) return failed(e);
  if ((e = hipEventSynchronize(b)) != hipSuccess) return failed(e);
  float ms = 0.f;
  if ((e = hipEventElapsedTime(&ms, a, b)) != hipSuccess) return failed(e);
  uint64_t h[2] = {0, 0};
  if ((e = hipMemcpy(h, clocks, sizeof(h), hipMemcpyDeviceToHost)) != hipSuccess) return failed(e);
  // 32 x 32 x 16 multiply-adds per MFMA, 8 MFMAs per iteration, threads / 64 waves per workgroup
  const double flops = (double)grid * (threads / 64) * (double)iters * 8.0 * 32768.0;
  *tflops = flops / ((double)ms * 1e-3) / 1e12;
  if (clock_ghz) *clock_ghz = h[1] ? (double)h[0] / ((double)h[1] * 10.0) : 0.0;   // cycles per 10 ns
  cleanup();
  return DBSP_OK;
}
