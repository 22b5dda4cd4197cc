// Measurement aid, not a step of the method: the rate that back-to-back bf16 MFMAs reach on this chip when
// nothing else is going on (no global or LDS traffic, four independent accumulators per wave).  bench.py
// reports it next to the published peak, so that a roofline fraction can be read against both.
#include "citrus_internal.h"

namespace citrus {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kProbeWaves = 8;      // two per SIMD
constexpr int kProbeChains = 4;     // independent accumulators per wave
constexpr int kProbeBlocksPerCu = 2;

__global__ __launch_bounds__(kProbeWaves * 64) void mfma_probe_kernel(int iters, float* sink) {
  const int lane = threadIdx.x % 64;
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = static_cast<__bf16>(0.001f * static_cast<float>((lane + i) % 7));
    b[i] = static_cast<__bf16>(0.002f * static_cast<float>((lane + 3 * i) % 5));
  }
  f32x16 acc[kProbeChains];
#pragma unroll
  for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int c = 0; c < kProbeChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
  sink[static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x] = s;
}

}  // namespace
}  // namespace citrus

extern "C" {

int32_t citrus_probe_mfma(int32_t iters, float* sink, size_t sink_floats, int64_t* mfma_count, void* hip_stream) {
  using namespace citrus;
  if (sink == nullptr || mfma_count == nullptr) return CITRUS_ERR_NULL;
  if (iters < 1 || iters > (1 << 20)) return CITRUS_ERR_SHAPE;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return CITRUS_ERR_DEVICE;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return CITRUS_ERR_DEVICE;
  const int blocks = cus * kProbeBlocksPerCu;
  if (sink_floats < static_cast<size_t>(blocks) * kProbeWaves * 64) return CITRUS_ERR_WORKSPACE;
  *mfma_count = static_cast<int64_t>(blocks) * kProbeWaves * iters * 4 * kProbeChains;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(kProbeWaves * 64), 0, static_cast<hipStream_t>(hip_stream),
                     iters, sink);
  return hip_status(hipGetLastError());
}

}  // extern "C"
