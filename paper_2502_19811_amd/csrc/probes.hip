// Measurement aids: the device's own ceilings, measured with the same instructions the GroupGEMM uses, so that
// the layer's figures can be read against what this board sustains and not only against the published peak.
#include "moe_internal.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Register-only MFMA loop: 4 x 4 accumulator blocks per wavefront (the GroupGEMM's shape), operands that never
// change.  RANDOM: bf16 values uniform in [-0.5, 0.5) from a per-lane generator; otherwise zeros (which draw far
// less power, hence clock higher).
template <bool RANDOM>
__global__ __launch_bounds__(256) void k_probe_mfma(float* out, int iters) {
  bf16x8 a[4], b[4];
  uint32_t s = 12345u + threadIdx.x * 2654435761u + blockIdx.x * 40503u;
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int t = 0; t < 8; t++) {
      s = s * 1664525u + 1013904223u;
      a[i][t] = (__bf16)(RANDOM ? ((s >> 8) & 0xffff) / 65536.0f - 0.5f : 0.f);
      s = s * 1664525u + 1013904223u;
      b[i][t] = (__bf16)(RANDOM ? ((s >> 8) & 0xffff) / 65536.0f - 0.5f : 0.f);
    }
  f32x16 c[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) c[i][j] = (f32x16){0};
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], c[i][j], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int t = 0; t < 16; t++) sum += c[i][j][t];
  out[blockIdx.x * 256 + threadIdx.x] = sum;
}

__global__ __launch_bounds__(256) void k_probe_copy(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

}  // namespace moe

using namespace moe;

namespace {
// Runs launch() reps times between two events on the stream and returns the mean time of one in ms (< 0: HIP error).
template <typename F>
float timed(hipStream_t st, int reps, F launch) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return -1.f;
  if (hipEventCreate(&e1) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return -1.f;
  }
  float ms = -1.f;
  launch();   // warm-up
  if (hipEventRecord(e0, st) == hipSuccess) {
    for (int i = 0; i < reps; i++) launch();
    if (hipEventRecord(e1, st) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
        hipEventElapsedTime(&ms, e0, e1) == hipSuccess && hipGetLastError() == hipSuccess)
      ms /= reps;
    else
      ms = -1.f;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return ms;
}
int compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  return n;
}
}  // namespace

extern "C" {

int moe_probe_mfma(int32_t random_data, int32_t iters, void* scratch, size_t scratch_bytes, float* tflops,
                   void* hip_stream) {
  if (!scratch || !tflops || iters < 1 || iters > (1 << 20)) return MOE_ERR_INVALID_ARG;
  const int n_cu = compute_units();
  if (n_cu <= 0) return MOE_ERR_HIP;
  if (scratch_bytes < (size_t)n_cu * 256 * sizeof(float)) return MOE_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)hip_stream;
  float* out = (float*)scratch;
  const float ms = timed(st, 3, [&] {
    if (random_data) hipLaunchKernelGGL(k_probe_mfma<true>, dim3(n_cu), dim3(256), 0, st, out, iters);
    else hipLaunchKernelGGL(k_probe_mfma<false>, dim3(n_cu), dim3(256), 0, st, out, iters);
  });
  if (ms <= 0.f) return MOE_ERR_HIP;
  const double flop = (double)n_cu * 4 * iters * 16 * (2.0 * 32 * 32 * 16);
  *tflops = (float)(flop / (ms * 1e-3) / 1e12);
  return MOE_OK;
}

int moe_probe_copy(void* dst, const void* src, size_t bytes, float* gbytes_per_s, void* hip_stream) {
  if (!dst || !src || !gbytes_per_s || bytes < 16 || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15))
    return MOE_ERR_INVALID_ARG;
  const int n_cu = compute_units();
  if (n_cu <= 0) return MOE_ERR_HIP;
  hipStream_t st = (hipStream_t)hip_stream;
  const float ms = timed(st, 5, [&] {
    hipLaunchKernelGGL(k_probe_copy, dim3(n_cu * 16), dim3(256), 0, st, (u32x4*)dst, (const u32x4*)src, bytes / 16);
  });
  if (ms <= 0.f) return MOE_ERR_HIP;
  *gbytes_per_s = (float)(2.0 * (double)bytes / (ms * 1e-3) / 1e9);   // read + written
  return MOE_OK;
}

}  // extern "C"
