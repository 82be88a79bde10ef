// Measurement aids: the device's own ceilings, measured with the same instructions the GroupGEMM uses, so that
// the layer's figures can be read against what this board sustains and not only against the published peak.
#include <type_traits>

#include "moe_internal.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Register-only MFMA loop: a wavefront's 128 x 128 outputs (the GroupGEMM's shape), operands that never change.
// RANDOM: bf16 values uniform in [-0.5, 0.5) from a per-lane generator; otherwise zeros (which draw far less power,
// hence clock higher).  SHAPE16: 64 blocks of v_mfma_f32_16x16x32_bf16 instead of 16 blocks of
// v_mfma_f32_32x32x16_bf16 -- the same flop per iteration with half the accumulator traffic per flop.
template <bool RANDOM, bool SHAPE16>
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
  float sum = 0.f;
  if constexpr (!SHAPE16) {
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
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 4; j++)
#pragma unroll
        for (int t = 0; t < 16; t++) sum += c[i][j][t];
  } else {
    f32x4 c[8][8];
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
      for (int j = 0; j < 8; j++) c[i][j] = (f32x4){0};
    for (int it = 0; it < iters; it += 2) {   // two iterations of the other shape's flop at a time
#pragma unroll
      for (int i = 0; i < 8; i++)
#pragma unroll
        for (int j = 0; j < 8; j++) c[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3], b[j & 3], c[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
      for (int j = 0; j < 8; j++)
#pragma unroll
        for (int t = 0; t < 4; t++) sum += c[i][j][t];
  }
  out[blockIdx.x * 256 + threadIdx.x] = sum;
}

// The MFMA loop again, now with the data movement of a GroupGEMM K step around it, arranged as the GroupGEMM's main
// loop arranges it, so that the price of each kind of traffic can be read off, in TFLOP/s, core clock and share of
// cycles the matrix cores are busy.  An iteration is one K step (32 values of K) of a wavefront's 128 x 128 outputs:
// 32 v_mfma_f32_32x32x16_bf16 in 8 groups of 4 -- or, SHAPE16, 64 v_mfma_f32_16x16x32_bf16 in 8 groups of 8 -- and per
// group optionally two ds_read_b128 that fetch operand fragments of the next (half) step from LDS into the other of
// two register sets (random bf16 data; 16 KiB per wavefront and K step with either shape) and one global -> LDS load
// of 1 KiB (a workgroup's 32 KiB per K step, from a 2 MiB region that stays in the L2 -- or, STREAM, two loads in
// eight from a region of 4 MiB per workgroup that is streamed through, i.e. from HBM); optionally a workgroup barrier
// per K step.  No wait depends on the loads except a bound on how many are in flight.
template <bool SHAPE16, bool LDS_READS, bool DMA, bool BARRIER, bool STREAM>
__global__ __launch_bounds__(256, 1) void k_probe_mix(const char* __restrict__ gsrc, float* out, uint64_t* clk, int iters) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];   // 64 KiB of operand data + 32 KiB landing zone
  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  uint32_t s = 12345u + tid * 2654435761u + blockIdx.x * 40503u;
  for (int i = tid; i < 96 * 1024 / 4; i += 256) {
    s = s * 1664525u + 1013904223u;
    const __bf16 lo = (__bf16)(((s >> 8) & 0xffff) / 65536.0f - 0.5f);
    s = s * 1664525u + 1013904223u;
    const __bf16 hi = (__bf16)(((s >> 8) & 0xffff) / 65536.0f - 0.5f);
    ((uint32_t*)smem)[i] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
  }
  __syncthreads();
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
  auto lds_frag = [](uint32_t a) { return *(const bf16x8 __attribute__((address_space(3)))*)(uintptr_t)a; };
  const uint32_t rd = lds0 + w * 16384 + lane * 16;      // the wavefront reads its own quarter of the operand data
  const uint32_t land = lds0 + 65536 + w * 8192;          // and lands its loads in its own 8 KiB
  const uint32_t goff = (uint32_t)(blockIdx.x & 31) * 65536u + w * 16384 + lane * 16;
  const char* stream_base = gsrc + ((size_t)4 << 20) + (size_t)blockIdx.x * ((size_t)4 << 20);
  // load q (of 8) of K step `it`
  auto load = [&](int it, int q) {
    const bool st = STREAM && (q & 3) == 0;
    const char* base = st ? stream_base : gsrc + (size_t)((it & 3) * 4096);
    const uint32_t off = st ? (uint32_t)(((it * 2 + (q >> 2)) * 4096) & ((4 << 20) - 1)) + w * 1024 + lane * 16 : goff + (q & 3) * 1024;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(land + q * 1024) : "memory");
  };
  auto sync_point = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    if (DMA) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
    if (BARRIER) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  using C0 = std::integral_constant<int, 0>;
  using C1 = std::integral_constant<int, 1>;
  float sum = 0.f;
  uint64_t cycles0, ticks0;   // core clock cycles; 100 MHz device clock
  if constexpr (!SHAPE16) {
    bf16x8 a[2][4], b[2][4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
      a[0][i] = a[1][i] = lds_frag(rd + i * 1024);
      b[0][i] = b[1][i] = lds_frag(rd + (4 + i) * 1024);
    }
    f32x16 c[4][4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) c[i][j] = (f32x16){0};
    // half h of K step it: the MFMAs of register set `cur`, the fragments of the next half step into set `nxt`
    auto half_step = [&](int it, int h, auto cur_c, auto nxt_c) {
      constexpr int cur = decltype(cur_c)::value, nxt = decltype(nxt_c)::value;
#pragma unroll
      for (int q = 0; q < 4; q++) {
        if (q > 0) __builtin_amdgcn_sched_barrier(0);
        if (DMA) load(it, h * 4 + q);
        if (LDS_READS) {
          a[nxt][q] = lds_frag(rd + ((it * 6 + h * 3 + q) & 15) * 1024);
          b[nxt][q] = lds_frag(rd + ((it * 6 + h * 3 + 4 + q) & 15) * 1024);
        }
#pragma unroll
        for (int m = q * 4; m < q * 4 + 4; m++) c[m >> 2][m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[cur][m & 3], a[cur][m >> 2], c[m >> 2][m & 3], 0, 0, 0);
#pragma unroll
        for (int m = 0; m < 4; m++) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (LDS_READS && m < 2) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      }
    };
    cycles0 = clock64();
    ticks0 = wall_clock64();
    for (int it = 0; it < iters; it++) {
      half_step(it, 0, C0{}, C1{});
      sync_point();
      half_step(it, 1, C1{}, C0{});
    }
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 4; j++)
#pragma unroll
        for (int t = 0; t < 16; t++) sum += c[i][j][t];
  } else {
    bf16x8 a[2][8], b[2][8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
      a[0][i] = a[1][i] = lds_frag(rd + i * 1024);
      b[0][i] = b[1][i] = lds_frag(rd + (8 + i) * 1024);
    }
    f32x4 c[8][8];
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
      for (int j = 0; j < 8; j++) c[i][j] = (f32x4){0};
    // K step it: the MFMAs of register set `cur`, the fragments of the next step into set `nxt`
    auto k_step = [&](int it, auto cur_c, auto nxt_c) {
      constexpr int cur = decltype(cur_c)::value, nxt = decltype(nxt_c)::value;
#pragma unroll
      for (int q = 0; q < 8; q++) {
        if (q > 0) __builtin_amdgcn_sched_barrier(0);
        if (DMA) load(it, q);
        if (LDS_READS) {
          a[nxt][q] = lds_frag(rd + ((it * 3 + q) & 15) * 1024);
          b[nxt][q] = lds_frag(rd + ((it * 3 + 8 + q) & 15) * 1024);
        }
#pragma unroll
        for (int j = 0; j < 8; j++) c[q][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[cur][j], a[cur][q], c[q][j], 0, 0, 0);
#pragma unroll
        for (int m = 0; m < 8; m++) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (LDS_READS && m < 2) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      }
    };
    cycles0 = clock64();
    ticks0 = wall_clock64();
    for (int it = 0; it < iters; it += 2) {
      k_step(it, C0{}, C1{});
      sync_point();
      k_step(it + 1, C1{}, C0{});
      sync_point();
    }
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
      for (int j = 0; j < 8; j++)
#pragma unroll
        for (int t = 0; t < 4; t++) sum += c[i][j][t];
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (tid == 0) {
    clk[blockIdx.x * 2] = clock64() - cycles0;
    clk[blockIdx.x * 2 + 1] = wall_clock64() - ticks0;
  }
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
  iters += iters & 1;
  const float ms = timed(st, 3, [&] {
    if (random_data == 2) hipLaunchKernelGGL((k_probe_mfma<true, true>), dim3(n_cu), dim3(256), 0, st, out, iters);
    else if (random_data) hipLaunchKernelGGL((k_probe_mfma<true, false>), dim3(n_cu), dim3(256), 0, st, out, iters);
    else hipLaunchKernelGGL((k_probe_mfma<false, false>), dim3(n_cu), dim3(256), 0, st, out, iters);
  });
  if (ms <= 0.f) return MOE_ERR_HIP;
  const double flop = (double)n_cu * 4 * iters * 16 * (2.0 * 32 * 32 * 16);
  *tflops = (float)(flop / (ms * 1e-3) / 1e12);
  return MOE_OK;
}

int moe_probe_mix(int32_t mode, int32_t iters, void* scratch, size_t scratch_bytes, float* tflops, float* core_ghz,
                  void* hip_stream) {
  if (!scratch || !tflops || iters < 1 || iters > (1 << 22) || mode < 0 || mode > 31 || ((uintptr_t)scratch & 15))
    return MOE_ERR_INVALID_ARG;
  const bool lds = mode & 1, dma = mode & 2, bar = mode & 4, stream = mode & 8, shape16 = mode & 16;
  iters += iters & 1;   // (the 16x16x32 loop takes two K steps at a time)
  if (stream && !dma) return MOE_ERR_INVALID_ARG;
  const int n_cu = compute_units();
  if (n_cu <= 0) return MOE_ERR_HIP;
  // layout of scratch: 4 MiB that the L2-resident loads read, then (streaming only) 4 MiB per workgroup; the
  // results land in the first region's last MiB, which no load reads (sums, then the cycle counts 512 KiB further on)
  const size_t need = ((size_t)4 << 20) + (stream ? (size_t)n_cu * ((size_t)4 << 20) : 0);
  if (scratch_bytes < need) return MOE_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)hip_stream;
  const char* g = (const char*)scratch;
  float* out = (float*)((char*)scratch + ((size_t)3 << 20));
  uint64_t* clk = (uint64_t*)((char*)scratch + ((size_t)3 << 20) + ((size_t)512 << 10));
  if ((size_t)n_cu * 256 * sizeof(float) > ((size_t)512 << 10) || n_cu > 512) return MOE_ERR_UNSUPPORTED;
  constexpr int lds_bytes = 96 * 1024;
  using Kern = void (*)(const char*, float*, uint64_t*, int);
  // [shape][lds][dma][barrier][stream]; streaming without loads does not exist
  static const Kern table[2][2][2][2][2] = {
      {{{{k_probe_mix<false, false, false, false, false>, nullptr}, {k_probe_mix<false, false, false, true, false>, nullptr}},
        {{k_probe_mix<false, false, true, false, false>, k_probe_mix<false, false, true, false, true>},
         {k_probe_mix<false, false, true, true, false>, k_probe_mix<false, false, true, true, true>}}},
       {{{k_probe_mix<false, true, false, false, false>, nullptr}, {k_probe_mix<false, true, false, true, false>, nullptr}},
        {{k_probe_mix<false, true, true, false, false>, k_probe_mix<false, true, true, false, true>},
         {k_probe_mix<false, true, true, true, false>, k_probe_mix<false, true, true, true, true>}}}},
      {{{{k_probe_mix<true, false, false, false, false>, nullptr}, {k_probe_mix<true, false, false, true, false>, nullptr}},
        {{k_probe_mix<true, false, true, false, false>, k_probe_mix<true, false, true, false, true>},
         {k_probe_mix<true, false, true, true, false>, k_probe_mix<true, false, true, true, true>}}},
       {{{k_probe_mix<true, true, false, false, false>, nullptr}, {k_probe_mix<true, true, false, true, false>, nullptr}},
        {{k_probe_mix<true, true, true, false, false>, k_probe_mix<true, true, true, false, true>},
         {k_probe_mix<true, true, true, true, false>, k_probe_mix<true, true, true, true, true>}}}}};
  const Kern kern = table[shape16][lds][dma][bar][stream];
  if (!kern) return MOE_ERR_INVALID_ARG;
  hipError_t err = hipSuccess;
  const float ms = timed(st, 1, [&] {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e == hipSuccess) {
      hipLaunchKernelGGL(kern, dim3(n_cu), dim3(256), lds_bytes, st, g, out, clk, iters);
      e = hipGetLastError();
    }
    if (e != hipSuccess) err = e;
  });
  if (err != hipSuccess || ms <= 0.f) return MOE_ERR_HIP;
  const double flop = (double)n_cu * 4 * iters * 32 * (2.0 * 32 * 32 * 16);   // a K step of 128 x 128 outputs per wavefront
  *tflops = (float)(flop / (ms * 1e-3) / 1e12);
  if (core_ghz) {
    // core clock inside the loop: cycles over elapsed time (100 MHz ticks), mean over the workgroups
    uint64_t host[512 * 2];
    if (hipMemcpyAsync(host, clk, (size_t)n_cu * 16, hipMemcpyDeviceToHost, st) != hipSuccess) return MOE_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return MOE_ERR_HIP;
    double sum = 0;
    for (int i = 0; i < n_cu; i++) sum += host[2 * i + 1] ? (double)host[2 * i] / ((double)host[2 * i + 1] * 10.0) : 0.0;
    *core_ghz = (float)(sum / n_cu);
  }
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
