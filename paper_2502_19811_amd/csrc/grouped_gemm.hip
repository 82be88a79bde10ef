// GroupGEMM kernels of layer0 (gathered rows of x times W1, activation fused) and layer1 (h times W2, with
// data-movement workgroups reducing finished column panels), for gfx950.
//
// Design (paper Section 3.2.1 maps to CDNA4 like this):
//  * one persistent workgroup per compute unit walks a device-built tile schedule; a workgroup is either a
//    GEMM workgroup or a data-movement workgroup, chosen by its index (the division point of Section 3.2.2);
//  * a GEMM workgroup is 4 wavefronts, one per SIMD; a tile is BM x 256 outputs with BM = 256, 128 or 64, and
//    accumulates in fp32 with v_mfma_f32_32x32x16_bf16;
//  * operands go global -> LDS directly (global_load_lds_dwordx4, 16 bytes per lane, no registers in between),
//    through a ring of 4 stages of depth 32; rows of A are gathered through per-lane row offsets that stay in
//    registers for the whole tile (the row-index caching of Section 4);
//  * A is read from LDS with ds_read_b128 (K-contiguous rows, XOR-swizzled by row), B (stored K x N as the
//    weights are) with ds_read_b64_tr_b16, which hands every lane the 4 K-consecutive values of its column;
//  * a layer0 tile waits for the ready flag of the source segment of its last row (Section 2.2.1: a tile
//    cannot start before all of its tokens have arrived).
#include "moe_internal.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

enum { MODE_L0_GELU = 0, MODE_L0_SWIGLU = 1, MODE_L1 = 2 };

constexpr int BK = kTileK, NS = kStages, BN = kTileN;
constexpr int B_STAGE = BK * BN * 2;  // 16 KiB

__device__ __forceinline__ bf16x8 lds_read_a(uint32_t addr) {
  return *(const bf16x8 __attribute__((address_space(3)))*)(uintptr_t)addr;
}
// Two transposing reads: lane gets B[k0..k0+3][n] and B[k0+4..k0+7][n] of its column n.
__device__ __forceinline__ bf16x8 lds_read_b(uint32_t a0, uint32_t a1) {
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(uintptr_t)a0);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(uintptr_t)a1);
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}
// 16 bytes per lane from sbase + voff straight into LDS at lds_base + lane * 16.  Written as asm so that the
// compiler's wait-count pass does not serialise later LDS reads behind it; completion is awaited by hand
// with s_waitcnt vmcnt.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base)
               : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// GELU in its erf form, 0.5 v (1 + erf(v / sqrt 2)).  erf is evaluated with the classic 5-term rational
// approximation 1 - (a1 t + ... + a5 t^5) exp(-z^2), t = 1 / (1 + 0.3275911 z) (absolute error below 1.5e-7,
// far under the bf16 rounding of the result); it needs a handful of registers, which matters next to 256
// live accumulators.
__device__ __forceinline__ float gelu_erf(float v) {
  const float z = fabsf(v) * 0.70710678118654752f;
  const float t = 1.0f / (1.0f + 0.3275911f * z);
  float poly = 1.061405429f;
  poly = poly * t - 1.453152027f;
  poly = poly * t + 1.421413741f;
  poly = poly * t - 0.284496736f;
  poly = poly * t + 0.254829592f;
  const float erf_abs = 1.0f - poly * t * __expf(-z * z);
  const float erf_v = v < 0.f ? -erf_abs : erf_abs;
  return 0.5f * v * (1.0f + erf_v);
}
__device__ __forceinline__ float silu(float v) { return v / (1.0f + __expf(-v)); }

// Wait until *flag >= want.  Returns false if the spin limit (when set) ran out.
__device__ __forceinline__ bool spin_until_ge(const uint32_t* flag, uint32_t want, uint32_t spin_limit) {
  uint32_t polls = 0;
  while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) < want) {
    __builtin_amdgcn_s_sleep(8);
    if (spin_limit && ++polls >= spin_limit) return false;
  }
  return true;
}

// Top-k weighted reduction of one unit: 32 tokens x one 256-column panel of Y.
__device__ __forceinline__ void combine_unit(const GemmParams& p, int panel, int chunk) {
  const int tid = threadIdx.x;
  const int cg = tid & 31;
#pragma unroll
  for (int i = 0; i < kCombineChunk / 8; i++) {
    const int t = chunk * kCombineChunk + i * 8 + (tid >> 5);
    if (t >= p.T) continue;
    float acc[8];
#pragma unroll
    for (int c = 0; c < 8; c++) acc[c] = 0.f;
    const size_t col = (size_t)panel * BN + cg * 8;
    for (int j = 0; j < p.k; j++) {
      const int row = p.inv_perm[t * p.k + j];
      const float w = p.topk_weights[t * p.k + j];
      const u32x4 v = *(const u32x4*)(p.C + (size_t)row * p.ldc + col);
#pragma unroll
      for (int c = 0; c < 4; c++) {
        acc[2 * c] += w * __uint_as_float(v[c] << 16);
        acc[2 * c + 1] += w * __uint_as_float(v[c] & 0xffff0000u);
      }
    }
    u32x4 o;
#pragma unroll
    for (int c = 0; c < 4; c++) {
      typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
      bf16x2 pr = {(__bf16)acc[2 * c], (__bf16)acc[2 * c + 1]};
      o[c] = __builtin_bit_cast(uint32_t, pr);
    }
    *(u32x4*)(p.out + (size_t)t * p.H + col) = o;
  }
}

// Claims combine units until none are left.  A unit of panel n may start once every M-tile of that panel is done.
__device__ __forceinline__ void combine_loop(const GemmParams& p, int32_t* lds_slot) {
  const int n_panels = p.H / BN;
  const int n_chunks = (p.T + kCombineChunk - 1) / kCombineChunk;
  const int total = n_panels * n_chunks;
  const uint32_t need = (uint32_t)*p.n_tiles;
  int acquired_panel = -1;
  while (true) {
    __syncthreads();
    if (threadIdx.x == 0) {
      int u = atomicAdd(p.combine_counter, 1);
      if (u < total) {
        const int panel = u / n_chunks;
        if (panel != acquired_panel && !spin_until_ge(&p.panel_done[panel], need, p.spin_limit)) {
          atomicExch(p.status, (int)MOE_ERR_TIMEOUT);
          u = total;
        }
      }
      *lds_slot = u;
    }
    __syncthreads();
    const int u = *lds_slot;
    if (u >= total) break;
    const int panel = u / n_chunks;
    if (panel != acquired_panel) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      acquired_panel = panel;
    }
    combine_unit(p, panel, u % n_chunks);
  }
}

template <int WM, int MT, int NT, int MODE>
__global__ __launch_bounds__(256, 1) void k_group_gemm(GemmParams p) {
  constexpr int WN = 4 / WM;
  constexpr int BM = WM * MT * 32;
  static_assert(WN * NT * 32 == BN, "tile must be 256 columns wide");
  constexpr int A_STAGE = BM * BK * 2;
  constexpr int STAGE = A_STAGE + B_STAGE;
  constexpr int LA = BM / 64;  // A loads per lane per stage
  constexpr int LB = 4;        // B loads per lane per stage
  constexpr int LS = LA + LB;

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int32_t lds_slot;
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = w / WN, wn = w % WN;
  const int g = lane >> 4, j16 = lane & 15;

  if (MODE == MODE_L1 && (int)blockIdx.x >= p.n_mfma) {
    if (p.fused_combine) combine_loop(p, &lds_slot);
    return;
  }

  // LDS read addresses (stage 0), constant over the kernel
  uint32_t a_rd[2], b_rd[NT];
  {
    const int r = wm * (MT * 32) + (lane & 31);
    const int s = (r >> 2) & 3;
#pragma unroll
    for (int kk = 0; kk < 2; kk++) a_rd[kk] = lds0 + r * 64 + (((kk * 2 + (lane >> 5)) ^ s) << 4);
    const int swz = (j16 >> 2) | ((g >> 1) << 2);
    const int krow = 8 * (g >> 1) + (j16 >> 2);
#pragma unroll
    for (int nt = 0; nt < NT; nt++)
      b_rd[nt] = lds0 + A_STAGE + krow * 512 + (((wn * NT + nt) ^ swz) << 6) + (16 * (g & 1) + 4 * (j16 & 3)) * 2;
  }

  const int n_items = *p.n_items;
  for (int item = blockIdx.x; item < n_items; item += p.n_mfma) {
    const uint32_t it = p.items[item];
    const int m_tile = it >> 12, n_tile = it & 0xfff;
    const int expert = p.tile_expert[m_tile];
    const int row0 = p.tile_row0[m_tile];
    const int nrows = p.tile_rows[m_tile];

    // every wavefront must be done with the LDS stages of the previous tile before they are refilled
    __syncthreads();
    if (MODE != MODE_L1 && p.seg_ready != nullptr) {
      if (tid == 0) {
        const bool ok = spin_until_ge(&p.seg_ready[p.tile_ready[m_tile]], p.ready_epoch, p.spin_limit);
        if (!ok) atomicExch(p.status, (int)MOE_ERR_TIMEOUT);
        lds_slot = ok;
      }
      __syncthreads();
      if (!lds_slot) continue;
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "");
    }

    // per-lane global offsets of the loads of one stage
    uint32_t aoff[LA], boff[LB];
#pragma unroll
    for (int j = 0; j < LA; j++) {
      const int r = (w * LA + j) * 16 + (lane >> 2);
      const int c = (lane & 3) ^ ((r >> 2) & 3);
      int sr = row0 + (r < nrows ? r : nrows - 1);   // rows past the ragged end re-read the last row
      if (MODE != MODE_L1) sr = p.a_rows[sr];
      aoff[j] = (uint32_t)sr * p.lda_bytes + c * 16;
    }
    const int col0 = (MODE == MODE_L0_SWIGLU) ? n_tile * (BN / 2) : n_tile * BN;
#pragma unroll
    for (int j = 0; j < LB; j++) {
      const int kr = (w * LB + j) * 2 + (lane >> 5);
      const int cpb = lane & 31;
      const int blk = (cpb >> 2) ^ ((kr & 3) | (((kr >> 3) & 1) << 2));
      const int c8 = (blk * 4 + (cpb & 3)) * 8;  // column of the tile this lane fetches
      int gcol;
      if (MODE == MODE_L0_SWIGLU) {
        // a wavefront's 32*NT columns are [gate | up] of the same 16*NT hidden units
        const int region = c8 / (NT * 32), within = c8 % (NT * 32);
        const int half = within / (NT * 16), fo = within % (NT * 16);
        gcol = half * p.F + col0 + region * (NT * 16) + fo;
      } else {
        gcol = col0 + c8;
      }
      boff[j] = ((uint32_t)kr * p.ldb + gcol) * 2;
    }
    const char* Ab = p.A;
    const char* Bb = p.B + (uint64_t)expert * p.b_expert_bytes;
    const size_t bstep = (size_t)BK * p.ldb * 2;

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
      for (int j = 0; j < NT; j++) acc[i][j] = (f32x16){0};

    // One stage = LA loads of A rows and LB loads of B rows per lane.  The loads are issued one at a time between
    // groups of MFMAs: a burst would fill the vector-memory queue and stall the MFMAs queued behind it.
    auto issue_a = [&](int stage, int j) { dma16(Ab, aoff[j], lds0 + stage * STAGE + (w * LA + j) * 1024); };
    auto issue_b = [&](int stage, int j) { dma16(Bb, boff[j], lds0 + stage * STAGE + A_STAGE + (w * LB + j) * 1024); };
    auto advance = [&]() {
      Ab += BK * 2;
      Bb += bstep;
    };
    bf16x8 af[2][MT], bfr[2][NT];
    // Group q (of 4) of a half step: the LDS reads of fragment q for the next half step and a quarter of the MFMAs
    // of this one.  rd_off / rd_kk: stage offset and 16-deep sub-step the fragments are read from.
    auto group = [&](int cur, int nxt, uint32_t rd_off, int rd_kk, int q) {
      constexpr int PER = MT * NT / 4;
      if (q < MT) af[nxt][q] = lds_read_a(rd_off + a_rd[rd_kk] + q * 32 * 64);
      if (q < NT)
        bfr[nxt][q] = lds_read_b(rd_off + b_rd[q] + rd_kk * 16 * 512, rd_off + b_rd[q] + (rd_kk * 16 + 4) * 512);
#pragma unroll
      for (int i = 0; i < PER; i++) {
        const int m = q * PER + i, mt = m / NT, nt = m % NT;
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][mt], bfr[cur][nt], acc[mt][nt], 0, 0, 0);
      }
      const int n_reads = (q < MT ? 1 : 0) + (q < NT ? 2 : 0);
#pragma unroll
      for (int i = 0; i < PER; i++) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (i < n_reads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
#pragma unroll
      for (int i = PER; i < 3; i++)
        if (i < n_reads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    };
    auto half1 = [&](int stage_issue, bool do_issue, uint32_t so) {
#pragma unroll
      for (int q = 0; q < 4; q++) {
        if (do_issue && q < LA) issue_a(stage_issue, q);
        group(0, 1, so, 1, q);
      }
    };
    auto half2 = [&](int stage_issue, bool do_issue, uint32_t sn) {
#pragma unroll
      for (int q = 0; q < 4; q++) {
        if (do_issue && q < LB) issue_b(stage_issue, q);
        group(1, 0, sn, 0, q);
      }
    };

    const int nk = p.K / BK;  // >= NS - 1 (checked on the host)
#pragma unroll
    for (int s = 0; s < NS - 1; s++) {
#pragma unroll
      for (int j = 0; j < LA; j++) issue_a(s, j);
#pragma unroll
      for (int j = 0; j < LB; j++) issue_b(s, j);
      advance();
    }
    wait_vmcnt<(NS - 2) * LS>();
    __syncthreads();
#pragma unroll
    for (int mt = 0; mt < MT; mt++) af[0][mt] = lds_read_a(a_rd[0] + mt * 32 * 64);
#pragma unroll
    for (int nt = 0; nt < NT; nt++) bfr[0][nt] = lds_read_b(b_rd[nt], b_rd[nt] + 4 * 512);

    int kt = 0;
    for (; kt < nk - (NS - 1); kt++) {
      const int st = (kt + NS - 1) % NS;
      half1(st, true, (kt % NS) * STAGE);
      // stage kt+1 has landed for this lane (younger: stage kt+2 and the A rows of stage kt+3); after the barrier
      // it has for all, and all are done reading stage kt
      wait_vmcnt<LS + LA>();
      __syncthreads();
      half2(st, true, ((kt + 1) % NS) * STAGE);
      advance();
    }
    half1(0, false, (kt % NS) * STAGE);
    wait_vmcnt<LS>();
    __syncthreads();
    half2(0, false, ((kt + 1) % NS) * STAGE);
    kt++;
    half1(0, false, (kt % NS) * STAGE);
    wait_vmcnt<0>();
    __syncthreads();
    half2(0, false, ((kt + 1) % NS) * STAGE);
    kt++;
    half1(0, false, (kt % NS) * STAGE);
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
      for (int nt = 0; nt < NT; nt++)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[1][mt], bfr[1][nt], acc[mt][nt], 0, 0, 0);

    // epilogue: lane holds column (lane & 31) of each 32x32 block, rows (i/4)*8 + (lane/32)*4 + i%4
    const int rbase = wm * (MT * 32) + (lane >> 5) * 4;
    if (MODE == MODE_L0_SWIGLU) {
      const int f0 = col0 + wn * (NT * 16) + (lane & 31);
#pragma unroll
      for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int nt = 0; nt < NT / 2; nt++)
#pragma unroll
          for (int i = 0; i < 16; i++) {
            const int r = rbase + mt * 32 + (i >> 2) * 8 + (i & 3);
            if (r < nrows) {
              const float hval = silu(acc[mt][nt][i]) * acc[mt][nt + NT / 2][i];
              ((__bf16*)p.C)[(size_t)(row0 + r) * p.ldc + f0 + nt * 32] = (__bf16)hval;
            }
          }
    } else {
      const int c0 = col0 + wn * (NT * 32) + (lane & 31);
#pragma unroll
      for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int nt = 0; nt < NT; nt++) {
          __builtin_amdgcn_sched_barrier(0);  // keeps the activation temporaries of one block live at a time
#pragma unroll
          for (int i = 0; i < 16; i++) {
            const int r = rbase + mt * 32 + (i >> 2) * 8 + (i & 3);
            if (r < nrows) {
              float v = acc[mt][nt][i];
              if (MODE == MODE_L0_GELU) v = gelu_erf(v);
              ((__bf16*)p.C)[(size_t)(row0 + r) * p.ldc + c0 + nt * 32] = (__bf16)v;
            }
          }
        }
    }
    if (MODE == MODE_L1) {
      // publish: this M-tile of column panel n_tile is in memory
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      __syncthreads();
      if (tid == 0) __hip_atomic_fetch_add(&p.panel_done[n_tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (MODE == MODE_L1 && p.fused_combine) combine_loop(p, &lds_slot);
}

template <int WM, int MT, int NT, int MODE>
static hipError_t launch_gemm(const GemmParams& p, int grid, hipStream_t st) {
  constexpr int BM = WM * MT * 32;
  constexpr int lds = NS * (BM * BK * 2 + B_STAGE);
  auto kern = k_group_gemm<WM, MT, NT, MODE>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, p);
  return hipGetLastError();
}

hipError_t launch_layer0(const GemmParams& p, int tile_m, int act, int grid, hipStream_t st) {
  if (act == MOE_ACT_SWIGLU) {
    if (tile_m == 256) return launch_gemm<2, 4, 4, MODE_L0_SWIGLU>(p, grid, st);
    if (tile_m == 128) return launch_gemm<2, 2, 4, MODE_L0_SWIGLU>(p, grid, st);
    return launch_gemm<1, 2, 2, MODE_L0_SWIGLU>(p, grid, st);
  }
  if (tile_m == 256) return launch_gemm<2, 4, 4, MODE_L0_GELU>(p, grid, st);
  if (tile_m == 128) return launch_gemm<2, 2, 4, MODE_L0_GELU>(p, grid, st);
  return launch_gemm<1, 2, 2, MODE_L0_GELU>(p, grid, st);
}

hipError_t launch_layer1(const GemmParams& p, int tile_m, int grid, hipStream_t st) {
  if (tile_m == 256) return launch_gemm<2, 4, 4, MODE_L1>(p, grid, st);
  if (tile_m == 128) return launch_gemm<2, 2, 4, MODE_L1>(p, grid, st);
  return launch_gemm<1, 2, 2, MODE_L1>(p, grid, st);
}

// ---------------------------------------------------------------------------------------------
// Stand-alone top-k weighted reduction (used when the layer1 kernel runs without data-movement workgroups).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_combine(CombineParams p) {
  const int cols8 = p.H / 8;
  const size_t total = (size_t)p.T * cols8;
  for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (size_t)gridDim.x * 256) {
    const int t = (int)(idx / cols8);
    const size_t col = (idx % cols8) * 8;
    float acc[8];
#pragma unroll
    for (int c = 0; c < 8; c++) acc[c] = 0.f;
    for (int j = 0; j < p.k; j++) {
      const int row = p.inv_perm[t * p.k + j];
      const float w = p.topk_weights[t * p.k + j];
      const u32x4 v = *(const u32x4*)(p.Y + (size_t)row * p.H + col);
#pragma unroll
      for (int c = 0; c < 4; c++) {
        acc[2 * c] += w * __uint_as_float(v[c] << 16);
        acc[2 * c + 1] += w * __uint_as_float(v[c] & 0xffff0000u);
      }
    }
    u32x4 o;
#pragma unroll
    for (int c = 0; c < 4; c++) {
      typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
      bf16x2 pr = {(__bf16)acc[2 * c], (__bf16)acc[2 * c + 1]};
      o[c] = __builtin_bit_cast(uint32_t, pr);
    }
    *(u32x4*)(p.out + (size_t)t * p.H + col) = o;
  }
}

hipError_t launch_combine(const CombineParams& p, hipStream_t st) {
  if (p.T == 0) return hipSuccess;
  const size_t total = (size_t)p.T * (p.H / 8);
  int grid = (int)((total + 255) / 256);
  if (grid > 256 * 16) grid = 256 * 16;
  hipLaunchKernelGGL(k_combine, dim3(grid), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace moe
