// GroupGEMM kernels of layer0 (gathered rows of x times W1, activation fused) and layer1 (h times W2), the top-k
// reduction in its three places (a kernel of its own, data-movement workgroups inside the layer1 kernel, the layer1
// epilogue), the one-launch variant of the two GroupGEMMs, and the plan-time weight packing, for gfx950.
//
// Design (paper Section 3.2.1 maps to CDNA4 like this):
//  * one persistent workgroup per compute unit walks a device-built tile schedule; a workgroup is either a
//    GEMM workgroup or a data-movement workgroup, chosen by its index (the division point of Section 3.2.2); the
//    data movement there is to do on one GPU: reducing finished column panels of layer1, prefetching weight panels;
//  * a GEMM workgroup is 4 wavefronts, one per SIMD; a tile is BM x 256 outputs with BM = 256, 128 or 64, and
//    accumulates in fp32 with v_mfma_f32_32x32x16_bf16;
//  * operands go global -> LDS directly (global_load_lds_dwordx4, 16 bytes per lane, no registers in between):
//    B through a ring of 4 stages of depth 32, A through a ring of 5 blocks of half the tile's rows by depth 64, so
//    that a load of A fetches whole 128-byte lines (8 rows per instruction); rows of A are gathered through
//    per-lane row offsets that stay in registers for the whole tile (the row-index caching of Section 4);
//  * A is read from LDS with ds_read_b128 (K-contiguous rows, XOR-swizzled by row); B either as the weights are
//    stored (K x N) with ds_read_b64_tr_b16, which hands every lane the 4 K-consecutive values of its column, or, with
//    packed weights (k_pack_weights: every stage already an LDS image in operand order), with one ds_read_b128;
//  * a layer0 tile waits for the ready flag of the source segment of its last row (Section 2.2.1: a tile
//    cannot start before all of its tokens have arrived);
//  * the tile schedules are built on the device (index_build.hip): one queue of 32-byte item records per XCD,
//    taken with one atomic per tile, a tile ahead, and stolen from the other XCDs' queues at the end.
#include <atomic>
#include <mutex>

#include "moe_internal.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

enum { MODE_L0_GELU = 0, MODE_L0_SWIGLU = 1, MODE_L1 = 2 };

constexpr int BK = kTileK, NS = kStages, BN = kTileN;
#ifndef MOE_READ_GROUPS
#define MOE_READ_GROUPS 2
#endif
constexpr int kReadGroups = MOE_READ_GROUPS;        // of the 4 groups of a half step, how many carry the LDS reads
constexpr int kFragsPerGroup = 4 / kReadGroups;     // fragments (of at most 4 per operand) requested per such group
constexpr int kMaxPanels = 128;   // column panels whose publication can be batched per workgroup
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
// Packed weights: a fragment (32 columns x 16 values of K) lies in LDS in lane order, 16 bytes per lane.
__device__ __forceinline__ bf16x8 lds_read_b_packed(uint32_t a) {
  return *(const bf16x8 __attribute__((address_space(3)))*)(uintptr_t)a;
}
// 16 bytes per lane from sbase + voff straight into LDS at lds_base + lane * 16.  Written as asm so that the
// compiler's wait-count pass does not serialise later LDS reads behind it; completion is awaited by hand
// with s_waitcnt vmcnt.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base)
               : "memory");
}
// The same with the LDS address given as a base in a scalar register plus a constant: the addition writes M0 itself.
template <int OFF>
__device__ __forceinline__ void dma16_at(const void* sbase, uint32_t voff, uint32_t lds_base) {
  if constexpr (OFF == 0) {
    dma16(sbase, voff, lds_base);
  } else {
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base), "n"(OFF)
                 : "memory", "scc");
  }
}
// Tells the compiler that a pointer / integer is the same in every lane (keeps it in scalar registers).
__device__ __forceinline__ const char* uniform(const char* ptr) {
  const uint64_t v = (uint64_t)(uintptr_t)ptr;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const char*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

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
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * z);
  float poly = 1.061405429f;
  poly = poly * t - 1.453152027f;
  poly = poly * t + 1.421413741f;
  poly = poly * t - 0.284496736f;
  poly = poly * t + 0.254829592f;
  const float erf_abs = 1.0f - poly * t * __builtin_amdgcn_exp2f(z * z * -1.4426950408889634f);
  const float erf_v = v < 0.f ? -erf_abs : erf_abs;
  return 0.5f * v * (1.0f + erf_v);
}
// v * sigmoid(v) with the hardware exp2 and reciprocal (about 1 ulp each; the result is rounded to bf16 anyway).
__device__ __forceinline__ float silu(float v) {
  return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * -1.4426950408889634f));
}

// Wait until *flag >= want.  Returns false if the spin limit (when set) ran out.
__device__ __forceinline__ bool spin_until_ge(const uint32_t* flag, uint32_t want, uint32_t spin_limit) {
  uint32_t polls = 0;
  while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) < want) {
    __builtin_amdgcn_s_sleep(8);
    if (spin_limit && ++polls >= spin_limit) return false;
  }
  return true;
}

// Top-k weighted reduction of one unit: kCombineChunk tokens x one 256-column panel of Y.  A thread owns 8 columns
// (16 bytes) of every 8th token of the unit; the rows of several tokens are requested before any is used, because
// with one workgroup per compute unit only loads in flight can cover the memory latency.
template <int K>
__device__ __forceinline__ void combine_unit_k(const GemmParams& p, int panel, int chunk, int k_runtime) {
  constexpr int KK = K > 0 ? K : 1;
  constexpr int TB = K == 0 ? 1 : (K <= 2 ? 8 : (K <= 4 ? 4 : 2));   // tokens per batch of a thread
  constexpr int NB = kCombineChunk / 8 / TB;                           // batches per unit
  const int tid = threadIdx.x;
  const int cg = tid & 31, ts = tid >> 5;
  const size_t col = (size_t)panel * BN + cg * 8;
  if (K == 0) {
    // any other k: one token at a time
    for (int i0 = 0; i0 < kCombineChunk / 8; i0++) {
      const int t = chunk * kCombineChunk + i0 * 8 + ts;
      if (t >= p.T) continue;
      float acc[8];
#pragma unroll
      for (int c = 0; c < 8; c++) acc[c] = 0.f;
      for (int j = 0; j < k_runtime; j++) {
        const int row = p.inv_perm[t * k_runtime + j];
        const float w = p.topk_weights[t * k_runtime + j];
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
        bf16x2 pr = {(__bf16)acc[2 * c], (__bf16)acc[2 * c + 1]};
        o[c] = __builtin_bit_cast(uint32_t, pr);
      }
      *(u32x4*)(p.out + (size_t)t * p.H + col) = o;
    }
    return;
  }
  // Two batches in flight: the rows of batch i+1 are requested before batch i is summed and stored.
  float w[2][TB][KK];
  u32x4 v[2][TB][KK];
  auto request = [&](int buf, int batch) {
    int row[TB][KK];
#pragma unroll
    for (int b = 0; b < TB; b++) {
      const int t = chunk * kCombineChunk + (batch * TB + b) * 8 + ts;
      const int tt = t < p.T ? t : p.T - 1;
#pragma unroll
      for (int j = 0; j < KK; j++) {
        row[b][j] = p.inv_perm[tt * KK + j];
        w[buf][b][j] = p.topk_weights[tt * KK + j];
      }
    }
#pragma unroll
    for (int b = 0; b < TB; b++)
#pragma unroll
      for (int j = 0; j < KK; j++) v[buf][b][j] = *(const u32x4*)(p.C + (size_t)row[b][j] * p.ldc + col);
  };
  auto finish = [&](int buf, int batch) {
#pragma unroll
    for (int b = 0; b < TB; b++) {
      const int t = chunk * kCombineChunk + (batch * TB + b) * 8 + ts;
      float acc[8];
#pragma unroll
      for (int c = 0; c < 8; c++) acc[c] = 0.f;
#pragma unroll
      for (int j = 0; j < KK; j++)
#pragma unroll
        for (int c = 0; c < 4; c++) {
          acc[2 * c] += w[buf][b][j] * __uint_as_float(v[buf][b][j][c] << 16);
          acc[2 * c + 1] += w[buf][b][j] * __uint_as_float(v[buf][b][j][c] & 0xffff0000u);
        }
      if (t < p.T) {
        u32x4 o;
#pragma unroll
        for (int c = 0; c < 4; c++) {
          bf16x2 pr = {(__bf16)acc[2 * c], (__bf16)acc[2 * c + 1]};
          o[c] = __builtin_bit_cast(uint32_t, pr);
        }
        *(u32x4*)(p.out + (size_t)t * p.H + col) = o;
      }
    }
  };
  static_assert(NB % 2 == 0, "batches are processed in pairs");
  request(0, 0);
#pragma unroll 1
  for (int i = 0; i < NB; i += 2) {
    request(1, i + 1);
    finish(0, i);
    if (i + 2 < NB) request(0, i + 2);
    finish(1, i + 1);
  }
}

__device__ __forceinline__ void combine_unit(const GemmParams& p, int panel, int chunk) {
  switch (p.k) {
    case 1: combine_unit_k<1>(p, panel, chunk, 1); break;
    case 2: combine_unit_k<2>(p, panel, chunk, 2); break;
    case 4: combine_unit_k<4>(p, panel, chunk, 4); break;
    case 8: combine_unit_k<8>(p, panel, chunk, 8); break;
    default: combine_unit_k<0>(p, panel, chunk, p.k); break;
  }
}

// Claims combine units until none are left.  A unit of panel n may start once every M-tile of that panel is done.
// all_at_once: the panels are all published together at the end of the GEMM work (no data-movement workgroups), so
// the workgroup waits for the last panel once and needs a single acquire instead of one per panel.
__device__ __forceinline__ void combine_loop(const GemmParams& p, int32_t* lds_slot, bool all_at_once) {
  const int n_panels = p.H / BN;
  const int n_chunks = (p.T + kCombineChunk - 1) / kCombineChunk;
  const int total = n_panels * n_chunks;
  const uint32_t need = (uint32_t)*p.n_tiles;
  int acquired_panel = -1;
  if (all_at_once) {
    __syncthreads();
    if (threadIdx.x == 0) {
      bool ok = true;
      for (int n = 0; n < n_panels && ok; n++) ok = spin_until_ge(&p.panel_done[n], need, p.spin_limit);
      if (!ok) atomicExch(p.status, (int)MOE_ERR_TIMEOUT);
      *lds_slot = ok;
    }
    __syncthreads();
    if (!*lds_slot) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    acquired_panel = n_panels;   // everything is acquired
  }
  while (true) {
    __syncthreads();
    if (threadIdx.x == 0) {
      int u = atomicAdd(p.combine_counter, 1);
      if (u < total && !all_at_once) {
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
    if (!all_at_once && panel != acquired_panel) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      acquired_panel = panel;
    }
    combine_unit(p, panel, u % n_chunks);
  }
}

// ---------------------------------------------------------------------------------------------
// Schedule queues: XCD x owns the list positions base[x] + i * stride, i < len[x].
// ---------------------------------------------------------------------------------------------
struct Queue {
  int own_len, own_base;   // this workgroup's XCD, read once
};
__device__ __forceinline__ int queue_pos(const GemmParams& p, int x, int i) {
  return (p.queue_base ? p.queue_base[x] : x) + i * p.queue_stride;
}
// Takes the next item of XCD x's queue; returns its list position or -1 when that queue is used up.
__device__ __forceinline__ int take_from(const GemmParams& p, int x, int len, int base) {
  if (len == 0) return -1;
  const int i = __hip_atomic_fetch_add(&p.queue_heads[x], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return i < len ? base + i * p.queue_stride : -1;
}
// The other XCDs' leftovers, nearest first; -1 when every queue is used up.  All heads and lengths are read first
// (one round trip): at the end of a kernel, and in small problems, most queues are empty and an atomic on each
// of them from every workgroup would serialise on the counters.
__device__ __forceinline__ int steal(const GemmParams& p, int xcd) {
  int head[kXcds], len[kXcds];
#pragma unroll
  for (int d = 1; d < kXcds; d++) {
    const int x = (xcd + d) & (kXcds - 1);
    head[d] = __hip_atomic_load(&p.queue_heads[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    len[d] = p.queue_len[x];
  }
#pragma unroll
  for (int d = 1; d < kXcds; d++) {
    if (head[d] >= len[d]) continue;
    const int x = (xcd + d) & (kXcds - 1);
    const int idx = take_from(p, x, len[d], queue_pos(p, x, 0));
    if (idx >= 0) return idx;
  }
  return -1;
}
// Data-movement workgroup that runs ahead of the GEMM workgroups of its XCD (the specialisation of Section 3.2.1 put
// to local use): it follows the head of the XCD's queue and reads one word of every 128-byte line of the packed
// weight panel of the items about to be handed out, so that the panel is on its way from HBM into the Infinity Cache
// (and this XCD's L2) before a GEMM workgroup's three K steps of lead have to cover the miss.  Pays where a weight
// panel serves few M-tiles (many small experts): there the GEMM workgroups wait for HBM, not for the matrix cores.
// `part` of `n_parts`: the workgroups sharing an XCD split every panel between them.  The loop ends when the queue is
// handed out, or when its head has not moved for about a second (the GEMM side waiting for a ready flag): a
// workgroup that stops prefetching costs time, never correctness.
constexpr int kPrefetchUnroll = 16;
__device__ __forceinline__ void prefetch_loop(const GemmParams& p, int xcd, int part, int n_parts) {
  const int len = p.queue_len[xcd];
  const int base = queue_pos(p, xcd, 0);
  const uint64_t panel_bytes = (uint64_t)(p.K / BK) * B_STAGE;
  const int lines = (int)(panel_bytes / 128);
  const int tid = threadIdx.x;
  int i = 0, last_expert = -1, last_n = -1;
  uint32_t idle = 0, sink = 0;
  while (i < len) {
    const int head = uniform(__hip_atomic_load(&p.queue_heads[xcd], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    if (head >= len) break;   // everything handed out: nothing left to be ahead of
    // items handed out a while ago are being streamed by their workgroups already
    if (i < head - p.prefetch_behind) i = head - p.prefetch_behind;
    if (i >= head + p.prefetch_ahead) {
      if (++idle > (1u << 20)) break;
      __builtin_amdgcn_s_sleep(32);
      continue;
    }
    idle = 0;
    const int expert = uniform(p.items[base + i * p.queue_stride].expert);
    const int n_tile = uniform(p.items[base + i * p.queue_stride].n_tile);
    i++;
    if (expert == last_expert && n_tile == last_n) continue;   // the M-tiles of a block share the panel
    last_expert = expert;
    last_n = n_tile;
    const char* src = p.B + ((uint64_t)expert * p.n_tiles_n + n_tile) * panel_bytes;
    for (int l0 = part * 256 * kPrefetchUnroll; l0 < lines; l0 += n_parts * 256 * kPrefetchUnroll) {
      uint32_t v[kPrefetchUnroll];
#pragma unroll
      for (int u = 0; u < kPrefetchUnroll; u++) {
        const int l = l0 + u * 256 + tid;
        v[u] = l < lines ? *(const uint32_t*)(src + (size_t)l * 128) : 0u;
      }
#pragma unroll
      for (int u = 0; u < kPrefetchUnroll; u++) sink ^= v[u];
    }
  }
  if (p.K < 0) p.status[63] = (int32_t)sink;   // never true: keeps the loads
}
// The last n_prefetch workgroups of a launch take the prefetch role (multiples of 8: workgroup b runs on XCD b % 8,
// so any 8 consecutive workgroups cover the 8 XCDs).
__device__ __forceinline__ bool prefetch_role(const GemmParams& p) {
  const int first = (int)gridDim.x - p.n_prefetch;
  if (p.n_prefetch <= 0 || (int)blockIdx.x < first) return false;
  prefetch_loop(p, blockIdx.x & (kXcds - 1), ((int)blockIdx.x - first) >> 3, p.n_prefetch >> 3);
  return true;
}

__device__ __forceinline__ void block_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

#ifdef MOE_TILE_TRACE
// Measurement build only (tile_trace.py compiles the library with -DMOE_TILE_TRACE): every workgroup notes, per tile,
// the time (100 MHz device clock) at which it started on it, had the operands of the first K step in LDS, finished
// the main loop and finished the epilogue; and, in core clock cycles, how long the main loop took and how much of that
// its first wavefront spent at the synchronisation point of each K step (waiting for its operand loads to land and
// for the other wavefronts).
constexpr int kTraceWgs = 256, kTraceTiles = 128, kTraceWords = 6;
__device__ uint64_t g_trace_stamp[2][kTraceWgs][kTraceTiles][kTraceWords];
__device__ int32_t g_trace_kind[2][kTraceWgs][kTraceTiles];
__device__ int32_t g_trace_count[2][kTraceWgs];
// (The count is kept in LDS, slot: a load from global memory here would make the compiler wait for everything in
// flight, the successor's first operand loads included.)
__device__ __forceinline__ void trace_tile(int layer, int kind, uint64_t t0, uint64_t t1, uint64_t t2, uint64_t t3,
                                           uint64_t loop_cycles, uint64_t sync_cycles, volatile uint32_t* slot) {
  if (threadIdx.x != 0 || blockIdx.x >= kTraceWgs) return;
  const int n = (int)slot[layer];
  if (n >= kTraceTiles) return;
  slot[layer] = (uint32_t)(n + 1);
  g_trace_stamp[layer][blockIdx.x][n][0] = t0;
  g_trace_stamp[layer][blockIdx.x][n][1] = t1;
  g_trace_stamp[layer][blockIdx.x][n][2] = t2;
  g_trace_stamp[layer][blockIdx.x][n][3] = t3;
  g_trace_stamp[layer][blockIdx.x][n][4] = loop_cycles;
  g_trace_stamp[layer][blockIdx.x][n][5] = sync_cycles;
  g_trace_kind[layer][blockIdx.x][n] = kind;
  g_trace_count[layer][blockIdx.x] = n + 1;
}
#define MOE_TRACE_STAMP(var) var = wall_clock64()
#define MOE_TRACE_CYCLES(var) var = clock64()
#define MOE_TRACE_ADD_CYCLES(sum, since) sum += clock64() - since
#else
#define MOE_TRACE_STAMP(var)
#define MOE_TRACE_CYCLES(var)
#define MOE_TRACE_ADD_CYCLES(sum, since)
#endif

// Publishes one finished M-tile of column panel `panel` to the data-movement side: every wavefront makes its stores
// visible device-wide, then one thread bumps the panel's counter.
__device__ __forceinline__ void publish_panel(const GemmParams& p, int panel) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_fetch_add(&p.panel_done[panel], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// What a workgroup knows about a tile before it starts on it.
struct Tile {
  int idx;        // list position, -1: none
  ItemRec rec;
  int arow[8];    // rows of A this lane loads, per half of the tile's rows (layer0: gathered token rows, layer1: rows of h)
  int pre;        // 1: the loads of its first NS-1 stages were issued during the previous tile's epilogue
};
__device__ __forceinline__ ItemRec make_uniform(ItemRec r) {
  r.m_tile = uniform(r.m_tile); r.n_tile = uniform(r.n_tile); r.expert = uniform(r.expert); r.row0 = uniform(r.row0);
  r.nrows = uniform(r.nrows); r.kind = uniform(r.kind); r.ready_seg = uniform(r.ready_seg);
  return r;
}
__device__ __forceinline__ ItemRec load_item(const GemmParams& p, int idx) { return make_uniform(p.items[idx]); }
// Global offsets and running base pointers of a tile's operand loads.
struct LoadState {
  uint32_t aoff[8], boff[4];
  const char* Ab;
  const char* Bb;
};

// LDS of a tile of BM rows.  B is kept in a ring of NSX stages of one K step, loaded NSX - 1 steps ahead; A in a ring
// of NSX + 1 blocks in front of it, a block being one half of the tile's rows by 64
// values of K (128 bytes per row: whole cache lines of the operand, 8 rows per load instruction; fetching the 64
// bytes of one K step per row, 16 rows per instruction, is 1-2 % slower).  Block b = 2d + h holds rows [h*BM/2, (h+1)*BM/2) for
// K steps 2d and 2d+1; a block per K step is loaded, NSX - 1 steps ahead like B.
// NSX is 4 (three steps of lead) except for the 64-row tiles of the ragged expert ends, which get 6: a K step of
// theirs is 8 MFMAs per wavefront, so three steps of lead are a third of a memory round trip and the tile would
// spend half its time waiting for its operands; their small A blocks leave the LDS for two more B stages.
constexpr int kDeepStages = 6;
constexpr int a_block_bytes(int bm) { return bm * 64; }
constexpr int b_ring_offset(int bm, int nsx) { return (nsx + 1) * a_block_bytes(bm); }
// The epilogue stages C in 32 KiB that are free at the end of a tile even when the successor's first loads are under
// way (A blocks 0..2, B stages 0..2): A blocks 3 and 4 of a 256-row tile, the space behind the rings otherwise.
constexpr int staging_offset(int bm, int nsx) { return bm == 256 ? 3 * a_block_bytes(bm) : b_ring_offset(bm, nsx) + nsx * B_STAGE; }
constexpr int kLdsBytesShallow = b_ring_offset(256, NS) + NS * B_STAGE;   // 144 KiB; covers the smaller tiles' layouts with NSX = 4 too
constexpr int kLdsBytes = staging_offset(64, kDeepStages) + 32768;         // 156 KiB: the 64-row tiles with 6 stages
static_assert(staging_offset(128, NS) + 32768 <= kLdsBytesShallow && staging_offset(64, NS) + 32768 <= kLdsBytesShallow, "staging fits");
static_assert(kLdsBytes >= kLdsBytesShallow && kLdsBytes <= 160 * 1024 - 2048, "LDS of a compute unit, less the kernels' static variables");

// Rows of A the lane loads for a tile of the given height class: LA = 1, 2 or 4 loads per block and two blocks (row
// halves) per tile; a load covers 8 rows, 8 lanes per row.  arow[h * LA + j]: row half h, load j.
template <int MODE>
__device__ __forceinline__ void load_arows(const GemmParams& p, Tile& t, int lane, int w) {
  const int la = 1 << t.rec.kind;
#pragma unroll
  for (int i = 0; i < 8; i++) {
    if (i < 2 * la) {
      const int h = i / la, j = i % la;
      const int r = h * (32 * la) + (w * la + j) * 8 + (lane >> 3);
      const int sr = t.rec.row0 + (r < t.rec.nrows ? r : t.rec.nrows - 1);   // past the ragged end: the last row again
      t.arow[i] = MODE != MODE_L1 ? p.a_rows[sr] : sr;
    }
  }
}

// Address set-up of a tile and its first loads: A blocks and B stages 0 .. NSX-2, in the order A0 A1 B0 A2 B1 ...
// A(NSX-2) B(NSX-3) B(NSX-2) (what K step 0 needs first, then a block and a stage per further step).
// A: lane l of a load fetches the 16 bytes at position (l & 7) ^ ((row / 2) & 7) of its row's 128-byte line, so that
// the line lands in LDS (linearly, 16 bytes per lane) with its chunks XOR-swizzled by row: the 16 rows one pass of
// ds_read_b128 touches then fall on distinct banks.
template <int WM, int MT, int NT, int MODE, bool PK, int NSX>
__device__ __forceinline__ void setup_and_issue(const GemmParams& p, uint32_t lds0, const Tile& t, LoadState& ls, int lane,
                                                int w, bool issue) {
  constexpr int BM = WM * MT * 32;
  constexpr int A_BLOCK = a_block_bytes(BM);
  constexpr int B_RING = b_ring_offset(BM, NSX);
  constexpr int LA = BM / 64, LB = 4;
  constexpr int LEAD = NSX - 1;   // K steps the loads run ahead
#pragma unroll
  for (int i = 0; i < 2 * LA; i++) {
    const int r = (w * LA + i % LA) * 8 + (lane >> 3);   // row inside the block
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    ls.aoff[i] = (uint32_t)t.arow[i] * p.lda_bytes + c * 16;
  }
  const int col0 = (MODE == MODE_L0_SWIGLU) ? t.rec.n_tile * (BN / 2) : t.rec.n_tile * BN;
#pragma unroll
  for (int j = 0; j < LB; j++) {
    if (PK) {
      // packed weights: a stage is 16 KiB in a row, already in its LDS order
      ls.boff[j] = (uint32_t)((w * LB + j) * 1024 + lane * 16);
      continue;
    }
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
    ls.boff[j] = ((uint32_t)kr * p.ldb + gcol) * 2;
  }
  ls.Ab = uniform(p.A);
  ls.Bb = PK ? uniform(p.B + ((uint64_t)t.rec.expert * p.n_tiles_n + t.rec.n_tile) * ((uint64_t)(p.K / BK) * B_STAGE))
             : uniform(p.B + (uint64_t)t.rec.expert * p.b_expert_bytes);
  const size_t bstep = PK ? (size_t)B_STAGE : (size_t)BK * p.ldb * 2;
  if (issue) {
    auto a_block = [&](int b) {
#pragma unroll
      for (int j = 0; j < LA; j++)
        dma16(ls.Ab + (b >> 1) * 128, ls.aoff[(b & 1) * LA + j], lds0 + b * A_BLOCK + (w * LA + j) * 1024);
    };
    auto b_stage = [&](int st) {
#pragma unroll
      for (int j = 0; j < LB; j++) dma16(ls.Bb + st * bstep, ls.boff[j], lds0 + B_RING + st * B_STAGE + (w * LB + j) * 1024);
    };
    a_block(0);
    a_block(1);
    b_stage(0);
#pragma unroll
    for (int st = 2; st < LEAD; st++) {
      a_block(st);
      b_stage(st - 1);
    }
    b_stage(LEAD - 1);
  }
  ls.Bb += LEAD * bstep;   // ls.Ab stays the row start: the K position of A comes from the block number
}

// Workgroup-wide: is the source segment of tile t there?  block = true waits for it (up to the spin limit).
template <int MODE>
__device__ __forceinline__ bool segment_ready(const GemmParams& p, const Tile& t, volatile int32_t* lds_slot, bool block) {
  if (MODE == MODE_L1 || p.seg_ready == nullptr) return true;
  if (threadIdx.x == 0) {
    const uint32_t* flag = &p.seg_ready[t.rec.ready_seg];
    bool ok;
    if (block) {
      ok = spin_until_ge(flag, p.ready_epoch, p.spin_limit);
      if (!ok) atomicExch(p.status, (int)MOE_ERR_TIMEOUT);
    } else {
      ok = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) >= p.ready_epoch;
    }
    lds_slot[1] = ok;
  }
  __syncthreads();
  const bool ok = lds_slot[1] != 0;
  __syncthreads();
  if (ok) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "");
  return ok;
}

// One tile of BM = WM*MT*32 rows by 256 columns: address set-up and first loads, main loop, epilogue.  While the
// tile runs the workgroup finds out what its next tile is without waiting for any of the round trips: the queue
// atomic is issued up front; once the last operand load has landed (48 MFMAs before the end) its result is shared
// through LDS and the item record is requested.  A tile followed by one of the same height also starts the
// successor's first operand stages during its own epilogue (next.pre = 1); otherwise only the rows of A the next
// tile gathers are requested, after the epilogue.  next.idx = -1: no further tile.
template <int WM, int MT, int NT, int MODE, bool PK, int NSX = NS>
__device__ __forceinline__ void run_tile(const GemmParams& p, char* smem, volatile int32_t* lds_slot, const Tile& cur,
                                         Tile& next, int xcd, const Queue& q, int& pending_panel,
                                         volatile int32_t* lds_panel_count_ptr, volatile uint32_t* lds_mask) {
  constexpr int WN = 4 / WM;
  constexpr int BM = WM * MT * 32;
  static_assert(WN * NT * 32 == BN, "tile must be 256 columns wide");
  constexpr int A_BLOCK = a_block_bytes(BM);
  constexpr int B_RING = b_ring_offset(BM, NSX);
  constexpr int AB = NSX + 1;     // blocks of the A ring
  constexpr int LEAD = NSX - 1;   // K steps the loads run ahead; odd, so that the steps without loads at the end start on an odd step
  static_assert(LEAD % 2 == 1 && (BM != 256 || NSX == NS), "see staging_offset: the 256-row epilogue stages in A blocks 3 and 4");
  constexpr int LA = BM / 64;  // A loads per lane per K step (one block)
  constexpr int LB = 4;        // B loads per lane per K step (one stage)
  constexpr int LS = LA + LB;
  constexpr int FPB = BM / 64; // 32-row fragments per A block

#ifdef MOE_TILE_TRACE
  uint64_t tt0 = 0, tt1 = 0, tt2 = 0, tt3 = 0, tc_loop = 0, tc_sync = 0, tc_mark = 0;
#endif
  MOE_TRACE_STAMP(tt0);
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  // The thread index is made opaque per tile: otherwise the lane-dependent address constants of all three tile
  // heights are hoisted out of the tile loop, kept live across it and spilled.
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = w / WN, wn = w % WN;
  const int g = lane >> 4, j16 = lane & 15;
  const int row0 = uniform(cur.rec.row0), nrows = uniform(cur.rec.nrows), n_tile = uniform(cur.rec.n_tile);
  const int col0 = (MODE == MODE_L0_SWIGLU) ? n_tile * (BN / 2) : n_tile * BN;

  // LDS read addresses: a_rd[parity of the K step][16-deep half of the step] inside an A block, b_rd inside a B stage
  uint32_t a_rd[2][2], b_rd[NT];
  {
    const int l = lane & 31;
    const int s = (l >> 1) & 7;
#pragma unroll
    for (int sub = 0; sub < 2; sub++)
#pragma unroll
      for (int kk = 0; kk < 2; kk++) a_rd[sub][kk] = lds0 + l * 128 + (((sub * 4 + kk * 2 + (lane >> 5)) ^ s) << 4);
    const int swz = (j16 >> 2) | ((g >> 1) << 2);
    const int krow = 8 * (g >> 1) + (j16 >> 2);
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
      if (PK) {
        // column block of the packed tile this wavefront's block nt is: SwiGLU tiles hold [4 gate | 4 up] blocks of the
        // same 128 hidden units, of which a wavefront takes the gate and up blocks of its own units
        // (block nt lies a constant number of KiB behind block 0: b_block_offset below)
        const int c = MODE == MODE_L0_SWIGLU ? (nt / (NT / 2)) * 4 + wn * (NT / 2) + nt % (NT / 2) : wn * NT + nt;
        b_rd[nt] = lds0 + B_RING + c * 1024 + lane * 16;
      } else {
        b_rd[nt] = lds0 + B_RING + krow * 512 + (((wn * NT + nt) ^ swz) << 6) + (16 * (g & 1) + 4 * (j16 & 3)) * 2;
      }
    }
  }
  // Measurement aid: the fences a tile-granular hand-off between the two GroupGEMMs would need (a layer1 tile
  // acquiring what layer0 tiles on other XCDs released), without the hand-off itself.
  if (MODE == MODE_L1 && p.handoff_fences) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  // address set-up and the first loads (A blocks 0..2, B stages 0..2)
  LoadState ls;
  setup_and_issue<WM, MT, NT, MODE, PK, NSX>(p, lds0, cur, ls, lane, w, !cur.pre);
  const char* Ab = uniform(ls.Ab);
  const char* Bb = uniform(ls.Bb);
  const size_t bstep = PK ? (size_t)B_STAGE : (size_t)BK * p.ldb * 2;

  // Not cleared: the MFMAs of the tile's first half step take a zero constant as their addend instead (clearing 256
  // accumulator registers is 256 instructions, 0.8 us of a tile with the matrix cores idle).
  f32x16 acc[MT][NT];

  // Per K step and lane: LA loads of A (block kt+LEAD: the other half of the rows than the block before, 64 values of K)
  // and LB loads of B (stage kt+LEAD).  The loads are issued one at a time between groups of MFMAs: a burst would fill
  // the vector-memory queue and stall the MFMAs queued behind it.
  using P0 = std::integral_constant<int, 0>;
  using P1 = std::integral_constant<int, 1>;
  // Where K step kt finds its operands in the rings and where its loads go, kept incrementally: written as
  // (kt ...) % AB the compiler turns the read addresses into per-lane vectors that it rebases every step, and the
  // scalar divisions pile up at the top of the loop, where no MFMA covers them (2 % of the kernel's time).
  struct Ring {
    uint32_t oa, ob;      // LDS offsets of the A block of row half 0 of kt's pair of steps and of B stage kt
    uint32_t a0, a1;      // A blocks of step kt, row halves 0 and 1 (LDS offsets)
    uint32_t an0, an1;    // ... of step kt + 1
    uint32_t b, bn;       // B stage kt, kt + 1
    uint32_t adst, bdst;  // slots of A block kt + LEAD and B stage kt + LEAD
  };
  auto wrap_a = [](uint32_t x) { return x >= (uint32_t)AB * A_BLOCK ? x - (uint32_t)AB * A_BLOCK : x; };
  auto wrap_b = [](uint32_t x) {
    if constexpr ((NSX & (NSX - 1)) == 0) return x & ((uint32_t)NSX * B_STAGE - 1);   // (offsets are multiples of B_STAGE)
    else return x >= (uint32_t)NSX * B_STAGE ? x - (uint32_t)NSX * B_STAGE : x;
  };
  // The state of the step after r's, whose parity is PARNEW: the A ring's part and the B ring's part (worked out in
  // different groups of MFMAs, see half1 and half2).
  auto advance_a = [&](const Ring& r, Ring& n, auto parnew) {
    constexpr int PARNEW = decltype(parnew)::value;
    n.oa = PARNEW == 0 ? wrap_a(r.oa + 2 * A_BLOCK) : r.oa;   // an even step begins a new pair of A blocks
    n.a0 = r.an0;
    n.a1 = r.an1;
    if (PARNEW == 0) {
      n.an0 = n.a0;
      n.an1 = n.a1;
    } else {
      n.an0 = wrap_a(n.oa + 2 * A_BLOCK);
      n.an1 = wrap_a(n.oa + 3 * A_BLOCK);
    }
    n.adst = wrap_a(n.oa + (uint32_t)(LEAD + PARNEW) * A_BLOCK);
  };
  auto advance_b = [&](const Ring& r, Ring& n) {
    n.ob = wrap_b(r.ob + B_STAGE);
    n.b = r.bn;
    n.bn = wrap_b(n.ob + B_STAGE);
    n.bdst = wrap_b(n.ob + (uint32_t)LEAD * B_STAGE);
  };
  Ring ring, next_ring;   // K step 0; the step after it (filled in as the step goes)
  ring.oa = 0;
  ring.ob = 0;
  ring.a0 = ring.an0 = 0;
  ring.a1 = ring.an1 = A_BLOCK;
  ring.b = 0;
  ring.bn = B_STAGE;
  ring.adst = (uint32_t)LEAD * A_BLOCK;
  ring.bdst = (uint32_t)LEAD * B_STAGE;
  next_ring = ring;
  const char* a_src = Ab + ((LEAD - 1) / 2) * 128;   // what the A block of an even step is loaded from; + 128: of the odd step after it
  // where fragment q (32 rows) of this wavefront sits: row half and offset inside the block
  auto frag_off = [&](const uint32_t (&blk)[2], int q) {
    const int f = wm * MT + q;   // WM == 2: f / FPB == wm for every q
    return (WM == 2 ? (wm ? blk[1] : blk[0]) : blk[f / FPB]) + (uint32_t)(f % FPB) * (32 * 128);
  };
  // The read addresses of a half step as one per-lane base per operand plus constants that go into the instructions'
  // offset fields: one address addition per operand and half step instead of one per fragment.
  //   A: the block (or, 64-row tiles, the two blocks) the wavefront's fragments lie in; fragment q is q * 4 KiB further on
  //   B (packed): block 0 of the wavefront; block nt is b_block_offset(nt) further on
  struct HalfBases { uint32_t a[2], b; };
  auto half_bases = [&](const uint32_t (&blk)[2], uint32_t b_off, int rd_par, int rd_kk) {
    HalfBases hb;
    hb.a[0] = (WM == 2 ? (wm ? blk[1] : blk[0]) : blk[0]) + a_rd[rd_par][rd_kk];
    hb.a[1] = WM == 2 ? hb.a[0] : blk[1] + a_rd[rd_par][rd_kk];
    hb.b = b_off + b_rd[0] + rd_kk * (B_STAGE / 2);
    return hb;
  };
  auto a_frag_addr = [&](const HalfBases& hb, int q) {
    // WM == 2: f = wm * MT + q lies in block wm at position q (MT == FPB); WM == 1: fragment q is block q / FPB
    return WM == 2 ? hb.a[0] + (uint32_t)q * (32 * 128) : hb.a[q / FPB] + (uint32_t)(q % FPB) * (32 * 128);
  };
  auto b_block_offset = [](int nt) {
    return (uint32_t)(MODE == MODE_L0_SWIGLU ? (nt / (NT / 2)) * 4 + nt % (NT / 2) : nt) * 1024;
  };
  static_assert(WM == 1 || MT == FPB, "a wavefront's fragments fill one A block");
  bf16x8 af[2][MT], bfr[2][NT];
  // Group q (of 4) of a half step: the LDS reads of fragment q for the next half step and a quarter of the MFMAs
  // of this one.  blk / b_off / rd_par / rd_kk: A blocks, B stage, parity and 16-deep half of the step read from.
  auto group = [&](int cb, int nb, const HalfBases& hb, uint32_t b_off, int rd_kk, int q, auto first) {
    constexpr bool FIRST = decltype(first)::value;   // the tile's first half step: nothing accumulated yet
    constexpr int PER = MT * NT / 4;
    // The fragments of the next half step are all requested in the first kReadGroups groups, so that they are back
    // well before the half step ends: the workgroup barrier between the halves waits for every outstanding LDS
    // read, and a read issued just before it would stall all four matrix pipes for an LDS round trip.
    int n_reads = 0;
#pragma unroll
    for (int f = q * kFragsPerGroup; f < (q + 1) * kFragsPerGroup; f++) {
      if (q < kReadGroups && f < MT) {
        af[nb][f] = lds_read_a(a_frag_addr(hb, f));
        n_reads += 1;
      }
      if (q < kReadGroups && f < NT) {
        if (PK) bfr[nb][f] = lds_read_b_packed(hb.b + b_block_offset(f));
        else bfr[nb][f] = lds_read_b(b_off + b_rd[f] + rd_kk * 16 * 512, b_off + b_rd[f] + (rd_kk * 16 + 4) * 512);
        n_reads += PK ? 1 : 2;
      }
    }
#pragma unroll
    for (int i = 0; i < PER; i++) {
      const int m = q * PER + i, mt = m / NT, nt = m % NT;
      if constexpr (FIRST) acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cb][nt], af[cb][mt], (f32x16){0}, 0, 0, 0);
      else acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cb][nt], af[cb][mt], acc[mt][nt], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < PER; i++) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < n_reads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
#pragma unroll
    for (int i = PER; i < 12; i++)
      if (i < n_reads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
  };
  // read addresses of the half step about to begin (first half of step 0) and of the one after it
  HalfBases hb_first, hb_second;
  {
    const uint32_t blk0[2] = {ring.a0, ring.a1};
    hb_first = half_bases(blk0, ring.b, 0, 1);
    hb_second = hb_first;
  }
  // first half of K step kt (parity PAR): MFMAs of its first 16 values of K, fragments of its second 16, A block kt+LEAD
  auto half1 = [&](auto par, bool do_issue, auto first) {
    constexpr int PAR = decltype(par)::value;
    const uint32_t blk[2] = {ring.a0, ring.a1};
    const uint32_t b_off = ring.b;
    const char* src = a_src + PAR * 128;
    const uint32_t dst = lds0 + ring.adst + w * LA * 1024;
    const HalfBases hb = hb_first;   // worked out under the MFMAs of the half step before
    (void)blk;
#pragma unroll
    for (int q = 0; q < 4; q++) {
      if (q > 0) __builtin_amdgcn_sched_barrier(0);   // the loads stay where they are written: one per group
      if (q == 3) {   // under this group's MFMAs: the A ring's next positions, and the read addresses of the second half
        advance_a(ring, next_ring, std::integral_constant<int, 1 - PAR>{});
        const uint32_t blk2[2] = {ring.an0, ring.an1};
        hb_second = half_bases(blk2, ring.bn, 1 - PAR, 0);
      }
      group(0, 1, hb, b_off, 1, q, first);
      // (behind the group's MFMAs, so that a half step begins with an MFMA and not with the load's set-up)
      if (do_issue && q < LA) {
        const uint32_t off = ls.aoff[((PAR + LEAD) & 1) * LA + q];
        if (q == 0) dma16_at<0>(src, off, dst);
        else if (q == 1) dma16_at<1024>(src, off, dst);
        else if (q == 2) dma16_at<2048>(src, off, dst);
        else dma16_at<3072>(src, off, dst);
      }
    }
  };
  // second half: MFMAs of the second 16 values, fragments of the first 16 of step kt+1, B stage kt+LEAD; the last
  // groups of both halves also work out where the next step finds its operands, so that this is done under MFMAs
  auto half2 = [&](auto par, bool do_issue) {
    constexpr int PAR = decltype(par)::value;
    const uint32_t blk[2] = {ring.an0, ring.an1};
    const uint32_t b_off = ring.bn;
    const uint32_t dst = lds0 + B_RING + ring.bdst + w * LB * 1024;
    const HalfBases hb = hb_second;
    (void)blk;
#pragma unroll
    for (int q = 0; q < 4; q++) {
      if (q > 0) __builtin_amdgcn_sched_barrier(0);
      if (q == 3) {   // the B ring's next positions, and the read addresses of the next step's first half
        advance_b(ring, next_ring);
        const uint32_t blk1[2] = {next_ring.a0, next_ring.a1};
        hb_first = half_bases(blk1, next_ring.b, 1 - PAR, 1);
      }
      group(1, 0, hb, b_off, 0, q, std::false_type{});
      if (do_issue && q < LB) {
        if (q == 0) dma16_at<0>(Bb, ls.boff[q], dst);
        else if (q == 1) dma16_at<1024>(Bb, ls.boff[q], dst);
        else if (q == 2) dma16_at<2048>(Bb, ls.boff[q], dst);
        else dma16_at<3072>(Bb, ls.boff[q], dst);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    ring = next_ring;
    if (PAR == 1) a_src += 128;
  };

  // The next item of this XCD's queue is requested before anything else of this tile is outstanding; the
  // operand loads of the first stages were issued before (by the previous tile, or by the kernel for the first).
  int next_raw = 0;
  if (tid == 0) next_raw = take_from(p, xcd, q.own_len, q.own_base);
  // A tile starts the loads of a successor of its own height during its epilogue, which needs the successor's
  // segment to be there already: the ready flags are sampled here (lane s of the first wavefront reads
  // flag s) and looked at when the successor is known.  A flag raised later than this only costs the early start.
  constexpr bool kCanPre = true;   // (kept as a switch: the early start costs about 30 VGPRs)
  constexpr int kKind = (WM == 2 && MT == 4) ? 2 : (WM == 2 ? 1 : 0);   // height class of this variant's tiles
  const bool flags_on = MODE != MODE_L1 && p.seg_ready != nullptr;
  uint32_t flag_v = 0;
  if (kCanPre && flags_on && tid < p.n_segments)
    flag_v = __hip_atomic_load(&p.seg_ready[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);

  const int nk = p.K / BK;  // even and >= 4 (checked on the host)
  // A blocks 0 and 1 and B stage 0 landed?  Everything issued after them (A blocks 2 .. LEAD-1, B stages 1 .. LEAD-1, and
  // whatever the previous tile's epilogue stored) may still be outstanding; loads return in order.
  wait_vmcnt<(LEAD - 2) * LA + (LEAD - 1) * LB>();
  block_barrier();
  MOE_TRACE_STAMP(tt1);
  MOE_TRACE_CYCLES(tc_loop);
  {
    const uint32_t blk[2] = {ring.a0, ring.a1};
#pragma unroll
    for (int mt = 0; mt < MT; mt++) af[0][mt] = lds_read_a(frag_off(blk, mt) + a_rd[0][0]);
  }
#pragma unroll
  for (int nt = 0; nt < NT; nt++) bfr[0][nt] = PK ? lds_read_b_packed(b_rd[nt]) : lds_read_b(b_rd[nt], b_rd[nt] + 4 * 512);

  int kt = 0;
  auto step = [&](auto par, auto first) {
    half1(par, true, first);
    // B stage kt+1 and the A blocks of step kt+1 (up to block kt+2) have landed for this lane; younger, in issue
    // order: B stage kt+2, blocks and stages kt+3 .. kt+LEAD-1, A block kt+LEAD: LEAD-2 steps' worth of loads.
    // After the barrier they have for all, and all are done reading step kt.  The scheduler must not move MFMAs of the
    // first half behind the barrier: they are what covers the latency of the half's LDS reads before the wait.
    __builtin_amdgcn_sched_barrier(0);
    MOE_TRACE_CYCLES(tc_mark);
    wait_vmcnt<(LEAD - 2) * LS>();
    block_barrier();
    MOE_TRACE_ADD_CYCLES(tc_sync, tc_mark);
    __builtin_amdgcn_sched_barrier(0);
    half2(par, true);
    Bb += bstep;
    kt++;
  };
  const int kt_end = nk - LEAD;   // odd; at least 1 (the caller picks NSX so that nk > LEAD)
  step(P0{}, std::true_type{});   // kt_end is odd: an even number of steps with loads follows
  while (kt + 2 <= kt_end) {
    step(P1{}, std::false_type{});
    step(P0{}, std::false_type{});
  }

  // The last LEAD steps (parities 1, 0, ..., 1) issue nothing.  With r steps still to come after the current one, what
  // is younger than the loads the step waits for is B stage kt+2 and the blocks and stages of the r-2 steps after it.
  static_assert(LEAD == 3 || LEAD == 5, "the steps without loads are written out for these two");
  if constexpr (LEAD == 5) {
    half1(P1{}, false, std::false_type{});
    __builtin_amdgcn_sched_barrier(0);
    wait_vmcnt<LB + 2 * LS>();
    block_barrier();
    __builtin_amdgcn_sched_barrier(0);
    half2(P1{}, false);
    kt++;
    half1(P0{}, false, std::false_type{});
    __builtin_amdgcn_sched_barrier(0);
    wait_vmcnt<LB + LS>();
    block_barrier();
    __builtin_amdgcn_sched_barrier(0);
    half2(P0{}, false);
    kt++;
  }
  half1(P1{}, false, std::false_type{});
  wait_vmcnt<LB>();   // younger than the last A block: the last B stage
  block_barrier();
  half2(P1{}, false);
  kt++;
  half1(P0{}, false, std::false_type{});
  wait_vmcnt<0>();
  // No operand load is in flight any more, so memory operations the compiler waits for by itself no longer stall
  // behind them: thread 0 turns its queue ticket into a list position (stealing from other XCDs if its own queue is
  // used up) and hands it to the workgroup across the barrier; everybody then asks for the item record, whose
  // latency the remaining 48 MFMAs cover.
  uint64_t ready_mask = ~0ull;
  if (kCanPre && flags_on) ready_mask = __ballot(tid < p.n_segments && flag_v >= p.ready_epoch);
  if (tid == 0) {
    if (next_raw < 0) next_raw = steal(p, xcd);
    lds_slot[0] = next_raw;
    if (kCanPre && flags_on) {
      lds_mask[0] = (uint32_t)ready_mask;
      lds_mask[1] = (uint32_t)(ready_mask >> 32);
    }
  }
  block_barrier();
  next.idx = uniform((int)lds_slot[0]);
  if (kCanPre && flags_on)
    ready_mask = (uint32_t)uniform((int)lds_mask[0]) | ((uint64_t)(uint32_t)uniform((int)lds_mask[1]) << 32);
  ItemRec raw_rec;
  if (next.idx >= 0) raw_rec = p.items[next.idx];
  half2(P0{}, false);
  kt++;
  half1(P1{}, false, std::false_type{});
#pragma unroll
  for (int mt = 0; mt < MT; mt++)
#pragma unroll
    for (int nt = 0; nt < NT; nt++)
      acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[1][nt], af[1][mt], acc[mt][nt], 0, 0, 0);

  // The previous tile is published only now: its stores have drained during this tile's main loop, so the release
  // does not wait for them (publishing right after the stores would stall the next tile behind the store burst).
  if (MODE == MODE_L1 && pending_panel >= 0) {
    publish_panel(p, pending_panel);
    pending_panel = -1;
  }
  if (MODE != MODE_L1 && p.handoff_fences) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // the previous tile's stores
  block_barrier();   // every wavefront is done reading the operand stages
  MOE_TRACE_STAMP(tt2);
#ifdef MOE_TILE_TRACE
  tc_loop = clock64() - tc_loop;
#endif

  if (next.idx >= 0) next.rec = make_uniform(raw_rec);
  // early start of the successor (see above): its gather rows are requested now, its first loads after the first
  // 32-row block of the epilogue, into LDS the epilogue does not use
  bool do_pre = false;
  if (kCanPre && !p.no_pre && next.idx >= 0 && next.rec.kind == kKind && ((ready_mask >> (next.rec.ready_seg & 63)) & 1)) do_pre = true;
  next.pre = do_pre;
  if (kCanPre && do_pre) load_arows<MODE>(p, next, lane, w);

  // Epilogue.  The MFMAs ran with the operands swapped (B fragment first), so a lane holds, for output row
  // lane & 31 of each 32x32 block, the columns 8*(i/4) + 4*(lane/32) + i%4: four consecutive columns per group of
  // four accumulator registers.  The wavefront's part of the tile goes out in pieces of 32 rows x 128 bytes (64 bytes
  // where the wavefront has a single 32-column block of output): a piece
  // is staged in LDS as bf16 (8-byte writes, 16-byte chunks XOR-swizzled by row) and written out in full 16-byte
  // chunks, 8 rows of 128 bytes per store instruction; 2-byte stores straight from the accumulators cost a tenth of
  // the tile's time.  Two staging buffers per wavefront: while piece s is converted and staged, the chunks of piece
  // s-1 are on their way back from LDS, so that only the first and the last piece pay an LDS round trip.
  constexpr int OUT_NT = (MODE == MODE_L0_SWIGLU) ? NT / 2 : NT;   // 32-column blocks of output per wavefront
  constexpr int PW = OUT_NT >= 2 ? 2 : 1;                           // 32-column blocks per piece
  constexpr int PH = OUT_NT / PW;                                   // pieces per 32-row block
  constexpr int PRB = PW * 64;                                      // bytes per staged row of a piece
  constexpr int PNC = PRB / 16;                                     // 16-byte chunks per staged row
  constexpr int RPB = 256 / PRB;                                    // rows per 256 bytes of LDS banks
  constexpr int NST = 32 * PNC / 64;                                // 16-byte stores per lane and piece
  constexpr int NPIECE = MT * PH;
  static_assert(OUT_NT % PW == 0, "pieces tile the wavefront's columns");
  const uint32_t cbase = lds0 + staging_offset(BM, NSX) + w * (2 * 32 * PRB);   // 2 buffers x 32 rows x 128 bytes per wavefront
  int lane_e = lane;   // opaque again: the epilogue's addresses are computed here, not before the main loop
  asm volatile("" : "+v"(lane_e));
  const int col_base = (MODE == MODE_L0_SWIGLU) ? col0 + wn * (NT * 16) : col0 + wn * (NT * 32);
  const bool full = nrows == BM;
  // converts piece s (row block s / PH, column blocks 2 * (s % PH) and the next) and stages it in buffer s & 1
  auto stage_piece = [&](int s) {
    const int mt = s / PH, nt0 = (s % PH) * PW;
    const int m = lane_e & 31, half = lane_e >> 5;
    const uint32_t row_addr = cbase + (s & 1) * (32 * PRB) + m * PRB + half * 8;
    const int sw = (m / RPB) & (PNC - 1);
#pragma unroll
    for (int n2 = 0; n2 < PW; n2++) {
      const int nt = nt0 + n2;
      if (MODE == MODE_L0_GELU) __builtin_amdgcn_sched_barrier(0);  // bounds the live activation temporaries
#pragma unroll
      for (int qd = 0; qd < 4; qd++) {
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
          if (MODE == MODE_L0_SWIGLU) v[i] = silu(acc[mt][nt][qd * 4 + i]) * acc[mt][nt + NT / 2][qd * 4 + i];
          else if (MODE == MODE_L0_GELU) v[i] = gelu_erf(acc[mt][nt][qd * 4 + i]);
          else v[i] = acc[mt][nt][qd * 4 + i];
        }
        bf16x2 lo = {(__bf16)v[0], (__bf16)v[1]}, hi = {(__bf16)v[2], (__bf16)v[3]};
        u32x2 pk = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
        const int chunk = n2 * 4 + qd;
        *(u32x2 __attribute__((address_space(3)))*)(uintptr_t)(row_addr + ((chunk ^ sw) << 4)) = pk;
      }
    }
  };
  // reads the 16-byte chunks of piece s this lane stores (rows it * 8 + lane / 8, chunk lane % 8)
  auto fetch_piece = [&](int s, u32x4* v) {
    const int c = lane_e % PNC;
#pragma unroll
    for (int it = 0; it < NST; it++) {
      const int r = it * (64 / PNC) + lane_e / PNC;
      v[it] = *(const u32x4 __attribute__((address_space(3)))*)(uintptr_t)(
          cbase + (s & 1) * (32 * PRB) + r * PRB + ((c ^ ((r / RPB) & (PNC - 1))) << 4));
    }
  };
  auto store_piece = [&](int s, const u32x4* v) {
    const int mt = s / PH, ph = s % PH;
    const int c = lane_e % PNC;
#pragma unroll
    for (int it = 0; it < NST; it++) {
      const int grow = wm * (MT * 32) + mt * 32 + it * (64 / PNC) + lane_e / PNC;
      u32x4* dst = (u32x4*)(p.C + (size_t)(row0 + grow) * p.ldc + col_base + ph * (PW * 32) + c * 8);
      if (full) *dst = v[it];
      else if (grow < nrows) *dst = v[it];
    }
  };
  stage_piece(0);
#pragma unroll
  for (int s = 1; s <= NPIECE; s++) {
    __builtin_amdgcn_sched_barrier(0);   // one piece at a time: keeps the address temporaries few
    u32x4 v[NST];
    fetch_piece(s - 1, v);
    if (s < NPIECE) stage_piece(s);
    store_piece(s - 1, v);
    if constexpr (kCanPre) {
      if (s == PH && do_pre) {   // the first 32-row block is out
        if (flags_on) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "");
        LoadState ls_next;
        setup_and_issue<WM, MT, NT, MODE, PK, NSX>(p, lds0, next, ls_next, lane_e, w, true);
      }
    }
  }
  if (MODE == MODE_L1 && p.fused_combine) {
    if (p.batch_publish) {
      if (tid == 0) lds_panel_count_ptr[n_tile] += 1;
    } else {
      pending_panel = n_tile;
    }
  }
  // Top-k reduction in the layer1 epilogue (the vertical fusion Section 3.2.1 weighs against its specialised
  // blocks).  The k rows of a token lie in tiles of different experts, finished by different workgroups at different
  // times, so the tile still writes its rows of Y; then every row announces itself on a counter per (token, column
  // panel), and the row that finds the other k-1 already there reduces the token: it reads the k rows back in slot
  // order and writes the output row -- the same sum in the same order as the stand-alone kernel, whoever comes last.
  // Nobody waits for anybody; the price is one device-wide release per tile (the rows must be visible before they are
  // announced) and one acquire.
  if (MODE == MODE_L1 && p.epilogue_combine) {
    volatile int32_t* last_list = (volatile int32_t*)(smem + staging_offset(BM, NSX));   // the staging area is free again
    int32_t* last_count = (int32_t*)(smem + staging_offset(BM, NSX) + 256 * 4);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __syncthreads();
    if (tid == 0) *last_count = 0;
    __syncthreads();
    const int n_panels = p.H / BN;
    if (tid < nrows) {
      const int t = p.perm[row0 + tid] / p.k;
      const uint32_t before = __hip_atomic_fetch_add(&p.arrive[(size_t)t * n_panels + n_tile], 1u, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
      if (before + 1 == (uint32_t)p.k) last_list[atomicAdd(last_count, 1)] = t;
    }
    __syncthreads();
    const int n_last = uniform(*(volatile int32_t*)last_count);
    if (n_last > 0) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      const size_t col = (size_t)n_tile * BN + (tid & 31) * 8;
      for (int e = tid >> 5; e < n_last; e += 8) {
        const int t = last_list[e];
        float acc[8];
#pragma unroll
        for (int c = 0; c < 8; c++) acc[c] = 0.f;
        for (int j = 0; j < p.k; j++) {
          const int row = p.inv_perm[t * p.k + j];
          const float wj = p.topk_weights[t * p.k + j];
          const u32x4 v = *(const u32x4*)(p.C + (size_t)row * p.ldc + col);
#pragma unroll
          for (int c = 0; c < 4; c++) {
            acc[2 * c] += wj * __uint_as_float(v[c] << 16);
            acc[2 * c + 1] += wj * __uint_as_float(v[c] & 0xffff0000u);
          }
        }
        u32x4 o;
#pragma unroll
        for (int c = 0; c < 4; c++) {
          bf16x2 pr = {(__bf16)acc[2 * c], (__bf16)acc[2 * c + 1]};
          o[c] = __builtin_bit_cast(uint32_t, pr);
        }
        *(u32x4*)(p.out + (size_t)t * p.H + col) = o;
      }
    }
    __syncthreads();   // the list is read out before the next tile's epilogue reuses the staging area
  }
  // rows of A the next tile gathers (requested only now: held across the epilogue they push it into spilling)
  if (next.idx >= 0 && !do_pre) load_arows<MODE>(p, next, lane, w);
#ifdef MOE_TILE_TRACE
  MOE_TRACE_STAMP(tt3);
  trace_tile(MODE == MODE_L1 ? 1 : 0, kKind + (cur.pre ? 4 : 0), tt0, tt1, tt2, tt3, tc_loop, tc_sync, lds_mask + 2);
#endif
}

template <int MODE, bool PK>
__global__ __launch_bounds__(256, 1) void k_group_gemm(GemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int32_t lds_slot[2];
  __shared__ uint32_t lds_mask[4];   // 0, 1: ready flags seen by the workgroup; 2, 3: tiles noted by a measurement build
  __shared__ int32_t lds_panel_count[kMaxPanels];   // layer1, batched publication: tiles finished per column panel
  const int tid = threadIdx.x;
#ifdef MOE_TILE_TRACE
  if (tid == 0) {   // a workgroup that gets no tile in this launch has noted none
    lds_mask[2] = lds_mask[3] = 0;
    if (blockIdx.x < kTraceWgs) g_trace_count[MODE == MODE_L1 ? 1 : 0][blockIdx.x] = 0;
  }
#endif
  if (MODE == MODE_L1) {
    for (int i = tid; i < kMaxPanels; i += 256) lds_panel_count[i] = 0;
  }
  if (PK && prefetch_role(p)) return;
  if (MODE == MODE_L1 && (int)blockIdx.x >= p.n_mfma) {
    if (p.fused_combine) combine_loop(p, &lds_slot[1], false);
    return;
  }
  const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int xcd = blockIdx.x & (kXcds - 1);
  Queue q;
  q.own_len = p.queue_len[xcd];
  q.own_base = queue_pos(p, xcd, 0);
  int pending_panel = -1;   // layer1: column panel of the last finished tile, not yet published
  // 64-row tiles run with the deeper operand rings whenever the reduction is long enough to fill them
  const bool deep64 = p.deep_short_tiles && p.K / BK > kDeepStages - 1;

  // first tile: found synchronously
  Tile cur, next;
  auto take_sync = [&](Tile& t) {
    if (tid == 0) {
      int idx = take_from(p, xcd, q.own_len, q.own_base);
      if (idx < 0) idx = steal(p, xcd);
      lds_slot[0] = idx;
    }
    __syncthreads();
    t.idx = uniform((int)lds_slot[0]);
    t.pre = 0;
    __syncthreads();
    if (t.idx >= 0) {
      t.rec = load_item(p, t.idx);
      load_arows<MODE>(p, t, lane, w);
    }
  };
  take_sync(cur);
  while (cur.idx >= 0) {
    // every wavefront is done with the LDS of the previous tile before its slots are refilled
    __syncthreads();
    if (!cur.pre && !segment_ready<MODE>(p, cur, lds_slot, true)) {
      take_sync(cur);   // timed out (status says so): give the tile up and take another one
      continue;
    }
    next.idx = -1;
    if (cur.rec.kind == 2) run_tile<2, 4, 4, MODE, PK>(p, smem, lds_slot, cur, next, xcd, q, pending_panel, lds_panel_count, lds_mask);
    else if (cur.rec.kind == 1) run_tile<2, 2, 4, MODE, PK>(p, smem, lds_slot, cur, next, xcd, q, pending_panel, lds_panel_count, lds_mask);
    else if (deep64) run_tile<1, 2, 2, MODE, PK, kDeepStages>(p, smem, lds_slot, cur, next, xcd, q, pending_panel, lds_panel_count, lds_mask);
    else run_tile<1, 2, 2, MODE, PK>(p, smem, lds_slot, cur, next, xcd, q, pending_panel, lds_panel_count, lds_mask);
    cur = next;
  }
  if (MODE == MODE_L1 && p.fused_combine) {
    if (p.batch_publish) {
      // no data-movement workgroup is waiting for single tiles: one release for everything this workgroup wrote
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      __syncthreads();
      for (int i = tid; i < p.H / BN; i += 256)
        if (lds_panel_count[i] > 0)
          __hip_atomic_fetch_add(&p.panel_done[i], (uint32_t)lds_panel_count[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else if (pending_panel >= 0) {
      publish_panel(p, pending_panel);
    }
    combine_loop(p, &lds_slot[1], p.batch_publish != 0);
  }
}

// ---------------------------------------------------------------------------------------------
// Both GroupGEMMs in one persistent launch (the pipelining between the layers of Fig. 3/4 without a kernel boundary
// in between).  A workgroup first walks the layer0 queues exactly as k_group_gemm does, counting its finished tiles
// per M-tile in LDS; every publish_every tiles, and when the layer0 queues are used up, it makes its stores visible
// device-wide (one agent-scope release for all tiles since the last one: a release per tile would cost a tenth of
// layer0) and adds its counts to tile_done[].  It then walks the layer1 queues; a layer1 tile of M-tile m starts once
// tile_done[m] has reached the number of layer0 column tiles.  No deadlock: a workgroup only reaches layer1 after
// every layer0 item has been handed out, and the workgroups holding them wait for nothing but the ready flags (a
// bounded wait).  Once a workgroup has seen every workgroup finish layer0 it stops checking, and only then lets a
// tile start its successor's loads early.
// ---------------------------------------------------------------------------------------------
template <int MODE0, bool PK>
__global__ __launch_bounds__(256, 1) void k_fused_layers(GemmParams p0, GemmParams p1, FuseParams f) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int32_t lds_slot[2];
  __shared__ uint32_t lds_mask[4];   // 0, 1: ready flags seen by the workgroup; 2, 3: tiles noted by a measurement build
  __shared__ int32_t lds_panel_count[kMaxPanels];      // unused here; run_tile takes it
  __shared__ int32_t lds_tile_cnt[kScheduleTileCap];   // layer0 tiles this workgroup finished per M-tile, not yet published
  const int tid = threadIdx.x;
#ifdef MOE_TILE_TRACE
  if (tid == 0) {
    lds_mask[2] = lds_mask[3] = 0;
    if (blockIdx.x < kTraceWgs) g_trace_count[0][blockIdx.x] = g_trace_count[1][blockIdx.x] = 0;
  }
#endif
  for (int i = tid; i < kScheduleTileCap; i += 256) lds_tile_cnt[i] = 0;
  for (int i = tid; i < kMaxPanels; i += 256) lds_panel_count[i] = 0;
  const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int xcd = blockIdx.x & (kXcds - 1);
  const int n_tiles = min(*p0.n_tiles, (int)kScheduleTileCap);
  int pending_panel = -1;
  __syncthreads();

  auto take_sync = [&](const GemmParams& p, const Queue& q, Tile& t, auto mode) {
    constexpr int MODE = decltype(mode)::value;
    if (tid == 0) {
      int idx = take_from(p, xcd, q.own_len, q.own_base);
      if (idx < 0) idx = steal(p, xcd);
      lds_slot[0] = idx;
    }
    __syncthreads();
    t.idx = uniform((int)lds_slot[0]);
    t.pre = 0;
    __syncthreads();
    if (t.idx >= 0) {
      t.rec = load_item(p, t.idx);
      load_arows<MODE>(p, t, lane, w);
    }
  };
  // all stores of this workgroup so far become visible device-wide, then its counts are added
  auto publish = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __syncthreads();
    for (int i = tid; i < n_tiles; i += 256) {
      const int c = lds_tile_cnt[i];
      if (c > 0) {
        __hip_atomic_fetch_add(&f.tile_done[i], (uint32_t)c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lds_tile_cnt[i] = 0;
      }
    }
    __syncthreads();
  };

  // ---- layer0
  {
    using M0 = std::integral_constant<int, MODE0>;
    Queue q;
    q.own_len = p0.queue_len[xcd];
    q.own_base = queue_pos(p0, xcd, 0);
    Tile cur, next;
    int since_publish = 0;
    take_sync(p0, q, cur, M0{});
    while (cur.idx >= 0) {
      __syncthreads();
      if (!cur.pre && !segment_ready<MODE0>(p0, cur, lds_slot, true)) {
        take_sync(p0, q, cur, M0{});   // timed out (status says so): the tile is given up
        continue;
      }
      next.idx = -1;
      const int m_tile = cur.rec.m_tile;
      if (cur.rec.kind == 2) run_tile<2, 4, 4, MODE0, PK>(p0, smem, lds_slot, cur, next, xcd, q, pending_panel, lds_panel_count, lds_mask);
      else if (cur.rec.kind == 1) run_tile<2, 2, 4, MODE0, PK>(p0, smem, lds_slot, cur, next, xcd, q, pending_panel, lds_panel_count, lds_mask);
      else run_tile<1, 2, 2, MODE0, PK>(p0, smem, lds_slot, cur, next, xcd, q, pending_panel, lds_panel_count, lds_mask);
      if (tid == 0 && (unsigned)m_tile < (unsigned)kScheduleTileCap) lds_tile_cnt[m_tile] += 1;
      cur = next;
      if (++since_publish >= f.publish_every && cur.idx >= 0) {
        // (if the successor's first loads are already in flight the fence waits for them too; the tile code's own
        // waits then find them done)
        publish();
        since_publish = 0;
      }
    }
    __syncthreads();
    publish();
    if (tid == 0) __hip_atomic_fetch_add(f.wgs_done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  // ---- layer1
  {
    using M1 = std::integral_constant<int, MODE_L1>;
    if ((int)blockIdx.x >= p1.n_mfma) return;
    GemmParams q1 = p1;
    q1.no_pre = 1;
    bool all_seen = false;
    Queue q;
    q.own_len = q1.queue_len[xcd];
    q.own_base = queue_pos(q1, xcd, 0);
    Tile cur, next;
    take_sync(q1, q, cur, M1{});
    while (cur.idx >= 0) {
      __syncthreads();
      if (!all_seen) {
        // the rows of this M-tile: wait until every layer0 column tile of it has been published
        if (tid == 0) {
          const uint32_t m = (uint32_t)cur.rec.m_tile < (uint32_t)kScheduleTileCap ? (uint32_t)cur.rec.m_tile : 0u;
          bool ok = spin_until_ge(&f.tile_done[m], (uint32_t)f.n_tiles_n0, q1.spin_limit ? q1.spin_limit : (1u << 26));
          if (!ok) atomicExch(q1.status, (int)MOE_ERR_TIMEOUT);
          const uint32_t done = __hip_atomic_load(f.wgs_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          lds_slot[1] = (ok ? 1 : 0) | (done >= gridDim.x ? 2 : 0);
        }
        __syncthreads();
        const int st = lds_slot[1];
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if (!(st & 1)) {
          take_sync(q1, q, cur, M1{});   // timed out: give the tile up
          continue;
        }
        if (st & 2) {
          all_seen = true;     // every workgroup has published everything: nothing left to wait for
          q1.no_pre = 0;
        }
      }
      next.idx = -1;
      if (cur.rec.kind == 2) run_tile<2, 4, 4, MODE_L1, PK>(q1, smem, lds_slot, cur, next, xcd, q, pending_panel, lds_panel_count, lds_mask);
      else if (cur.rec.kind == 1) run_tile<2, 2, 4, MODE_L1, PK>(q1, smem, lds_slot, cur, next, xcd, q, pending_panel, lds_panel_count, lds_mask);
      else run_tile<1, 2, 2, MODE_L1, PK>(q1, smem, lds_slot, cur, next, xcd, q, pending_panel, lds_panel_count, lds_mask);
      cur = next;
    }
  }
}

// The kernels need more dynamic LDS than the default limit.  The attribute belongs to the function on one device; it is
// set once per function and device (a bit per device, set after the call succeeded: two threads racing set it twice,
// which is harmless) and never inside a launch that may be under stream capture.
static hipError_t allow_large_lds(const void* kern, int lds_bytes) {
  struct Entry { const void* kern; std::atomic<uint64_t> devices; };
  static Entry entries[16];
  static std::atomic<int> n_entries{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  const int n = n_entries.load(std::memory_order_acquire);
  for (int i = 0; i < n; i++)
    if (entries[i].kern == kern && (entries[i].devices.load(std::memory_order_acquire) & bit)) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  if (e != hipSuccess) return e;
  for (int i = 0; i < n; i++)
    if (entries[i].kern == kern) {
      entries[i].devices.fetch_or(bit, std::memory_order_release);
      return hipSuccess;
    }
  static std::mutex mu;
  std::lock_guard<std::mutex> lock(mu);
  const int m = n_entries.load(std::memory_order_acquire);
  for (int i = 0; i < m; i++)
    if (entries[i].kern == kern) {
      entries[i].devices.fetch_or(bit, std::memory_order_release);
      return hipSuccess;
    }
  if (m < 16) {
    entries[m].kern = kern;
    entries[m].devices.store(bit, std::memory_order_release);
    n_entries.store(m + 1, std::memory_order_release);
  }
  return hipSuccess;   // table full: the attribute is simply set again next time
}

template <int MODE0, bool PK>
static hipError_t launch_fused(const GemmParams& p0, const GemmParams& p1, const FuseParams& f, int grid, hipStream_t st) {
  constexpr int lds = kLdsBytesShallow;   // (its per-M-tile counters take 8 KiB of LDS; every tile height runs with 4 stages)
  auto kern = k_fused_layers<MODE0, PK>;
  hipError_t e = allow_large_lds((const void*)kern, lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, p0, p1, f);
  return hipGetLastError();
}

hipError_t launch_fused_layers(const GemmParams& p0, const GemmParams& p1, const FuseParams& f, int act, int grid, hipStream_t st) {
  if (act == MOE_ACT_SWIGLU)
    return p0.b_packed ? launch_fused<MODE_L0_SWIGLU, true>(p0, p1, f, grid, st) : launch_fused<MODE_L0_SWIGLU, false>(p0, p1, f, grid, st);
  return p0.b_packed ? launch_fused<MODE_L0_GELU, true>(p0, p1, f, grid, st) : launch_fused<MODE_L0_GELU, false>(p0, p1, f, grid, st);
}

template <int MODE, bool PK>
static hipError_t launch_gemm(const GemmParams& p, int grid, hipStream_t st) {
  constexpr int lds = kLdsBytes;
  auto kern = k_group_gemm<MODE, PK>;
  hipError_t e = allow_large_lds((const void*)kern, lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, p);
  return hipGetLastError();
}

hipError_t launch_layer0(const GemmParams& p, int act, int grid, hipStream_t st) {
  if (act == MOE_ACT_SWIGLU) return p.b_packed ? launch_gemm<MODE_L0_SWIGLU, true>(p, grid, st) : launch_gemm<MODE_L0_SWIGLU, false>(p, grid, st);
  return p.b_packed ? launch_gemm<MODE_L0_GELU, true>(p, grid, st) : launch_gemm<MODE_L0_GELU, false>(p, grid, st);
}

hipError_t launch_layer1(const GemmParams& p, int grid, hipStream_t st) {
  return p.b_packed ? launch_gemm<MODE_L1, true>(p, grid, st) : launch_gemm<MODE_L1, false>(p, grid, st);
}

// ---------------------------------------------------------------------------------------------
// Weight packing (once per set of weights, outside the forward): B [E][K][ldb] row-major becomes, per expert, column
// tile and K step of 32, the 16 KiB LDS image of that stage: 16 fragments of 1 KiB, fragment (kk, c) = 16 values of K
// (kk-th half of the step) x 32 columns (c-th block of the tile), lane l of a wavefront owning the 8 K-consecutive
// values k = kk*16 + (l/32)*8 .. +7 of column l%32 -- the operand layout of v_mfma_f32_32x32x16_bf16.  A tile's stages
// follow each other in memory, so a workgroup streams one contiguous run per tile.
// Column blocks: plain layers, block c = columns [32c, 32c+32) of the tile.  SwiGLU W1 ([gate | up] column halves): tile
// n covers hidden units [128n, 128n+128); blocks 0..3 are their gate columns, blocks 4..7 their up columns.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_pack_weights(const uint16_t* __restrict__ B, uint16_t* __restrict__ out, int K, int ldb,
                                                      int n_tiles_n, int swiglu_F, size_t total_chunks) {
  // one 16-byte chunk (8 values of K for one column) per thread step
  const int nk = K / BK;
  for (size_t ch = (size_t)blockIdx.x * 256 + threadIdx.x; ch < total_chunks; ch += (size_t)gridDim.x * 256) {
    const int l = (int)(ch & 63);
    const int frag = (int)((ch >> 6) & 15);
    const size_t stage = ch >> 10;
    const int kt = (int)(stage % nk);
    const size_t en = stage / nk;
    const int n = (int)(en % n_tiles_n);
    const size_t e = en / n_tiles_n;
    const int kk = frag >> 3, c = frag & 7;
    const int k0 = kt * BK + kk * 16 + (l >> 5) * 8;
    int col;
    if (swiglu_F > 0) col = (c >> 2) * swiglu_F + n * (BN / 2) + (c & 3) * 32 + (l & 31);
    else col = n * BN + c * 32 + (l & 31);
    const uint16_t* src = B + (e * K + k0) * (size_t)ldb + col;
    u32x4 v;
#pragma unroll
    for (int i = 0; i < 4; i++) v[i] = (uint32_t)src[(size_t)(2 * i) * ldb] | ((uint32_t)src[(size_t)(2 * i + 1) * ldb] << 16);
    *(u32x4*)(out + ch * 8) = v;
  }
}

hipError_t launch_pack_weights(const void* B, void* out, int E, int K, int ldb, int n_tiles_n, int swiglu_F, hipStream_t st) {
  const size_t total_chunks = (size_t)E * n_tiles_n * (K / BK) * (B_STAGE / 16);
  if (total_chunks == 0) return hipSuccess;
  size_t grid = (total_chunks + 255) / 256;
  if (grid > 256 * 32) grid = 256 * 32;
  hipLaunchKernelGGL(k_pack_weights, dim3((unsigned)grid), dim3(256), 0, st, (const uint16_t*)B, (uint16_t*)out, K, ldb, n_tiles_n,
                     swiglu_F, total_chunks);
  return hipGetLastError();
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
      bf16x2 pr = {(__bf16)acc[2 * c], (__bf16)acc[2 * c + 1]};
      o[c] = __builtin_bit_cast(uint32_t, pr);
    }
    *(u32x4*)(p.out + (size_t)t * p.H + col) = o;
  }
}

__global__ __launch_bounds__(256) void k_zero_u32(uint32_t* __restrict__ ptr, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) ptr[i] = 0u;
}

hipError_t launch_zero_u32(uint32_t* ptr, size_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  size_t grid = (n + 255) / 256;
  if (grid > 1024) grid = 1024;
  hipLaunchKernelGGL(k_zero_u32, dim3((unsigned)grid), dim3(256), 0, st, ptr, n);
  return hipGetLastError();
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

#ifdef MOE_TILE_TRACE
// Measurement build only.  reset != 0: forget the tiles noted so far.  Otherwise copies out, per layer (0, 1) and
// workgroup (256), the number of tiles noted, and per tile (128 slots) the four time stamps, the two cycle counts and the height class
// (0 / 1 / 2 for 64 / 128 / 256 rows, +4 when the tile's first loads were started by its predecessor).  Host pointers.
extern "C" int moe_debug_tile_trace(int reset, uint64_t* stamps, int32_t* kinds, int32_t* counts) {
  if (hipDeviceSynchronize() != hipSuccess) return MOE_ERR_HIP;
  if (reset) {
    static const int32_t zeros[2][moe::kTraceWgs] = {};
    return hipMemcpyToSymbol(HIP_SYMBOL(moe::g_trace_count), zeros, sizeof(zeros)) == hipSuccess ? MOE_OK : MOE_ERR_HIP;
  }
  if (!stamps || !kinds || !counts) return MOE_ERR_INVALID_ARG;
  if (hipMemcpyFromSymbol(stamps, HIP_SYMBOL(moe::g_trace_stamp), sizeof(uint64_t) * 2 * moe::kTraceWgs * moe::kTraceTiles * moe::kTraceWords) != hipSuccess ||
      hipMemcpyFromSymbol(kinds, HIP_SYMBOL(moe::g_trace_kind), sizeof(int32_t) * 2 * moe::kTraceWgs * moe::kTraceTiles) != hipSuccess ||
      hipMemcpyFromSymbol(counts, HIP_SYMBOL(moe::g_trace_count), sizeof(int32_t) * 2 * moe::kTraceWgs) != hipSuccess)
    return MOE_ERR_HIP;
  return MOE_OK;
}
#endif

