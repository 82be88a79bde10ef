// Gate, shared-tensor row order, tile tables and tile schedules (integer work, bit-exact).
//
// Row order (paper Section 3.1.2, Fig. 5): rows of the shared tensor are grouped by expert and, inside an
// expert, sorted by source rank.  Source segment s owns a contiguous token range, so a stable counting sort of
// the pair ids q = t*k + j by expert id gives exactly that order.
#include "moe_internal.h"

namespace moe {

// ---------------------------------------------------------------------------------------------
// Gate (Section 2.1): softmax over E logits, top-k, renormalise.  One wavefront per token.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_route_topk(const float* __restrict__ logits, int T, int E, int k,
                                                    int32_t* __restrict__ ids, float* __restrict__ w) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  // each lane holds up to 4 experts: e = lane + 64*i
  float v[4];
  bool taken[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int e = lane + 64 * i;
    v[i] = e < E ? logits[(size_t)t * E + e] : -INFINITY;
    taken[i] = e >= E;
  }
  float sel_logit = 0.f;  // lane j keeps the logit of slot j
  float top = 0.f;
  for (int j = 0; j < k; j++) {
    // lane-local best among untaken (lowest expert id wins ties: i ascending, strict >)
    float bv = -INFINITY;
    int be = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      if (!taken[i] && (be == 0x7fffffff || v[i] > bv)) { bv = v[i]; be = lane + 64 * i; }
    }
    // wave argmax with ties to the lower expert id
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      float ov = __shfl_xor(bv, off);
      int oe = __shfl_xor(be, off);
      bool better = (oe != 0x7fffffff) && (be == 0x7fffffff || ov > bv || (ov == bv && oe < be));
      if (better) { bv = ov; be = oe; }
    }
#pragma unroll
    for (int i = 0; i < 4; i++) taken[i] = taken[i] || (be == lane + 64 * i);
    if (j == 0) top = bv;
    if (lane == j) sel_logit = bv;
    if (lane == 0) ids[(size_t)t * k + j] = be;
  }
  // weights: softmax restricted to the kept logits (equal to softmax over all E followed by renormalisation)
  float p = lane < k ? expf(sel_logit - top) : 0.f;
  float sum = p;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
  if (lane < k) w[(size_t)t * k + lane] = p / sum;
}

hipError_t launch_route_topk(const float* logits, int T, int E, int k, int32_t* ids, float* w, hipStream_t st) {
  if (T == 0) return hipSuccess;
  hipLaunchKernelGGL(k_route_topk, dim3((T + 3) / 4), dim3(256), 0, st, logits, T, E, k, ids, w);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Index build, step 1: per-workgroup histogram of expert ids.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_index_hist(IndexParams p) {
  __shared__ int32_t hist[kMaxExperts];
  const int E = p.s.E, R = p.s.R;
  for (int e = threadIdx.x; e < E; e += 256) hist[e] = 0;
  __syncthreads();
  const int base = blockIdx.x * kIndexChunk;
#pragma unroll
  for (int i = 0; i < kIndexChunk / 256; i++) {
    int q = base + i * 256 + threadIdx.x;
    if (q < R) atomicAdd(&hist[p.topk_ids[q]], 1);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += 256) p.ws.block_hist[blockIdx.x * E + e] = hist[e];
}

// ---------------------------------------------------------------------------------------------
// Step 2 (one workgroup): expert counts and offsets, per-workgroup bases, the M-tile table, and
// the counters of this forward reset to zero.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_index_scan(IndexParams p) {
  __shared__ int32_t cnt[kMaxExperts];
  __shared__ int32_t off[kMaxExperts + 1];
  __shared__ int32_t tbase[kMaxExperts + 1];
  const int E = p.s.E;
  for (int e = threadIdx.x; e < E; e += 256) {
    int run = 0;
    for (int b = 0; b < p.n_blocks; b++) {
      int c = p.ws.block_hist[b * E + e];
      p.ws.block_hist[b * E + e] = run;   // rows of expert e that come from earlier workgroups
      run += c;
    }
    cnt[e] = run;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int o = 0, tb = 0;
    for (int e = 0; e < E; e++) {
      off[e] = o;
      tbase[e] = tb;
      o += cnt[e];
      tb += (cnt[e] + p.tile_m - 1) / p.tile_m;
    }
    off[E] = o;
    tbase[E] = tb;
    p.ws.status[0] = 0;
    p.ws.status[1] = tb;
    p.ws.status[2] = tb * p.n_tiles_n0;
    p.ws.status[3] = tb * p.n_tiles_n1;
    p.ws.status[4] = 0;
    p.ws.status[5] = 0;
    p.ws.status[6] = 0;
  }
  for (int i = threadIdx.x; i < p.n_tiles_n1; i += 256) p.ws.panel_done[i] = 0;
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += 256) {
    p.ws.counts[e] = cnt[e];
    p.ws.offsets[e] = off[e];
    int nt = tbase[e + 1] - tbase[e];
    for (int i = 0; i < nt; i++) {
      int ti = tbase[e] + i;
      p.ws.tile_expert[ti] = e;
      p.ws.tile_row0[ti] = off[e] + i * p.tile_m;
      int left = cnt[e] - i * p.tile_m;
      p.ws.tile_rows[ti] = left < p.tile_m ? left : p.tile_m;
    }
  }
  if (threadIdx.x == 0) p.ws.offsets[E] = off[E];
}

// ---------------------------------------------------------------------------------------------
// Step 3: stable scatter.  A workgroup owns kIndexChunk consecutive pair ids, cut into runs of 64
// (one per wavefront pass); a pair's position is
//   offsets[e] + rows of e in earlier workgroups + rows of e in earlier runs + rows of e earlier in its run.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_index_scatter(IndexParams p) {
  constexpr int kRuns = kIndexChunk / 64;
  __shared__ int32_t run_cnt[kRuns][kMaxExperts];
  const int E = p.s.E, R = p.s.R, k = p.s.k;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < kRuns * kMaxExperts; i += 256) (&run_cnt[0][0])[i] = 0;
  __syncthreads();
  int key[kRuns / 4], rank[kRuns / 4];
  const int base = blockIdx.x * kIndexChunk;
#pragma unroll
  for (int s = 0; s < kRuns / 4; s++) {
    const int run = wave * (kRuns / 4) + s;
    const int q = base + run * 64 + lane;
    const bool valid = q < R;
    const int e = valid ? p.topk_ids[q] : -1;
    // lanes of this run holding the same expert
    uint64_t same = __ballot(valid);
#pragma unroll
    for (int bit = 0; bit < 8; bit++) {
      const uint64_t b = __ballot((e >> bit) & 1);
      same &= ((e >> bit) & 1) ? b : ~b;
    }
    const uint64_t below = same & ((1ull << lane) - 1ull);
    key[s] = e;
    rank[s] = __popcll(below);
    if (valid && below == 0) run_cnt[run][e] = __popcll(same);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += 256) {
    int acc = 0;
#pragma unroll
    for (int r = 0; r < kRuns; r++) {
      int c = run_cnt[r][e];
      run_cnt[r][e] = acc;
      acc += c;
    }
  }
  __syncthreads();
#pragma unroll
  for (int s = 0; s < kRuns / 4; s++) {
    const int run = wave * (kRuns / 4) + s;
    const int q = base + run * 64 + lane;
    const int e = key[s];
    if (e >= 0) {
      const int pos = p.ws.offsets[e] + p.ws.block_hist[blockIdx.x * E + e] + run_cnt[run][e] + rank[s];
      p.ws.perm[pos] = q;
      p.ws.inv_perm[q] = pos;
      p.ws.row_token[pos] = q / k;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Step 4 (one workgroup): the source segment each M-tile waits for, and the tile schedules.
//
// A tile can start once all its rows have arrived (Section 2.2.1); its rows are in source order, so that is
// the segment of its last row.
//
// Layer0 schedule: order 0 keeps all M-tiles of one expert together while sweeping groups of 8 column
// tiles, so that the workgroups running at the same time share weight panels (consecutive items go to
// consecutive XCDs, which therefore keep to their own column tiles); order 1 lists the tiles by the segment
// they wait for (Fig. 5: local and early-arriving rows first).
// Layer1 schedule: order 1 is column-panel-major over all experts (Fig. 6) in groups of 8 panels, one per XCD;
// order 0 is expert-major like layer0.
// ---------------------------------------------------------------------------------------------
__device__ inline void emit_expert_major(uint32_t* items, const int32_t* tile_expert, int n_tiles, int n_tiles_n,
                                         int tid, int nthreads) {
  // Position of item (m, n): experts in order; inside an expert, groups of 8 column tiles; inside a group,
  // M-tiles of the expert; inside an M-tile the 8 column tiles.  The tile table is expert-major, so the M-tiles
  // of an expert are the consecutive range [m_lo, m_hi).
  for (int m = tid; m < n_tiles; m += nthreads) {
    const int e = tile_expert[m];
    int m_lo = m, m_hi = m + 1;
    while (m_lo > 0 && tile_expert[m_lo - 1] == e) m_lo--;
    while (m_hi < n_tiles && tile_expert[m_hi] == e) m_hi++;
    const int cnt = m_hi - m_lo;
    const int ebase = m_lo * n_tiles_n;
    for (int n = 0; n < n_tiles_n; n++) {
      const int g = n >> 3, gw = min(8, n_tiles_n - g * 8);
      const int pos = ebase + g * 8 * cnt + (m - m_lo) * gw + (n & 7);
      items[pos] = pack_item(m, n);
    }
  }
}

__global__ __launch_bounds__(1024) void k_index_schedule(IndexParams p) {
  __shared__ int32_t seg_first[kMaxSegments + 1];  // first position of each ready-segment bucket
  __shared__ int32_t seg_fill[kMaxSegments];
  const int n_tiles = p.ws.status[1];
  const int tid = threadIdx.x;
  const int S = p.s.S, k = p.s.k;
  if (tid <= kMaxSegments) seg_first[tid] = 0;
  if (tid < kMaxSegments) seg_fill[tid] = 0;
  __syncthreads();
  for (int m = tid; m < n_tiles; m += 1024) {
    const int last = p.ws.tile_row0[m] + p.ws.tile_rows[m] - 1;
    const int t = p.ws.row_token[last];
    int s = 0;
    while (s + 1 < S && p.seg_offsets[s + 1] <= t) s++;
    p.ws.tile_ready[m] = s;
  }
  __syncthreads();
  // layer0
  if (p.layer0_order == 0) {
    emit_expert_major(p.ws.items0, p.ws.tile_expert, n_tiles, p.n_tiles_n0, tid, 1024);
  } else {
    // stable bucket sort of the M-tiles by ready segment (one thread: a few hundred tiles at most per bucket
    // pass), then all column tiles of one M-tile in a row
    if (tid == 0) {
      for (int m = 0; m < n_tiles; m++) seg_first[p.ws.tile_ready[m] + 1]++;
      for (int s = 0; s < S; s++) seg_first[s + 1] += seg_first[s];
    }
    __syncthreads();
    if (tid == 0) {
      for (int m = 0; m < n_tiles; m++) {
        const int s = p.ws.tile_ready[m];
        const int slot = seg_first[s] + seg_fill[s]++;
        p.ws.items1[slot] = m;  // scratch: M-tiles in segment order
      }
    }
    __syncthreads();
    for (int i = tid; i < n_tiles * p.n_tiles_n0; i += 1024) {
      const int slot = i / p.n_tiles_n0, n = i % p.n_tiles_n0;
      p.ws.items0[i] = pack_item(p.ws.items1[slot], n);
    }
    __syncthreads();
  }
  // layer1
  if (p.layer1_order == 0) {
    emit_expert_major(p.ws.items1, p.ws.tile_expert, n_tiles, p.n_tiles_n1, tid, 1024);
  } else {
    const int total = n_tiles * p.n_tiles_n1;
    for (int i = tid; i < total; i += 1024) {
      // groups of 8 panels; inside a group M-tile-major, the 8 panels of one M-tile in a row
      const int per_group = n_tiles * 8;
      const int g = i / per_group, r = i % per_group;
      const int gw = min(8, p.n_tiles_n1 - g * 8);
      const int m = r / gw, n = g * 8 + r % gw;
      p.ws.items1[i] = pack_item(m, n);
    }
  }
}

hipError_t launch_index_build(const IndexParams& p, hipStream_t st) {
  if (p.s.R == 0) return hipSuccess;
  hipLaunchKernelGGL(k_index_hist, dim3(p.n_blocks), dim3(256), 0, st, p);
  hipLaunchKernelGGL(k_index_scan, dim3(1), dim3(256), 0, st, p);
  hipLaunchKernelGGL(k_index_scatter, dim3(p.n_blocks), dim3(256), 0, st, p);
  hipLaunchKernelGGL(k_index_schedule, dim3(1), dim3(1024), 0, st, p);
  return hipGetLastError();
}

}  // namespace moe
