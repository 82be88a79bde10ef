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
    if (q < R) {
      int e = p.topk_ids[q];
      if ((unsigned)e >= (unsigned)E) {   // not an expert: reported through the status word, counted as the last expert
        p.ws.status[5] = p.forward_serial;
        e = E - 1;
      }
      atomicAdd(&hist[e], 1);
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += 256) p.ws.block_hist[blockIdx.x * E + e] = hist[e];
}

// ---------------------------------------------------------------------------------------------
// Tiling of an expert's rows: as many tiles of tile_m rows as fit, then the remainder is cut so that little
// of a tile is padding: with tile_m = 256 a remainder of up to 64 rows becomes one 64-row tile, up to 128 one
// 128-row tile, up to 192 a 128-row and a 64-row tile, more one ragged 256-row tile (tile_m = 128: 64 or 128).
// ---------------------------------------------------------------------------------------------
__device__ inline int tail_tiles(int rem, int tile_m, int* h0, int* h1) {
  // heights (kernel variant) of the tiles that cover a remainder of rem rows; returns their number (0..2)
  if (rem == 0) return 0;
  if (tile_m == 64) { *h0 = 64; return 1; }
  if (rem <= 64) { *h0 = 64; return 1; }
  if (rem <= 128 || tile_m == 128) { *h0 = 128; return 1; }
  if (rem <= 192) { *h0 = 128; *h1 = 64; return 2; }
  *h0 = 256;
  return 1;
}

// Exclusive prefix sum over 256 values in LDS (one per thread of the workgroup); returns the total.
__device__ inline int exclusive_scan_256(int32_t* buf, int v) {
  const int t = threadIdx.x;
  buf[t] = v;
  __syncthreads();
  for (int d = 1; d < 256; d <<= 1) {
    const int add = t >= d ? buf[t - d] : 0;
    __syncthreads();
    buf[t] += add;
    __syncthreads();
  }
  const int incl = buf[t], total = buf[255];
  __syncthreads();
  buf[t] = incl - v;
  __syncthreads();
  return total;
}

// ---------------------------------------------------------------------------------------------
// Step 2: stable scatter.  A workgroup owns kIndexChunk consecutive pair ids, cut into runs of 64
// (one per wavefront pass); a pair's position is
//   offsets[e] + rows of e in earlier workgroups + rows of e in earlier runs + rows of e earlier in its run.
// Every workgroup derives the expert offsets and its own bases from the per-workgroup histograms (a few
// thousand values at most), which saves a kernel between the histogram and the scatter; workgroup 0 also
// writes the counts, the offsets, the M-tile table and the zeroed counters of this forward.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_index_scatter(IndexParams p) {
  constexpr int kRuns = kIndexChunk / 64;
  __shared__ int32_t run_cnt[kRuns][kMaxExperts];
  __shared__ int32_t off[kMaxExperts];     // first row of each expert
  __shared__ int32_t before[kMaxExperts];  // rows of each expert owned by earlier workgroups
  __shared__ int32_t tbase[kMaxExperts];   // first M-tile of each expert (workgroup 0)
  const int E = p.s.E, R = p.s.R, k = p.s.k;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int my_cnt = 0;
  {
    const int e = threadIdx.x;   // E <= 256 = threads
    int mine = 0;
    constexpr int kHistLds = kRuns * kMaxExperts;   // run_cnt doubles as the landing area of the histograms
    const int n_hist = p.n_blocks * E;
    if (n_hist <= kHistLds) {
      // all histograms in one coalesced sweep, then summed out of LDS (a per-thread walk over the workgroups would
      // be a chain of dependent global loads)
      int32_t* hist = &run_cnt[0][0];
      for (int i = threadIdx.x; i < n_hist; i += 256) hist[i] = p.ws.block_hist[i];
      __syncthreads();
      if (e < E) {
        for (int b = 0; b < p.n_blocks; b++) {
          const int c = hist[b * E + e];
          if (b < (int)blockIdx.x) mine += c;
          my_cnt += c;
        }
      }
      __syncthreads();
    } else if (e < E) {
      for (int b = 0; b < p.n_blocks; b++) {
        const int c = p.ws.block_hist[b * E + e];
        if (b < (int)blockIdx.x) mine += c;
        my_cnt += c;
      }
    }
    before[threadIdx.x] = mine;
  }
  for (int i = threadIdx.x; i < kRuns * kMaxExperts; i += 256) (&run_cnt[0][0])[i] = 0;
  const int total_rows = exclusive_scan_256(off, my_cnt);
  if (blockIdx.x == 0) {
    const int e = threadIdx.x;
    int h0 = 0, h1 = 0;
    const int my_tiles = e < E ? my_cnt / p.tile_m + tail_tiles(my_cnt % p.tile_m, p.tile_m, &h0, &h1) : 0;
    const int n_tiles = exclusive_scan_256(tbase, my_tiles);
    if (threadIdx.x == 0) {
      p.ws.status[0] = 0;
      p.ws.status[1] = n_tiles;
      p.ws.status[2] = n_tiles * p.n_tiles_n0;
      p.ws.status[3] = n_tiles * p.n_tiles_n1;
      p.ws.status[4] = 0;
      p.ws.offsets[E] = total_rows;
    }
    if (threadIdx.x < 2 * kXcds) p.ws.status[8 + threadIdx.x] = 0;   // queue heads of both layers
    for (int i = threadIdx.x; i < p.n_tiles_n1; i += 256) p.ws.panel_done[i] = 0;
    for (int i = threadIdx.x; i < p.max_tiles + 1; i += 256) p.ws.tile_done[i] = 0;
    if (e < E) {
      p.ws.counts[e] = my_cnt;
      p.ws.offsets[e] = off[e];
      const int kind_full = p.tile_m == 256 ? 2 : (p.tile_m == 128 ? 1 : 0);
      const int nfull = my_cnt / p.tile_m;
      int ti = tbase[e], row = off[e];
      for (int i = 0; i < nfull; i++, ti++, row += p.tile_m) {
        p.ws.tile_expert[ti] = e;
        p.ws.tile_row0[ti] = row;
        p.ws.tile_rows[ti] = p.tile_m;
        p.ws.tile_kind[ti] = kind_full;
      }
      const int h[2] = {h0, h1};
      const int nt = my_tiles - nfull;
      int left = my_cnt % p.tile_m;
      for (int i = 0; i < nt; i++, ti++) {
        const int rows = left < h[i] ? left : h[i];
        p.ws.tile_expert[ti] = e;
        p.ws.tile_row0[ti] = row;
        p.ws.tile_rows[ti] = rows;
        p.ws.tile_kind[ti] = h[i] == 256 ? 2 : (h[i] == 128 ? 1 : 0);
        row += rows;
        left -= rows;
      }
    }
  }
  __syncthreads();
  int key[kRuns / 4], rank[kRuns / 4];
  const int base = blockIdx.x * kIndexChunk;
#pragma unroll
  for (int s = 0; s < kRuns / 4; s++) {
    const int run = wave * (kRuns / 4) + s;
    const int q = base + run * 64 + lane;
    const bool valid = q < R;
    int e = valid ? p.topk_ids[q] : -1;
    if (valid && (unsigned)e >= (unsigned)E) e = E - 1;   // as in the histogram
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
      const int pos = off[e] + before[e] + run_cnt[run][e] + rank[s];
      p.ws.perm[pos] = q;
      p.ws.inv_perm[q] = pos;
      p.ws.row_token[pos] = q / k;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Step 3: the source segment each M-tile waits for, and the tile schedules.
//
// A tile can start once all its rows have arrived (Section 2.2.1); its rows are in source order, so that is
// the segment of its last row.
//
// A schedule is a list of (M-tile, column tile) items.  Position i of the list belongs to XCD i % 8 (a
// workgroup takes the next position of its own XCD's share and, when that is used up, of the others'), so
// consecutive positions should differ in the column tile and keep the M-tile: the workgroups of one XCD then
// work on few column tiles of many M-tiles and share weight panels in their L2.  Tall tiles come first and the
// short tiles of the ragged ends last, so that the short ones fill the gaps at the end of the kernel.
// The orders (k_index_schedule, for up to 2048 M-tiles; see there for the locality order):
// Layer0, order 0: locality order (blocks of an expert's M-tiles per XCD, column tiles ascending inside a block).
// Order 1: per tile height, M-tiles by the segment they wait for (Fig. 5: rows that are local or arrive early first),
// all column tiles of an M-tile in a row.  Order 2: the locality order inside waves of source segments, the waves in
// arrival order.  Layer1: the locality order, or (in-kernel panel reduction) per tile height the M-tiles are dealt to
// the XCDs in contiguous chunks and every XCD sweeps its chunk column-panel-major, 4 panels at a time (Fig. 6).
// The one-workgroup builder below (any number of M-tiles) knows simpler versions of orders 0 and 1.
// ---------------------------------------------------------------------------------------------
constexpr int kTileCap = kScheduleTileCap;  // tiles whose table fits the LDS copies of the schedule builder

__device__ inline ItemRec make_item(const Workspace& ws, int m, int n) {
  ItemRec r;
  r.m_tile = m;
  r.n_tile = n;
  r.expert = ws.tile_expert[m];
  r.row0 = ws.tile_row0[m];
  r.nrows = ws.tile_rows[m];
  r.kind = ws.tile_kind[m];
  r.ready_seg = ws.tile_ready[m];
  r.pad = 0;
  return r;
}

// Layer0 items of the tiles order[lo..hi) (one height, expert-major), written from position base on.
// ord / exp_of: LDS copies (or the global arrays when the table is too large).
template <typename OrdT, typename ExpT>
__device__ inline void emit_expert_major(const Workspace& ws, ItemRec* items, const OrdT* ord, const ExpT* exp_of, int lo,
                                         int hi, int base, int n_tiles_n, int tid, int nthreads) {
  // one (tile, group of 8 column tiles) pair per thread step
  const int n_groups = (n_tiles_n + 7) >> 3;
  for (int w = tid; w < (hi - lo) * n_groups; w += nthreads) {
    const int i = lo + w / n_groups, g = w % n_groups;
    const int e = exp_of[ord[i]];
    int a = i, b = i + 1;
    while (a > lo && exp_of[ord[a - 1]] == e) a--;
    while (b < hi && exp_of[ord[b]] == e) b++;
    const int cnt = b - a;
    const int gw = min(8, n_tiles_n - g * 8);
    const int pos = base + (a - lo) * n_tiles_n + g * 8 * cnt + (i - a) * gw;
    ItemRec r = make_item(ws, ord[i], 0);
    for (int n = 0; n < gw; n++) {
      r.n_tile = g * 8 + n;
      items[pos + n] = r;
    }
  }
}

// Layer1 items of the tiles order[lo..hi): the tiles are dealt to the XCDs in contiguous chunks (an XCD then
// keeps to few experts); XCD x's queue continues, from position queue_pos[x] on, with its chunk swept per group of
// 4 column panels: the chunk's tiles, each with the 4 panels.  Panel groups ascend, so all M-tiles of the chunk
// finish panel group g before g + 1 (Fig. 6).
template <typename OrdT>
__device__ inline void emit_chunked(const Workspace& ws, ItemRec* items, const OrdT* ord, int lo, int hi,
                                    const int32_t* queue_pos, int n_tiles_n, int tid, int nthreads) {
  const int nt = hi - lo;
  if (nt == 0) return;
  const int chunk = (nt + kXcds - 1) / kXcds;
  const int n_groups = (n_tiles_n + 3) >> 2;
  for (int w = tid; w < nt * n_groups; w += nthreads) {
    const int i = w / n_groups, g = w % n_groups;
    const int x = i / chunk, j = i % chunk;
    const int cnt = min(chunk, nt - x * chunk);
    const int gw = min(4, n_tiles_n - g * 4);
    const int pos = queue_pos[x] + g * 4 * cnt + j * gw;
    ItemRec r = make_item(ws, ord[lo + i], 0);
    for (int n = 0; n < gw; n++) {
      r.n_tile = g * 4 + n;
      items[pos + n] = r;
    }
  }
}

__global__ __launch_bounds__(1024) void k_index_schedule_large(IndexParams p) {
  __shared__ int32_t cls_first[4];  // first position in order[] of the tiles of kind 2, 1, 0, and the end
  __shared__ int32_t key_pos[3 * kMaxSegments];
  __shared__ uint8_t keys[kTileCap];
  __shared__ uint8_t exp_lds[kTileCap];
  __shared__ uint16_t ord_lds[kTileCap];
  const int n_tiles = p.ws.status[1];
  const int tid = threadIdx.x;
  const int S = p.s.S;
  const bool in_lds = n_tiles <= kTileCap;
  const int nseg = p.layer0_order == 1 ? S : 1;
  const int nkeys = 3 * nseg;
  // the source segment each tile waits for; sort key = (height class, segment) or the height class alone
  for (int m = tid; m < n_tiles; m += 1024) {
    const int last = p.ws.tile_row0[m] + p.ws.tile_rows[m] - 1;
    const int t = p.ws.row_token[last];
    int s = 0;
    while (s + 1 < S && p.seg_offsets[s + 1] <= t) s++;
    p.ws.tile_ready[m] = s;
    if (in_lds) {
      keys[m] = (uint8_t)((2 - p.ws.tile_kind[m]) * nseg + (nseg > 1 ? s : 0));
      exp_lds[m] = (uint8_t)p.ws.tile_expert[m];
    }
  }
  __syncthreads();
  auto key_of = [&](int m) {
    return in_lds ? (int)keys[m] : (2 - p.ws.tile_kind[m]) * nseg + (nseg > 1 ? p.ws.tile_ready[m] : 0);
  };
  // stable counting sort: one thread per key value walks the keys twice, first counting, then placing
  if (tid < nkeys) {
    int c = 0;
    for (int m = 0; m < n_tiles; m++) c += (key_of(m) == tid);
    key_pos[tid] = c;
  }
  __syncthreads();
  if (tid == 0) {
    int pos = 0;
    for (int i = 0; i < nkeys; i++) {
      if (i % nseg == 0) cls_first[i / nseg] = pos;
      const int c = key_pos[i];
      key_pos[i] = pos;
      pos += c;
    }
    cls_first[3] = pos;
  }
  __syncthreads();
  if (tid < nkeys) {
    int pos = key_pos[tid];
    for (int m = 0; m < n_tiles; m++)
      if (key_of(m) == tid) {
        if (in_lds) ord_lds[pos] = (uint16_t)m; else p.ws.tile_order[pos] = m;
        pos++;
      }
  }
  __syncthreads();
  for (int c = 0; c < 3; c++) {
    const int lo = cls_first[c], hi = cls_first[c + 1];
    if (p.layer0_order == 0) {
      if (in_lds) emit_expert_major(p.ws, p.ws.items0, ord_lds, exp_lds, lo, hi, lo * p.n_tiles_n0, p.n_tiles_n0, tid, 1024);
      else emit_expert_major(p.ws, p.ws.items0, p.ws.tile_order, p.ws.tile_expert, lo, hi, lo * p.n_tiles_n0, p.n_tiles_n0, tid, 1024);
    } else {
      for (int i = tid; i < (hi - lo) * p.n_tiles_n0; i += 1024) {
        const int m = in_lds ? (int)ord_lds[lo + i / p.n_tiles_n0] : p.ws.tile_order[lo + i / p.n_tiles_n0];
        p.ws.items0[lo * p.n_tiles_n0 + i] = make_item(p.ws, m, i % p.n_tiles_n0);
      }
    }
  }
  if (p.layer0_order == 1) {
    // layer1 wants table order inside a height: rebuild order[] (the layer0 list is complete by now)
    __syncthreads();
    if (tid < 3) {
      int pos = cls_first[tid];
      for (int m = 0; m < n_tiles; m++)
        if (key_of(m) / nseg == tid) {
          if (in_lds) ord_lds[pos] = (uint16_t)m; else p.ws.tile_order[pos] = m;
          pos++;
        }
    }
    __syncthreads();
  }
  // layer1: one contiguous queue per XCD; queue x holds its chunk of every height class, tallest first
  __shared__ int32_t queue_pos[kXcds];
  const int cap = (n_tiles + 3 * kXcds) / kXcds * p.n_tiles_n1;   // room per queue
  if (tid < kXcds) queue_pos[tid] = tid * cap;
  __syncthreads();
  for (int c = 0; c < 3; c++) {
    const int lo = cls_first[c], hi = cls_first[c + 1];
    if (in_lds) emit_chunked(p.ws, p.ws.items1, ord_lds, lo, hi, queue_pos, p.n_tiles_n1, tid, 1024);
    else emit_chunked(p.ws, p.ws.items1, p.ws.tile_order, lo, hi, queue_pos, p.n_tiles_n1, tid, 1024);
    __syncthreads();
    if (tid < kXcds) {
      const int nt = hi - lo, chunk = (nt + kXcds - 1) / kXcds;
      const int cnt = nt == 0 ? 0 : max(0, min(chunk, nt - tid * chunk));
      queue_pos[tid] += cnt * p.n_tiles_n1;
    }
    __syncthreads();
  }
  if (tid < kXcds) {
    const int n0 = n_tiles * p.n_tiles_n0;
    p.ws.status[24 + tid] = tid < n0 ? (n0 - tid + kXcds - 1) / kXcds : 0;   // layer0: positions tid, tid + 8, ...
    p.ws.status[32 + tid] = queue_pos[tid] - tid * cap;
    p.ws.status[40 + tid] = tid * cap;
  }
}

// The schedule builder for tables of up to kTileCap tiles (anything but very large batches): a few workgroups, each
// of which copies the tile table into LDS, sorts it there (every tile finds its own rank, all in parallel) and
// then writes its share of the item records.  k_index_schedule_large above is the one-workgroup version without
// the size limit (and with simpler orders).
//
// Locality order (layer0 with order 0, layer1 with the separate combine kernel): per tile height, an expert's
// M-tiles are cut into blocks of up to block_m (4 by default); the blocks are dealt to the XCDs, whose queues hold
// their blocks one after the other, tallest first.  Inside a block of G M-tiles the column tiles ascend and the block's M-tiles are the inner
// loop.  The 32 workgroups of an XCD, taking consecutive items, then work on G M-tiles x about 32/G column tiles of
// one expert wherever in the block they are, and share both operands in their L2; an expert with few rows is
// streamed through one XCD only (its weight panels are fetched once).
constexpr int kScheduleWgs = 8;

struct ScheduleLds {
  int32_t row0[kTileCap];
  int32_t blk_off[kTileCap];   // M-tiles ahead of block b in its XCD's queue
  uint16_t rows[kTileCap];
  uint16_t ord0[kTileCap];     // layer0 order: position -> tile
  uint16_t ord1[kTileCap];     // layer1 order (height class, then table order)
  uint16_t blk_g[kTileCap];    // M-tiles of block b
  uint16_t blk_ord[kTileCap];  // blocks in dealing order: height class, then larger blocks first
  uint8_t blk_q[kTileCap];     // XCD queue of block b
  uint8_t blk_key[kTileCap + 4];
  uint8_t expert[kTileCap];
  uint8_t kind[kTileCap];
  uint8_t ready[kTileCap];
  uint8_t key0[kTileCap + 4];   // (height class, segment) or the height class alone; padded with 0xff
  uint8_t key1[kTileCap + 4];   // height class
  uint16_t sub_first[kTileCap];       // position in ord1 of the first tile of tile i's run (same height, expert, wave)
  uint16_t blk_of[kTileCap];          // block of the tile at position i of ord1
  int32_t scan_buf[1024];             // scratch of the prefix scans
  int32_t cls_first[4];
  int32_t cls_count[3];
  int32_t queue_pos[3][kXcds];
  int32_t q_len_t[kXcds], q_base_t[kXcds];   // locality order: M-tiles per XCD queue, and ahead of it
  int32_t n_blocks;
};

__device__ inline ItemRec make_item_lds(const ScheduleLds& L, int m, int n) {
  ItemRec r;
  r.m_tile = m;
  r.n_tile = n;
  r.expert = L.expert[m];
  r.row0 = L.row0[m];
  r.nrows = L.rows[m];
  r.kind = L.kind[m];
  r.ready_seg = L.ready[m];
  r.pad = 0;
  return r;
}

// ord[rank of tile m] = m for the stable order by key (keys < 0xff; the padding never counts).
__device__ inline void rank_sort(const uint8_t* key, uint16_t* ord, int n, int tid) {
  const uint32_t* words = (const uint32_t*)key;
  const int nw = (n + 3) >> 2;
  for (int m = tid; m < n; m += 1024) {
    const int km = key[m];
    int rank = 0;
    for (int j4 = 0; j4 < nw; j4++) {
      const uint32_t w = words[j4];
#pragma unroll
      for (int b = 0; b < 4; b++) {
        const int kj = (w >> (8 * b)) & 0xff, j = j4 * 4 + b;
        rank += (kj < km || (kj == km && j < m)) ? 1 : 0;
      }
    }
    ord[rank] = (uint16_t)m;
  }
}

// Inclusive prefix scan over up to 2048 values, two per thread (thread t holds elements 2t and 2t+1), running maximum
// (MAX) or running sum.  buf: LDS scratch of 1024 values.
template <bool MAX>
__device__ inline void scan_pairs(int32_t* buf, int& v0, int& v1) {
  const int t = threadIdx.x;
  constexpr int kNeutral = MAX ? -0x7fffffff : 0;
  v1 = MAX ? max(v0, v1) : v0 + v1;
  buf[t] = v1;
  __syncthreads();
  for (int d = 1; d < 1024; d <<= 1) {
    const int o = t >= d ? buf[t - d] : kNeutral;
    __syncthreads();
    buf[t] = MAX ? max(buf[t], o) : buf[t] + o;
    __syncthreads();
  }
  const int before = t > 0 ? buf[t - 1] : kNeutral;
  __syncthreads();
  v0 = MAX ? max(before, v0) : before + v0;
  v1 = MAX ? max(before, v1) : before + v1;
}

// Items of one layer in the locality order (see above); n_tiles_n column tiles.
__device__ inline void emit_blocks(const ScheduleLds& L, const uint16_t* ord, ItemRec* items, int n_tiles, int n_tiles_n,
                                   int block_m, int gtid, int gthreads) {
  for (int w = gtid; w < n_tiles * n_tiles_n; w += gthreads) {
    const int i = w / n_tiles_n, n = w % n_tiles_n;
    const int b = L.blk_of[i], g = L.blk_g[b], jm = (i - L.sub_first[i]) % block_m;
    const int pos = (L.q_base_t[L.blk_q[b]] + L.blk_off[b]) * n_tiles_n + n * g + jm;
    items[pos] = make_item_lds(L, ord[i], n);
  }
}

// Blocks of the locality order and their XCD queues.  The tiles (in ord1's order: height class, expert, source order)
// fall into runs of the same height class, expert and wave -- a wave being a group of consecutive source segments,
// n_waves of them over the S segments (1: no waves) -- and every run is cut into blocks of up to block_m M-tiles.
// The blocks are sorted by (wave, height class, larger first) and dealt to the XCD queues back and forth (0..7,
// 7..0, ...): with the sizes descending this keeps the queues level even when the experts' loads differ a lot, which
// round-robin does not (what is left uneven, the workgroups even out by taking from other XCDs' queues at the end).
// With waves the queues are segment-major across waves (tiles whose rows arrive early come first, Fig. 5) and
// weight-panel-major inside a wave (a block's M-tiles share every weight panel they sweep).
__device__ inline void build_blocks(ScheduleLds& L, const uint16_t* ord1, int n_tiles, int block_m, int n_waves, int S) {
  const int tid = threadIdx.x;
  auto run_key = [&](int i) {
    const int m = ord1[i];
    const int wave = n_waves > 1 ? (int)L.ready[m] * n_waves / S : 0;
    return ((2 - (int)L.kind[m]) << 16) | ((int)L.expert[m] << 8) | wave;
  };
  if (tid < kXcds) L.q_len_t[tid] = 0;
  const int i0 = 2 * tid, i1 = 2 * tid + 1;
  int f0 = -1, f1 = -1;
  if (i0 < n_tiles && (i0 == 0 || run_key(i0) != run_key(i0 - 1))) f0 = i0;
  if (i1 < n_tiles && run_key(i1) != run_key(i1 - 1)) f1 = i1;
  scan_pairs<true>(L.scan_buf, f0, f1);
  int s0 = 0, s1 = 0;
  if (i0 < n_tiles) { L.sub_first[i0] = (uint16_t)f0; s0 = (i0 - f0) % block_m == 0; }
  if (i1 < n_tiles) { L.sub_first[i1] = (uint16_t)f1; s1 = (i1 - f1) % block_m == 0; }
  const int start0 = s0, start1 = s1;
  scan_pairs<false>(L.scan_buf, s0, s1);
  if (i0 < n_tiles) L.blk_of[i0] = (uint16_t)(s0 - 1);
  if (i1 < n_tiles) L.blk_of[i1] = (uint16_t)(s1 - 1);
  if (i0 == n_tiles - 1) L.n_blocks = s0;
  if (i1 == n_tiles - 1) L.n_blocks = s1;
  __syncthreads();
  auto describe = [&](int i, int b) {   // tile i starts block b
    int g = 1;
    while (g < block_m && i + g < n_tiles && L.sub_first[i + g] == L.sub_first[i]) g++;
    const int key = run_key(i);
    L.blk_g[b] = (uint16_t)g;
    L.blk_key[b] = (uint8_t)((key & 0xff) * 24 + (key >> 16) * 8 + (8 - g));   // wave, height class, larger blocks first
  };
  if (i0 < n_tiles && start0) describe(i0, s0 - 1);
  if (i1 < n_tiles && start1) describe(i1, s1 - 1);
  const int n_blocks = L.n_blocks;
  for (int b = n_blocks + tid; b < n_blocks + 4; b += 1024) L.blk_key[b] = 0xff;
  __syncthreads();
  rank_sort(L.blk_key, L.blk_ord, n_blocks, tid);
  __syncthreads();
  for (int pos = tid; pos < n_blocks; pos += 1024) {
    const int r = pos / kXcds, i = pos % kXcds;
    const int x = (r & 1) ? kXcds - 1 - i : i;
    int off = 0;
    for (int r2 = 0; r2 < r; r2++) off += L.blk_g[L.blk_ord[r2 * kXcds + ((r2 & 1) ? kXcds - 1 - x : x)]];
    const int b = L.blk_ord[pos];
    L.blk_off[b] = off;
    L.blk_q[b] = (uint8_t)x;
    // the queue's last block: no later round has a block for this queue
    const int next = (r + 1) * kXcds + (((r + 1) & 1) ? kXcds - 1 - x : x);
    if (next >= n_blocks) L.q_len_t[x] = off + L.blk_g[b];
  }
  __syncthreads();
  if (tid == 0) {
    int pos = 0;
    for (int x = 0; x < kXcds; x++) {
      L.q_base_t[x] = pos;
      pos += L.q_len_t[x];
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(1024) void k_index_schedule(IndexParams p) {
  __shared__ __attribute__((aligned(16))) ScheduleLds L;
  const int n_tiles = p.ws.status[1];
  const int tid = threadIdx.x;
  const int S = p.s.S;
  const int nseg = p.layer0_order == 1 ? S : 1;
  // layer0: 0 expert-major (locality order), 1 by source segment, 2 locality order inside waves of source segments
  const bool local0 = p.layer0_order != 1, local1 = p.layer1_order == 0;
  const int n_waves0 = p.layer0_order == 2 ? max(1, min(p.layer0_waves, min(S, 8))) : 1;
  const int block_m = p.block_m;   // M-tiles per block of the locality order (1..8)
  __shared__ int32_t seg_lds[kMaxSegments + 1];
  if (tid <= S) seg_lds[tid] = p.seg_offsets[tid];
  if (tid < 3) L.cls_count[tid] = 0;
  __syncthreads();
  for (int m = tid; m < n_tiles + 4; m += 1024) {
    if (m >= n_tiles) {
      L.key0[m] = 0xff;
      L.key1[m] = 0xff;
      continue;
    }
    const int r0 = p.ws.tile_row0[m], nr = p.ws.tile_rows[m], kd = p.ws.tile_kind[m];
    const int t = p.ws.row_token[r0 + nr - 1];
    int s = 0;
    while (s + 1 < S && seg_lds[s + 1] <= t) s++;
    L.row0[m] = r0;
    L.rows[m] = (uint16_t)nr;
    L.kind[m] = (uint8_t)kd;
    L.expert[m] = (uint8_t)p.ws.tile_expert[m];
    L.ready[m] = (uint8_t)s;
    L.key0[m] = (uint8_t)((2 - kd) * nseg + (nseg > 1 ? s : 0));
    L.key1[m] = (uint8_t)(2 - kd);
    atomicAdd(&L.cls_count[2 - kd], 1);
    if (blockIdx.x == 0) p.ws.tile_ready[m] = s;
  }
  __syncthreads();
  rank_sort(L.key0, L.ord0, n_tiles, tid);
  if (nseg > 1) rank_sort(L.key1, L.ord1, n_tiles, tid);
  if (tid == 0) {
    int pos = 0;
    for (int c = 0; c < 3; c++) {
      L.cls_first[c] = pos;
      pos += L.cls_count[c];
    }
    L.cls_first[3] = pos;
  }
  // layer1 in panel-major order (in-kernel combine): XCD x gets a contiguous chunk of every height class
  const int cap = (n_tiles + 3 * kXcds) / kXcds * p.n_tiles_n1;   // room per queue
  if (tid < kXcds) {
    int pos = tid * cap;
    for (int c = 0; c < 3; c++) {
      L.queue_pos[c][tid] = pos;
      const int nt = L.cls_count[c], chunk = (nt + kXcds - 1) / kXcds;
      const int cnt = nt == 0 ? 0 : max(0, min(chunk, nt - tid * chunk));
      pos += cnt * p.n_tiles_n1;
    }
    if (blockIdx.x == 0 && !local1) {
      p.ws.status[32 + tid] = pos - tid * cap;
      p.ws.status[40 + tid] = tid * cap;
    }
    if (blockIdx.x == 0 && !local0) {
      const int n0 = n_tiles * p.n_tiles_n0;
      p.ws.status[24 + tid] = tid < n0 ? (n0 - tid + kXcds - 1) / kXcds : 0;   // positions tid, tid + 8, ...
    }
  }
  __syncthreads();
  const uint16_t* ord1 = nseg > 1 ? L.ord1 : L.ord0;   // height class, then table order (expert-major)
  const int gtid = blockIdx.x * 1024 + tid, gthreads = gridDim.x * 1024;
  if (local0) {
    build_blocks(L, ord1, n_tiles, block_m, n_waves0, S);
    if (blockIdx.x == 0 && tid < kXcds) {
      p.ws.status[24 + tid] = L.q_len_t[tid] * p.n_tiles_n0;
      p.ws.status[48 + tid] = L.q_base_t[tid] * p.n_tiles_n0;
    }
    emit_blocks(L, ord1, p.ws.items0, n_tiles, p.n_tiles_n0, block_m, gtid, gthreads);
  } else {
    // by source segment (Fig. 5): all column tiles of an M-tile in a row; list position i belongs to XCD i % 8
    for (int i = gtid; i < n_tiles * p.n_tiles_n0; i += gthreads)
      p.ws.items0[i] = make_item_lds(L, L.ord0[i / p.n_tiles_n0], i % p.n_tiles_n0);
  }
  if (local1) {
    if (!local0 || n_waves0 > 1) {
      __syncthreads();   // the layer0 items are out: the block tables can be rebuilt without waves
      build_blocks(L, ord1, n_tiles, block_m, 1, S);
    }
    if (blockIdx.x == 0 && tid < kXcds) {
      p.ws.status[32 + tid] = L.q_len_t[tid] * p.n_tiles_n1;
      p.ws.status[40 + tid] = L.q_base_t[tid] * p.n_tiles_n1;
    }
  }
  if (local1) {
    emit_blocks(L, ord1, p.ws.items1, n_tiles, p.n_tiles_n1, block_m, gtid, gthreads);
  } else {
    // panel-major (Fig. 6): every XCD sweeps its chunk of a height class per group of 4 column panels: the chunk's
    // tiles, each with the 4 panels; panel groups ascend, so all M-tiles of the chunk finish group g before g + 1
    const int n_groups1 = (p.n_tiles_n1 + 3) >> 2;
    for (int w = gtid; w < n_tiles * n_groups1; w += gthreads) {
      const int ig = w / n_groups1, g = w % n_groups1;
      const int m = ord1[ig], c = 2 - L.kind[m];
      const int i = ig - L.cls_first[c], nt = L.cls_count[c];
      const int chunk = (nt + kXcds - 1) / kXcds;
      const int x = i / chunk, j = i % chunk;
      const int cnt = min(chunk, nt - x * chunk);
      const int gw = min(4, p.n_tiles_n1 - g * 4);
      const int pos = L.queue_pos[c][x] + g * 4 * cnt + j * gw;
      ItemRec r = make_item_lds(L, m, 0);
      for (int n = 0; n < gw; n++) {
        r.n_tile = g * 4 + n;
        p.ws.items1[pos + n] = r;
      }
    }
  }
}

__global__ void k_tile_heights(const int32_t* __restrict__ kind, int32_t* __restrict__ height, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) height[i] = 64 << kind[i];
}

hipError_t launch_tile_heights(const int32_t* kind, int32_t* height, int n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_tile_heights, dim3((n + 255) / 256), dim3(256), 0, st, kind, height, n);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Stand-in for the peers of Section 3.1.2 on one GPU: a few workgroups play all sources in turn, copying each source's
// segment of token rows from a staging buffer into the receive buffer at a paced rate and then raising the
// segment's ready flag (data first, system-scope release, then the flag), the way a peer's one-sided stores would.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_arrival_producer(const uint4* __restrict__ staging, uint4* __restrict__ x,
                                                           ArrivalParams a) {
  const long long t_start = wall_clock64();   // 100 MHz
  long long sent = 0;                          // bytes (of all workgroups together) before the current chunk
  const int nwg = gridDim.x, wg = blockIdx.x;
  for (int s = 0; s < a.S; s++) {
    const size_t lo = (size_t)a.seg_offsets[s] * a.row_bytes / 16, hi = (size_t)a.seg_offsets[s + 1] * a.row_bytes / 16;
    for (size_t c = lo; c < hi; c += a.chunk16) {
      const size_t end = c + a.chunk16 < hi ? c + a.chunk16 : hi;
      // pace: this chunk may start once the bytes before it have had their time at the requested rate
      if (a.bytes_per_us > 0) {
        const long long due = t_start + (long long)((double)sent / a.bytes_per_us * 100.0);
        while (wall_clock64() < due) __builtin_amdgcn_s_sleep(16);
      }
      for (size_t i = c + (size_t)wg * 1024 + threadIdx.x; i < end; i += (size_t)nwg * 1024) x[i] = staging[i];
      sent += (long long)(end - c) * 16;
    }
    // the segment is there once every workgroup has written its share: the last one to arrive raises the flag
    __threadfence_system();
    __syncthreads();
    if (threadIdx.x == 0) {
      const uint32_t arrived = __hip_atomic_fetch_add(&a.seg_arrived[s], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
      if (arrived + 1 == (uint32_t)nwg) {
        __hip_atomic_store(&a.seg_arrived[s], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
        __hip_atomic_store(&a.seg_ready[s], a.epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
  }
}

hipError_t launch_arrival_producer(const void* staging, void* x, const ArrivalParams& a, int n_wg, hipStream_t st) {
  hipLaunchKernelGGL(k_arrival_producer, dim3(n_wg), dim3(1024), 0, st, (const uint4*)staging, (uint4*)x, a);
  return hipGetLastError();
}

// Queue heads, combine counter, panel counters and the status word back to zero: what the scatter kernel does at the
// start of a forward, for a forward that runs the schedules of an earlier index build again.
__global__ void k_reset_counters(Workspace ws, int n_tiles_n1, int max_tiles) {
  const int t = threadIdx.x;
  for (int i = t; i < max_tiles + 1; i += 256) ws.tile_done[i] = 0;
  if (t == 0) {
    ws.status[0] = 0;
    ws.status[4] = 0;
  }
  if (t < 2 * kXcds) ws.status[8 + t] = 0;
  for (int i = t; i < n_tiles_n1; i += 256) ws.panel_done[i] = 0;
}

hipError_t launch_reset_counters(const Workspace& ws, int n_tiles_n1, int max_tiles, hipStream_t st) {
  hipLaunchKernelGGL(k_reset_counters, dim3(1), dim3(256), 0, st, ws, n_tiles_n1, max_tiles);
  return hipGetLastError();
}

hipError_t launch_index_build(const IndexParams& p, hipStream_t st) {
  if (p.s.R == 0) return hipSuccess;
  hipLaunchKernelGGL(k_index_hist, dim3(p.n_blocks), dim3(256), 0, st, p);
  hipLaunchKernelGGL(k_index_scatter, dim3(p.n_blocks), dim3(256), 0, st, p);
  if (!uses_large_schedule(p.max_tiles, p.force_large_schedule))
    hipLaunchKernelGGL(k_index_schedule, dim3(kScheduleWgs), dim3(1024), 0, st, p);
  else
    hipLaunchKernelGGL(k_index_schedule_large, dim3(1), dim3(1024), 0, st, p);
  return hipGetLastError();
}

}  // namespace moe
