// Host side of libmoe_gfx950: plan object, workspace layout, and the extern "C" entry points.
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "moe_internal.h"

using namespace moe;

constexpr int kProfSlots = 256;

// Workspace of moe_layer_forward_static: device memory that exists from the moment the library is loaded, so that a
// forward on it allocates nothing.  Every GPU the library runs on holds its own copy at its own address; in host code
// the array's name is only a handle for hipGetSymbolAddress, never a pointer to pass on.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

struct moe_plan {
  Shape s;
  int32_t seg_offsets[kMaxSegments + 1];
  // options
  int32_t tile_m;
  int32_t n_dm;          // -1: table lookup
  int32_t deep_short_tiles;   // 1: 64-row tiles run with six operand stages instead of four
  int32_t n_prefetch;    // -1: table lookup; workgroups of each GroupGEMM launch that prefetch packed weight panels
  int32_t prefetch_ahead, prefetch_behind;   // items around the head of an XCD's queue they work on
  int32_t layer0_order;          // -1: chosen per forward (resident input: 0; ready flags in use: 2)
  int32_t layer0_waves;          // 0: from the table below
  int32_t expected_ingest_gbps;  // 0: unknown
  int32_t last_layer0_order;     // what the last forward ran with (for moe_get_schedule)
  int32_t layer1_order;
  int32_t spin_limit;
  int32_t phases;
  int32_t n_cu;          // 0: not queried yet
  int32_t profile;       // 1: record events around the phases of every forward
  int32_t prof_steps;    // forwards recorded since the last reset (at most kProfSlots)
  int32_t prof_dropped;  // forwards since the last reset that found every slot taken and were not recorded
  hipEvent_t ev[kProfSlots][5];
  bool ev_created;
  // derived
  int32_t n_index_blocks;
  int32_t max_tiles;
  int32_t large_schedule;  // 1: always the one-workgroup schedule builder
  int32_t block_m;         // M-tiles per block of the locality order
  int32_t fuse_layers;     // 1: both GroupGEMMs in one launch, layer1 tiles waiting on per-M-tile counters
  int32_t publish_every;   // one-launch variant: layer0 tiles between two publications of a workgroup
  int32_t handoff_fences;  // measurement aid: per-tile release / acquire fences in the GroupGEMMs
  int32_t alias_experts;   // measurement aid: every expert reads expert 0's weights (plain layout only)
  int32_t weights_packed;  // 1: W1 / W2 of a forward are in the layout moe_pack_weights writes
  int32_t serial;          // number of the last forward (tags the out-of-range report in the status words)
  int32_t n_tiles_n0, n_tiles_n1;
  size_t off_status, off_counts, off_offsets, off_perm, off_inv_perm, off_row_token, off_block_hist, off_tile_expert,
      off_tile_row0, off_tile_rows, off_tile_ready, off_tile_kind, off_tile_order, off_items0, off_items1, off_panel_done, off_tile_done, off_arrive, off_h, off_Y, total_bytes;
};

namespace {

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

void layout(moe_plan* p) {
  const Shape& s = p->s;
  p->n_index_blocks = (s.R + kIndexChunk - 1) / kIndexChunk;
  if (p->n_index_blocks < 1) p->n_index_blocks = 1;
  p->max_tiles = s.R / p->tile_m + 2 * s.E;
  p->n_tiles_n0 = s.act == MOE_ACT_SWIGLU ? s.F / (kTileN / 2) : s.F / kTileN;
  p->n_tiles_n1 = s.H / kTileN;
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o = align_up(o + bytes, 256);
    return at;
  };
  p->off_status = take(64 * 4);
  p->off_counts = take((size_t)s.E * 4);
  p->off_offsets = take((size_t)(s.E + 1) * 4);
  p->off_perm = take((size_t)s.R * 4);
  p->off_inv_perm = take((size_t)s.R * 4);
  p->off_row_token = take((size_t)s.R * 4);
  p->off_block_hist = take((size_t)p->n_index_blocks * s.E * 4);
  p->off_tile_expert = take((size_t)p->max_tiles * 4);
  p->off_tile_row0 = take((size_t)p->max_tiles * 4);
  p->off_tile_rows = take((size_t)p->max_tiles * 4);
  p->off_tile_ready = take((size_t)p->max_tiles * 4);
  p->off_tile_kind = take((size_t)p->max_tiles * 4);
  p->off_tile_order = take((size_t)p->max_tiles * 4);
  p->off_items0 = take((size_t)p->max_tiles * p->n_tiles_n0 * sizeof(ItemRec));
  p->off_items1 = take((size_t)(p->max_tiles + 3 * kXcds) * p->n_tiles_n1 * sizeof(ItemRec));
  p->off_panel_done = take((size_t)p->n_tiles_n1 * 4);
  p->off_tile_done = take((size_t)(p->max_tiles + 1) * 4);
  p->off_arrive = take((size_t)s.T * p->n_tiles_n1 * 4);
  p->off_h = take((size_t)s.R * s.F * 2);
  p->off_Y = take((size_t)s.R * s.H * 2);
  p->total_bytes = o;
}

Workspace view(const moe_plan* p, void* base) {
  char* b = (char*)base;
  Workspace w;
  w.status = (int32_t*)(b + p->off_status);
  w.counts = (int32_t*)(b + p->off_counts);
  w.offsets = (int32_t*)(b + p->off_offsets);
  w.perm = (int32_t*)(b + p->off_perm);
  w.inv_perm = (int32_t*)(b + p->off_inv_perm);
  w.row_token = (int32_t*)(b + p->off_row_token);
  w.block_hist = (int32_t*)(b + p->off_block_hist);
  w.tile_expert = (int32_t*)(b + p->off_tile_expert);
  w.tile_row0 = (int32_t*)(b + p->off_tile_row0);
  w.tile_rows = (int32_t*)(b + p->off_tile_rows);
  w.tile_ready = (int32_t*)(b + p->off_tile_ready);
  w.tile_kind = (int32_t*)(b + p->off_tile_kind);
  w.tile_order = (int32_t*)(b + p->off_tile_order);
  w.items0 = (ItemRec*)(b + p->off_items0);
  w.items1 = (ItemRec*)(b + p->off_items1);
  w.panel_done = (uint32_t*)(b + p->off_panel_done);
  w.tile_done = (uint32_t*)(b + p->off_tile_done);
  w.arrive = (uint32_t*)(b + p->off_arrive);
  w.h = (uint16_t*)(b + p->off_h);
  w.Y = (uint16_t*)(b + p->off_Y);
  return w;
}

int default_tile_m(const Shape& s) {
  // Tallest tile the schedule may use; the ragged end of an expert gets shorter tiles (128 / 64 rows) anyway.
  const int mean_rows = s.E > 0 ? s.R / s.E : 0;
  if (mean_rows >= 256) return 256;
  if (mean_rows >= 128) return 128;
  return 64;
}

// Division point between GEMM and data-movement workgroups of the layer1 kernel (Section 3.2.2): looked up, as the
// paper's metadata is, from a table of profiled shapes (the nearest one in rows per expert and experts).  The
// entries are the optima of the sweep tool (split_sweep.py: n_dm = 0, 2, 4, 8, 16, 32 on each shape): on one GPU the
// reduction is local HBM traffic of 40-70 us per forward and a workgroup taken from the GEMM side breaks the even
// split of the tall tiles over the compute units, so the curve of Fig. 8 has its minimum at its left edge on every
// shape profiled so far -- the GEMM workgroups reduce the panels themselves once they run out of tiles.
int default_n_dm(const Shape& s) {
  struct Row { int experts, rows_per_expert, hidden, n_dm; };
  static const Row table[] = {
      {8, 2048, 4096, 0},    // Mixtral-shaped           layer1 + reduction 1721 us at 0, 1767 at 2, ... 1817 at 32
      {64, 512, 3584, 0},    // Qwen2-shaped             763 / 878 / ... / 919
      {16, 2048, 4096, 0},   // Phi-3.5-shaped           1575 / 1641 / ... / 1794
      {8, 2048, 4096, 0},    // Mixtral TP8 slice        327 / 355 / ... / 396
      {64, 512, 2048, 0},    // Table 2's Qwen2 row      312 / 381 / ... / 393
  };
  const int rows = s.E > 0 ? s.R / s.E : 0;
  long best = -1;
  int n_dm = 0;
  for (const Row& r : table) {
    const long d = labs((long)r.rows_per_expert - rows) + 64L * labs((long)r.experts - s.E) + labs((long)r.hidden - s.H) / 8;
    if (best < 0 || d < best) {
      best = d;
      n_dm = r.n_dm;
    }
  }
  return n_dm;
}

// Division point between GEMM workgroups and workgroups that prefetch weight panels ahead of them, per GroupGEMM
// launch (Section 3.2.2 again: a number looked up from the shape).  Swept with bench.py (n_prefetch = 0, 8, 16, 24)
// on the two shapes with 64 small experts, where a weight panel serves two M-tiles and the weight stream is 2 TB/s:
// 683 / 703 / 720 / 743 us per forward on Table 2's Qwen2 row, 1859 / 1891 / 1925 / 1990 on the Qwen2-shaped workload.
// The minimum is at 0 there, and shapes with larger experts have less to gain, so the look-up returns 0 throughout.
int default_n_prefetch(const Shape& s) {
  (void)s;
  return 0;
}

// Waves the source segments are grouped into for the layer0 schedule when ready flags are in use (layer0_order 2):
// segment-major across waves so that tiles start as their rows arrive (Fig. 5), weight-panel-major inside a wave.
// Many waves follow a slow ingest closely but stream the layer0 weights once per wave; few waves keep the weight
// reuse of the expert-major order at the price of waiting for a wave's last segment.  Looked up, the way Section 3.2.2
// looks its division point up from profiled metadata, from the shape and the ingest rate the caller expects (option
// "expected_ingest_gbps").  The rule condenses the arrival experiment (arrival_experiment.py; arrival and layer
// together, 8 segments, fastest schedule per rate):
//                              25 GB/s           50 GB/s           100 GB/s          200 GB/s
//   Mixtral-shaped  (8 x 2048)  4 waves           4 waves           4 waves           4 waves
//   Phi-3.5-shaped (16 x 2048)  8 waves           4 waves           4 waves           4 waves
//   Qwen2-shaped    (64 x 512)  8 waves / by seg. 8 waves / by seg. expert-major      expert-major
// in two quantities: rows per expert (experts of two M-tiles have nothing to share inside a wave, so waves only cost
// them weight reuse) and rho = time the buffer takes to arrive / time layer0 takes when resident.
int default_layer0_waves(const Shape& s, int ingest_gbps) {
  const int rows_per_expert = s.E > 0 ? s.R / s.E : 0;
  const bool small_experts = rows_per_expert < 1024;
  int waves;
  if (ingest_gbps <= 0) {
    waves = small_experts ? 8 : 4;   // unknown rate
  } else {
    const double arrival_s = 2.0 * s.T * s.H / (ingest_gbps * 1e9);
    const double layer0_s = 2.0 * s.R * (double)s.H * s.F1 / 1.25e15;   // the layer0 GroupGEMM's rate on this part
    const double rho = arrival_s / layer0_s;
    if (small_experts) waves = rho >= 0.5 ? 8 : 1;
    else waves = rho > 1.5 ? 8 : 4;
  }
  if (waves > s.S) waves = s.S;
  return waves < 1 ? 1 : waves;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

extern "C" {

int moe_plan_create(moe_plan_t** plan, const moe_shape_t* shape, const int32_t* seg_offsets) {
  if (!plan || !shape || !seg_offsets) return MOE_ERR_INVALID_ARG;
  const moe_shape_t& sh = *shape;
  if (sh.T < 0 || sh.H <= 0 || sh.F <= 0 || sh.E <= 0 || sh.k <= 0 || sh.S <= 0) return MOE_ERR_INVALID_ARG;
  if (sh.act != MOE_ACT_GELU && sh.act != MOE_ACT_SWIGLU) return MOE_ERR_INVALID_ARG;
  if (sh.k > sh.E) return MOE_ERR_INVALID_ARG;
  if (sh.E > kMaxExperts || sh.k > kMaxTopK || sh.S > kMaxSegments) return MOE_ERR_UNSUPPORTED;
  if (sh.H % 256 != 0) return MOE_ERR_UNSUPPORTED;
  if (sh.F % (sh.act == MOE_ACT_SWIGLU ? 128 : 256) != 0) return MOE_ERR_UNSUPPORTED;
  if ((int64_t)sh.T * sh.k >= (1 << 24)) return MOE_ERR_UNSUPPORTED;
  // row offsets inside the kernels are 32-bit byte offsets
  if ((int64_t)sh.T * sh.H * 2 >= (1ll << 32) || (int64_t)sh.T * sh.k * sh.F * 2 >= (1ll << 32)) return MOE_ERR_UNSUPPORTED;
  if (seg_offsets[0] != 0 || seg_offsets[sh.S] != sh.T) return MOE_ERR_INVALID_ARG;
  for (int i = 0; i < sh.S; i++)
    if (seg_offsets[i + 1] < seg_offsets[i]) return MOE_ERR_INVALID_ARG;
  moe_plan* p = new (std::nothrow) moe_plan();
  if (!p) return MOE_ERR_INVALID_ARG;
  memset(p, 0, sizeof(*p));
  p->s.T = sh.T; p->s.H = sh.H; p->s.F = sh.F; p->s.E = sh.E; p->s.k = sh.k; p->s.S = sh.S; p->s.act = sh.act;
  p->s.R = sh.T * sh.k;
  p->s.F1 = sh.act == MOE_ACT_SWIGLU ? 2 * sh.F : sh.F;
  memcpy(p->seg_offsets, seg_offsets, sizeof(int32_t) * (sh.S + 1));
  p->tile_m = default_tile_m(p->s);
  p->n_dm = -1;
  p->n_prefetch = -1;
  p->deep_short_tiles = 1;
  p->prefetch_ahead = 16;
  p->prefetch_behind = 16;
  p->layer0_order = -1;
  p->layer1_order = 0;   // measured faster on every workload so far: see the sweep tool and default_n_dm
  p->serial = 0x2545F491;   // arbitrary start: an uninitialised workspace word is unlikely to match it
  p->block_m = 4;        // measured: 2-4 % faster on layer1 than 8, see the header
  p->publish_every = 16;
  p->spin_limit = 1 << 26;   // about 20 s of polling: a lost flag ends in MOE_ERR_TIMEOUT, not in a hung GPU
  p->phases = 15;
  p->n_cu = 0;
  layout(p);
  *plan = p;
  return MOE_OK;
}

int moe_plan_destroy(moe_plan_t* plan) {
  if (plan && plan->ev_created)
    for (int i = 0; i < kProfSlots; i++)
      for (int j = 0; j < 5; j++) (void)hipEventDestroy(plan->ev[i][j]);
  delete plan;
  return MOE_OK;
}

int moe_plan_set_option(moe_plan_t* p, const char* key, int64_t v) {
  if (!p || !key) return MOE_ERR_INVALID_ARG;
  if (!strcmp(key, "tile_m")) {
    if (v != 64 && v != 128 && v != 256) return MOE_ERR_INVALID_ARG;
    p->tile_m = (int32_t)v;
    layout(p);
    return MOE_OK;
  }
  if (!strcmp(key, "n_dm")) {
    if (v < -1 || v > 240) return MOE_ERR_INVALID_ARG;
    p->n_dm = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "deep_short_tiles")) {
    if (v != 0 && v != 1) return MOE_ERR_INVALID_ARG;
    p->deep_short_tiles = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "n_prefetch")) {
    if (v < -1 || v > 64 || (v > 0 && v % 8 != 0)) return MOE_ERR_INVALID_ARG;
    p->n_prefetch = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "prefetch_ahead") || !strcmp(key, "prefetch_behind")) {
    if (v < 0 || v > 4096) return MOE_ERR_INVALID_ARG;
    (key[9] == 'a' ? p->prefetch_ahead : p->prefetch_behind) = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "layer0_order")) {
    if (v < -1 || v > 2) return MOE_ERR_INVALID_ARG;
    p->layer0_order = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "layer0_waves")) {
    if (v < 0 || v > 8) return MOE_ERR_INVALID_ARG;
    p->layer0_waves = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "expected_ingest_gbps")) {
    if (v < 0 || v > 1000000) return MOE_ERR_INVALID_ARG;
    p->expected_ingest_gbps = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "layer1_order")) {
    if (v < 0 || v > 2) return MOE_ERR_INVALID_ARG;
    p->layer1_order = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "spin_limit")) {
    if (v < 0 || v > 0x7fffffff) return MOE_ERR_INVALID_ARG;
    p->spin_limit = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "phases")) {
    if (v < 0 || v > 15) return MOE_ERR_INVALID_ARG;
    p->phases = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "n_cu")) {
    if (v < 8 || v > 1024) return MOE_ERR_INVALID_ARG;
    p->n_cu = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "block_m")) {
    if (v < 1 || v > 8) return MOE_ERR_INVALID_ARG;
    p->block_m = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "large_schedule")) {
    if (v != 0 && v != 1) return MOE_ERR_INVALID_ARG;
    p->large_schedule = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "weights_packed")) {
    if (v != 0 && v != 1) return MOE_ERR_INVALID_ARG;
    p->weights_packed = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "fuse_layers")) {
    if (v != 0 && v != 1) return MOE_ERR_INVALID_ARG;
    p->fuse_layers = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "publish_every")) {
    if (v < 1 || v > 1 << 20) return MOE_ERR_INVALID_ARG;
    p->publish_every = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "handoff_fences")) {
    if (v != 0 && v != 1) return MOE_ERR_INVALID_ARG;
    p->handoff_fences = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "alias_experts")) {
    if (v != 0 && v != 1) return MOE_ERR_INVALID_ARG;
    p->alias_experts = (int32_t)v;
    return MOE_OK;
  }
  if (!strcmp(key, "profile")) {
    if (v != 0 && v != 1) return MOE_ERR_INVALID_ARG;
    if (v == 1 && !p->ev_created) {
      for (int i = 0; i < kProfSlots; i++)
        for (int j = 0; j < 5; j++)
          if (hipEventCreate(&p->ev[i][j]) != hipSuccess) return MOE_ERR_HIP;
      p->ev_created = true;
    }
    p->profile = (int32_t)v;
    p->prof_steps = 0;
    p->prof_dropped = 0;
    return MOE_OK;
  }
  return MOE_ERR_INVALID_ARG;
}

int moe_plan_get_option(const moe_plan_t* p, const char* key, int64_t* v) {
  if (!p || !key || !v) return MOE_ERR_INVALID_ARG;
  if (!strcmp(key, "tile_m")) *v = p->tile_m;
  else if (!strcmp(key, "n_dm")) *v = p->n_dm >= 0 ? p->n_dm : default_n_dm(p->s);
  else if (!strcmp(key, "n_prefetch")) *v = p->n_prefetch >= 0 ? p->n_prefetch : default_n_prefetch(p->s);
  else if (!strcmp(key, "deep_short_tiles")) *v = p->deep_short_tiles;
  else if (!strcmp(key, "prefetch_ahead")) *v = p->prefetch_ahead;
  else if (!strcmp(key, "prefetch_behind")) *v = p->prefetch_behind;
  else if (!strcmp(key, "layer0_order")) *v = p->layer0_order;
  else if (!strcmp(key, "layer0_waves")) *v = p->layer0_waves > 0 ? p->layer0_waves : default_layer0_waves(p->s, p->expected_ingest_gbps);
  else if (!strcmp(key, "expected_ingest_gbps")) *v = p->expected_ingest_gbps;
  else if (!strcmp(key, "layer1_order")) *v = p->layer1_order;
  else if (!strcmp(key, "spin_limit")) *v = p->spin_limit;
  else if (!strcmp(key, "phases")) *v = p->phases;
  else if (!strcmp(key, "n_cu")) *v = p->n_cu;
  else if (!strcmp(key, "profile")) *v = p->profile;
  else if (!strcmp(key, "profile_dropped")) *v = p->prof_dropped;
  else if (!strcmp(key, "large_schedule")) *v = p->large_schedule;
  else if (!strcmp(key, "block_m")) *v = p->block_m;
  else if (!strcmp(key, "weights_packed")) *v = p->weights_packed;
  else if (!strcmp(key, "alias_experts")) *v = p->alias_experts;
  else if (!strcmp(key, "handoff_fences")) *v = p->handoff_fences;
  else if (!strcmp(key, "fuse_layers")) *v = p->fuse_layers;
  else if (!strcmp(key, "publish_every")) *v = p->publish_every;
  else return MOE_ERR_INVALID_ARG;
  return MOE_OK;
}

size_t moe_plan_workspace_bytes(const moe_plan_t* p) { return p ? p->total_bytes : 0; }

int32_t moe_plan_max_tiles(const moe_plan_t* p) { return p ? p->max_tiles : 0; }

size_t moe_receive_buffer_bytes(int64_t M, int64_t N) { return (M < 0 || N < 0) ? 0 : (size_t)(2 * M * N); }

int moe_route_topk(const float* logits, int32_t T, int32_t E, int32_t k, int32_t* topk_ids, float* topk_weights,
                   void* hip_stream) {
  if (!logits || !topk_ids || !topk_weights) return MOE_ERR_INVALID_ARG;
  if (T < 0 || E <= 0 || k <= 0 || k > E) return MOE_ERR_INVALID_ARG;
  if (E > kMaxExperts || k > 64) return MOE_ERR_UNSUPPORTED;
  return launch_route_topk(logits, T, E, k, topk_ids, topk_weights, (hipStream_t)hip_stream) == hipSuccess ? MOE_OK
                                                                                                            : MOE_ERR_HIP;
}

}  // extern "C"

namespace {

int forward_impl(moe_plan_t* p, const void* x, const int32_t* topk_ids, const float* topk_weights, const void* W1,
                 const void* W2, int32_t act, void* out, void* workspace, size_t workspace_bytes,
                 const uint32_t* seg_ready, uint32_t ready_epoch, void* hip_stream) {
  if (!p || !x || !topk_ids || !topk_weights || !W1 || !W2 || !out || !workspace) return MOE_ERR_INVALID_ARG;
  if (act != p->s.act) return MOE_ERR_SHAPE_MISMATCH;
  if (workspace_bytes < p->total_bytes) return MOE_ERR_WORKSPACE_TOO_SMALL;
  if (!aligned16(x) || !aligned16(W1) || !aligned16(W2) || !aligned16(out) || !aligned16(topk_ids) ||
      !aligned16(topk_weights) || ((uintptr_t)workspace & 255))
    return MOE_ERR_INVALID_ARG;
  const Shape& s = p->s;
  if (s.T == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  if (p->n_cu == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return MOE_ERR_HIP;
    p->n_cu = n;
  }
  Workspace ws = view(p, workspace);
  // The layer0 tile order of this forward: the schedule is built inside the forward, so it can follow what the
  // forward is given.  All rows resident: expert-major (weight reuse first).  Ready flags in use: waves of source
  // segments (Fig. 5).  The one-workgroup builder for very large tile tables knows orders 0 and 1 only.
  const bool large = uses_large_schedule(p->max_tiles, p->large_schedule);
  int order0 = p->layer0_order >= 0 ? p->layer0_order : (seg_ready ? 2 : 0);
  const int waves0 = p->layer0_waves > 0 ? p->layer0_waves : default_layer0_waves(s, p->expected_ingest_gbps);
  if (order0 == 2 && large) order0 = 1;
  if (p->phases & 1) p->last_layer0_order = order0;
  else order0 = p->last_layer0_order;   // the schedules of the last index build are run again
  // a forward beyond the last event slot is not recorded (and counted as dropped) rather than overwriting an earlier one
  hipEvent_t* ev = (p->profile && p->prof_steps < kProfSlots) ? p->ev[p->prof_steps] : nullptr;
  if (p->profile && !ev) p->prof_dropped++;
  auto mark = [&](int i) { return !ev || hipEventRecord(ev[i], st) == hipSuccess; };
  if (!mark(0)) return MOE_ERR_HIP;

  if (p->phases & 1) {
    IndexParams ip;
    memset(&ip, 0, sizeof(ip));
    ip.s = s;
    ip.ws = ws;
    ip.topk_ids = topk_ids;
    ip.n_blocks = p->n_index_blocks;
    ip.tile_m = p->tile_m;
    ip.n_tiles_n0 = p->n_tiles_n0;
    ip.n_tiles_n1 = p->n_tiles_n1;
    ip.layer0_order = order0;
    ip.layer0_waves = waves0;
    ip.layer1_order = p->layer1_order == 1 ? 1 : 0;   // only the in-kernel panel reduction needs the panel-major order
    ip.max_tiles = p->max_tiles;
    ip.force_large_schedule = p->large_schedule;
    ip.block_m = p->block_m;
    ip.forward_serial = ++p->serial;
    memcpy(ip.seg_offsets, p->seg_offsets, sizeof(int32_t) * (s.S + 1));
    if (launch_index_build(ip, st) != hipSuccess) return MOE_ERR_HIP;
  } else {
    // the schedules of the last index build on this workspace are run again: their queue heads and counters start over
    if (launch_reset_counters(ws, p->n_tiles_n1, p->max_tiles, st) != hipSuccess) return MOE_ERR_HIP;
  }

  if (!mark(1)) return MOE_ERR_HIP;

  GemmParams g;
  memset(&g, 0, sizeof(g));
  g.tile_expert = ws.tile_expert;
  g.tile_row0 = ws.tile_row0;
  g.tile_rows = ws.tile_rows;
  g.tile_ready = ws.tile_ready;
  g.tile_kind = ws.tile_kind;
  g.status = ws.status;
  g.spin_limit = (uint32_t)p->spin_limit;
  g.n_tiles = ws.status + 1;
  g.F = s.F;
  g.T = s.T;
  g.k = s.k;
  g.H = s.H;
  g.handoff_fences = p->handoff_fences;
  g.deep_short_tiles = p->deep_short_tiles;

  const bool fused = p->layer1_order == 1 && (p->phases & 8);   // top-k reduction inside the layer1 kernel
  const bool in_epilogue = p->layer1_order == 2 && (p->phases & 8) && (p->phases & 4);   // ... in its epilogue
  // both GroupGEMMs in one launch (only with the separate combine kernel and the LDS-resident schedule builder's
  // tile count, which bounds the per-workgroup tile counters)
  const bool one_launch = p->fuse_layers && (p->phases & 2) && (p->phases & 4) && !fused && !large;

  GemmParams a = g;
  a.A = (const char*)x;
  a.lda_bytes = (uint32_t)s.H * 2;
  a.a_rows = ws.row_token;
  a.B = (const char*)W1;
  a.b_expert_bytes = (uint64_t)s.H * s.F1 * 2;
  a.ldb = (uint32_t)s.F1;
  a.b_packed = p->weights_packed;
  if (p->alias_experts && !p->weights_packed) a.b_expert_bytes = 0;   // measurement aid, see the option
  a.n_tiles_n = p->n_tiles_n0;
  a.C = ws.h;
  a.ldc = (uint32_t)s.F;
  a.K = s.H;
  a.items = ws.items0;
  a.seg_ready = seg_ready;
  a.ready_epoch = ready_epoch;
  a.n_segments = s.S;
  // no more workgroups than there can be items (small batches are bound by the launch, not by the work)
  const int64_t max_items0 = (int64_t)p->max_tiles * p->n_tiles_n0;
  const int grid0 = max_items0 < p->n_cu ? (max_items0 < 8 ? 8 : (int)max_items0) : p->n_cu;
  a.n_mfma = grid0;
  // prefetching workgroups: only with packed weights, a full launch and the separate kernels
  int n_prefetch = p->n_prefetch >= 0 ? p->n_prefetch : default_n_prefetch(s);
  if (!p->weights_packed || fused || one_launch) n_prefetch = 0;
  if (grid0 == p->n_cu && n_prefetch + 8 <= grid0) {
    a.n_prefetch = n_prefetch;
    a.prefetch_ahead = p->prefetch_ahead;
    a.prefetch_behind = p->prefetch_behind;
  }
  a.queue_heads = ws.status + 8;
  a.queue_len = ws.status + 24;
  if (order0 != 1 && !large) {
    a.queue_base = ws.status + 48;   // contiguous per-XCD queues (locality order)
    a.queue_stride = 1;
  } else {
    a.queue_base = nullptr;          // queue x = list positions x, x + 8, ...
    a.queue_stride = kXcds;
  }

  GemmParams b = g;
  b.A = (const char*)ws.h;
  b.lda_bytes = (uint32_t)s.F * 2;
  b.a_rows = nullptr;
  b.B = (const char*)W2;
  b.b_expert_bytes = (uint64_t)s.F * s.H * 2;
  b.ldb = (uint32_t)s.H;
  b.b_packed = p->weights_packed;
  if (p->alias_experts && !p->weights_packed) b.b_expert_bytes = 0;
  b.n_tiles_n = p->n_tiles_n1;
  b.C = ws.Y;
  b.ldc = (uint32_t)s.H;
  b.K = s.F;
  b.items = ws.items1;
  b.panel_done = ws.panel_done;
  int n_dm = fused ? (p->n_dm >= 0 ? p->n_dm : default_n_dm(s)) : 0;
  if (n_dm > p->n_cu - 8) n_dm = p->n_cu - 8;
  const int64_t max_items1 = (int64_t)p->max_tiles * p->n_tiles_n1;
  int grid1 = p->n_cu;
  if (!fused && max_items1 < grid1) grid1 = max_items1 < 8 ? 8 : (int)max_items1;
  b.n_mfma = grid1 - n_dm;
  if (grid1 == p->n_cu && n_prefetch + 8 <= grid1) {
    b.n_prefetch = n_prefetch;
    b.prefetch_ahead = p->prefetch_ahead;
    b.prefetch_behind = p->prefetch_behind;
  }
  b.fused_combine = fused ? 1 : 0;
  b.batch_publish = (fused && n_dm == 0 && s.H / kTileN <= 128) ? 1 : 0;
  b.inv_perm = ws.inv_perm;
  b.topk_weights = topk_weights;
  b.out = (uint16_t*)out;
  b.combine_counter = ws.status + 4;
  b.queue_heads = ws.status + 16;
  b.queue_len = ws.status + 32;
  b.queue_base = ws.status + 40;
  b.queue_stride = 1;
  if (in_epilogue) {
    b.epilogue_combine = 1;
    b.arrive = ws.arrive;
    b.perm = ws.perm;
    if (launch_zero_u32(ws.arrive, (size_t)s.T * p->n_tiles_n1, st) != hipSuccess) return MOE_ERR_HIP;
  }

  if (one_launch) {
    FuseParams f;
    f.tile_done = ws.tile_done;
    f.wgs_done = ws.tile_done + p->max_tiles;
    f.n_tiles_n0 = p->n_tiles_n0;
    f.publish_every = p->publish_every;
    const int grid = grid0 > grid1 ? grid0 : grid1;
    a.n_mfma = grid;
    b.n_mfma = grid;
    if (launch_fused_layers(a, b, f, s.act, grid, st) != hipSuccess) return MOE_ERR_HIP;
    if (!mark(2)) return MOE_ERR_HIP;   // the whole launch is booked as the layer0 phase
  } else {
    if ((p->phases & 2) && launch_layer0(a, s.act, grid0, st) != hipSuccess) return MOE_ERR_HIP;
    if (!mark(2)) return MOE_ERR_HIP;
    if ((p->phases & 4) && launch_layer1(b, grid1, st) != hipSuccess) return MOE_ERR_HIP;
  }
  if (!mark(3)) return MOE_ERR_HIP;
  if ((p->phases & 8) && !(fused && (p->phases & 4)) && !in_epilogue) {
    CombineParams c;
    c.Y = ws.Y;
    c.inv_perm = ws.inv_perm;
    c.topk_weights = topk_weights;
    c.out = (uint16_t*)out;
    c.T = s.T;
    c.k = s.k;
    c.H = s.H;
    if (launch_combine(c, st) != hipSuccess) return MOE_ERR_HIP;
  }
  if (!mark(4)) return MOE_ERR_HIP;
  if (ev) p->prof_steps++;
  return MOE_OK;
}

// Address of this device's copy of the static workspace, looked up once per device.
int static_scratch(void** ptr) {
  static std::mutex mu;
  static void* per_device[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(mu);
  if (!per_device[dev]) {
    void* a = nullptr;
    if (hipGetSymbolAddress(&a, HIP_SYMBOL(scratch)) != hipSuccess || !a) return MOE_ERR_HIP;
    per_device[dev] = a;
  }
  *ptr = per_device[dev];
  return MOE_OK;
}

}  // namespace

extern "C" {

int moe_layer_forward(moe_plan_t* p, const void* x, const int32_t* topk_ids, const float* topk_weights, const void* W1,
                      const void* W2, int32_t act, void* out, void* workspace, size_t workspace_bytes,
                      const uint32_t* seg_ready, uint32_t ready_epoch, void* hip_stream) {
  return forward_impl(p, x, topk_ids, topk_weights, W1, W2, act, out, workspace, workspace_bytes, seg_ready, ready_epoch,
                      hip_stream);
}

int moe_layer_forward_static(moe_plan_t* p, const void* x, const int32_t* topk_ids, const float* topk_weights,
                             const void* W1, const void* W2, int32_t act, void* out, const uint32_t* seg_ready,
                             uint32_t ready_epoch, void* hip_stream) {
  if (!p) return MOE_ERR_INVALID_ARG;
  if (p->total_bytes > kStaticScratchBytes) return MOE_ERR_WORKSPACE_TOO_SMALL;   // the plan needs more than the fixed 32 MiB
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != MOE_OK) return rc;
  return forward_impl(p, x, topk_ids, topk_weights, W1, W2, act, out, ws, kStaticScratchBytes, seg_ready, ready_epoch,
                      hip_stream);
}

int moe_pack_weights(const moe_plan_t* p, const void* W1, const void* W2, void* W1_packed, void* W2_packed, void* hip_stream) {
  if (!p || (!W1 != !W1_packed) || (!W2 != !W2_packed)) return MOE_ERR_INVALID_ARG;
  if ((W1 && (!aligned16(W1) || !aligned16(W1_packed) || W1 == W1_packed)) ||
      (W2 && (!aligned16(W2) || !aligned16(W2_packed) || W2 == W2_packed)))
    return MOE_ERR_INVALID_ARG;
  const Shape& s = p->s;
  hipStream_t st = (hipStream_t)hip_stream;
  if (W1 && launch_pack_weights(W1, W1_packed, s.E, s.H, s.F1, p->n_tiles_n0, s.act == MOE_ACT_SWIGLU ? s.F : 0, st) != hipSuccess)
    return MOE_ERR_HIP;
  if (W2 && launch_pack_weights(W2, W2_packed, s.E, s.F, s.H, p->n_tiles_n1, 0, st) != hipSuccess) return MOE_ERR_HIP;
  return MOE_OK;
}

int moe_plan_phase_times(moe_plan_t* p, float* ms, int32_t* n_steps) {
  if (!p || !ms || !n_steps) return MOE_ERR_INVALID_ARG;
  const int n = p->prof_steps;
  *n_steps = n;
  for (int j = 0; j < 4; j++) ms[j] = 0.f;
  if (n == 0) return MOE_OK;
  for (int i = 0; i < n; i++) {
    if (hipEventSynchronize(p->ev[i][4]) != hipSuccess) return MOE_ERR_HIP;
    for (int j = 0; j < 4; j++) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, p->ev[i][j], p->ev[i][j + 1]) != hipSuccess) return MOE_ERR_HIP;
      ms[j] += t;
    }
  }
  for (int j = 0; j < 4; j++) ms[j] /= n;
  p->prof_steps = 0;
  p->prof_dropped = 0;
  return MOE_OK;
}

int moe_plan_forward_times(moe_plan_t* p, float* ms, int32_t capacity, int32_t* n_steps) {
  if (!p || !ms || !n_steps || capacity < 0) return MOE_ERR_INVALID_ARG;
  int n = p->prof_steps;
  if (n > capacity) n = capacity;
  *n_steps = n;
  for (int i = 0; i < n; i++) {
    if (hipEventSynchronize(p->ev[i][4]) != hipSuccess) return MOE_ERR_HIP;
    if (hipEventElapsedTime(&ms[i], p->ev[i][0], p->ev[i][4]) != hipSuccess) return MOE_ERR_HIP;
  }
  return MOE_OK;
}

int moe_get_index_outputs(const moe_plan_t* p, const void* workspace, int32_t* expert_counts, int32_t* expert_offsets,
                          int32_t* perm, int32_t* inv_perm, void* hip_stream) {
  if (!p || !workspace) return MOE_ERR_INVALID_ARG;
  Workspace ws = view(p, const_cast<void*>(workspace));
  hipStream_t st = (hipStream_t)hip_stream;
  const Shape& s = p->s;
  auto cp = [&](void* dst, const void* src, size_t bytes) {
    return !dst || bytes == 0 || hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st) == hipSuccess;
  };
  if (!cp(expert_counts, ws.counts, (size_t)s.E * 4) || !cp(expert_offsets, ws.offsets, (size_t)(s.E + 1) * 4) ||
      !cp(perm, ws.perm, (size_t)s.R * 4) || !cp(inv_perm, ws.inv_perm, (size_t)s.R * 4))
    return MOE_ERR_HIP;
  return MOE_OK;
}

int moe_get_tile_table(const moe_plan_t* p, const void* workspace, int32_t* n_tiles, int32_t* tile_expert,
                       int32_t* tile_row0, int32_t* tile_rows, int32_t* tile_ready_seg, int32_t* tile_height,
                       void* hip_stream) {
  if (!p || !workspace) return MOE_ERR_INVALID_ARG;
  Workspace ws = view(p, const_cast<void*>(workspace));
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t tb = (size_t)p->max_tiles * 4;
  auto cp = [&](void* dst, const void* src, size_t bytes) {
    return !dst || bytes == 0 || hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st) == hipSuccess;
  };
  if (!cp(n_tiles, ws.status + 1, 4) || !cp(tile_expert, ws.tile_expert, tb) || !cp(tile_row0, ws.tile_row0, tb) ||
      !cp(tile_rows, ws.tile_rows, tb) || !cp(tile_ready_seg, ws.tile_ready, tb))
    return MOE_ERR_HIP;
  if (tile_height && launch_tile_heights(ws.tile_kind, tile_height, p->max_tiles, st) != hipSuccess) return MOE_ERR_HIP;
  return MOE_OK;
}

int64_t moe_plan_schedule_capacity(const moe_plan_t* p, int32_t layer) {
  if (!p || (layer != 0 && layer != 1)) return 0;
  return layer == 0 ? (int64_t)p->max_tiles * p->n_tiles_n0 : (int64_t)(p->max_tiles + 3 * kXcds) * p->n_tiles_n1;
}

int moe_get_schedule(const moe_plan_t* p, const void* workspace, int32_t layer, int32_t* items, int32_t* queues,
                     void* hip_stream) {
  if (!p || !workspace || !queues || (layer != 0 && layer != 1)) return MOE_ERR_INVALID_ARG;
  Workspace ws = view(p, const_cast<void*>(workspace));
  hipStream_t st = (hipStream_t)hip_stream;
  int32_t status[64];
  if (hipMemcpyAsync(status, ws.status, sizeof(status), hipMemcpyDeviceToHost, st) != hipSuccess) return MOE_ERR_HIP;
  if (items) {
    const size_t bytes = (size_t)moe_plan_schedule_capacity(p, layer) * sizeof(ItemRec);
    if (bytes && hipMemcpyAsync(items, layer == 0 ? ws.items0 : ws.items1, bytes, hipMemcpyDeviceToDevice, st) != hipSuccess)
      return MOE_ERR_HIP;
  }
  if (hipStreamSynchronize(st) != hipSuccess) return MOE_ERR_HIP;
  const bool strided0 = !(p->last_layer0_order != 1 && !uses_large_schedule(p->max_tiles, p->large_schedule));
  for (int x = 0; x < kXcds; x++) {
    if (layer == 0) {
      queues[x] = strided0 ? x : status[48 + x];
      queues[kXcds + x] = status[24 + x];
      queues[2 * kXcds + x] = strided0 ? kXcds : 1;
    } else {
      queues[x] = status[40 + x];
      queues[kXcds + x] = status[32 + x];
      queues[2 * kXcds + x] = 1;
    }
  }
  return MOE_OK;
}

int moe_play_arrival(const moe_plan_t* p, const void* staging, void* x, uint32_t* seg_ready, uint32_t* seg_counters,
                     uint32_t ready_epoch, double gbytes_per_s, int32_t n_workgroups, void* hip_stream) {
  if (!p || !staging || !x || !seg_ready || !seg_counters) return MOE_ERR_INVALID_ARG;
  if (!aligned16(staging) || !aligned16(x) || gbytes_per_s < 0 || n_workgroups < 1 || n_workgroups > 64)
    return MOE_ERR_INVALID_ARG;
  if (p->s.T == 0) return MOE_OK;
  ArrivalParams a;
  memset(&a, 0, sizeof(a));
  a.S = p->s.S;
  memcpy(a.seg_offsets, p->seg_offsets, sizeof(int32_t) * (p->s.S + 1));
  a.row_bytes = (uint32_t)p->s.H * 2;
  a.chunk16 = 64 * 1024 / 16;
  a.bytes_per_us = gbytes_per_s * 1e3;
  a.seg_ready = seg_ready;
  a.seg_arrived = seg_counters;
  a.epoch = ready_epoch;
  return launch_arrival_producer(staging, x, a, n_workgroups, (hipStream_t)hip_stream) == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int moe_last_device_status(const moe_plan_t* p, const void* workspace, void* hip_stream) {
  if (!p || !workspace) return MOE_ERR_INVALID_ARG;
  Workspace ws = view(p, const_cast<void*>(workspace));
  int32_t v[6] = {0, 0, 0, 0, 0, 0};
  if (hipMemcpyAsync(v, ws.status, sizeof(v), hipMemcpyDeviceToHost, (hipStream_t)hip_stream) != hipSuccess) return MOE_ERR_HIP;
  if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return MOE_ERR_HIP;
  if (v[0] != 0) return v[0];
  return v[5] == p->serial ? MOE_ERR_INVALID_ARG : MOE_OK;
}

const char* moe_status_string(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID_ARG: return "invalid argument";
    case MOE_ERR_SHAPE_MISMATCH: return "arguments disagree with the plan";
    case MOE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MOE_ERR_UNSUPPORTED: return "shape not supported";
    case MOE_ERR_HIP: return "HIP runtime error";
    case MOE_ERR_TIMEOUT: return "wait on a ready flag timed out";
    default: return "unknown status";
  }
}

}  // extern "C"
