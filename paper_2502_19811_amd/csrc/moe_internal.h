// Internal declarations shared by the kernels and the host API of libmoe_gfx950.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe_gfx950.h"

namespace moe {

constexpr int kMaxExperts = 256;
constexpr int kMaxTopK = 16;
constexpr int kMaxSegments = 64;
constexpr int kIndexChunk = 1024;   // (token, slot) pairs handled by one workgroup of the index build
constexpr int kTileN = 256;         // columns of B staged per GroupGEMM tile
constexpr int kTileK = 32;          // depth of one LDS stage
constexpr int kStages = 4;          // LDS stages in flight
constexpr int kCombineChunk = 256;  // tokens per unit of combine work
constexpr int kXcds = 8;            // XCDs of the device: workgroup i runs on XCD i % 8
constexpr int kScheduleTileCap = 2048;  // M-tiles up to which the multi-workgroup schedule builder is used

// Which schedule builder a plan uses: the one-workgroup kernel has no size limit (and simpler orders).
inline bool uses_large_schedule(int max_tiles, int force) { return force != 0 || max_tiles > kScheduleTileCap; }

// Item of a GroupGEMM schedule: one (M-tile, column tile) pair with the M-tile's table row copied in, so that a
// workgroup needs a single 32-byte read to start on it.
struct ItemRec {
  int32_t m_tile, n_tile, expert, row0, nrows, kind, ready_seg, pad;
};

// Device-side view of the workspace (all pointers into the caller's workspace buffer).
struct Workspace {
  int32_t* status;        // [64]  0: device status word, 1: n_tiles, 2: items of layer0, 3: items of layer1,
                          //       4: combine unit counter, 5: serial number of the last forward that saw an expert
                          //       id out of range; per XCD: 8..15 layer0 queue heads, 16..23 layer1 queue
                          //       heads, 24..31 layer0 queue lengths, 32..39 layer1 queue lengths, 40..47 layer1
                          //       queue bases, 48..55 layer0 queue bases (only with contiguous layer0 queues;
                          //       otherwise layer0's queue x is list positions x, x+8, ...)
  int32_t* counts;        // [E]
  int32_t* offsets;       // [E+1]
  int32_t* perm;          // [R] sorted row -> pair id
  int32_t* inv_perm;      // [R] pair id -> sorted row
  int32_t* row_token;     // [R] sorted row -> token (row of x to gather)
  int32_t* block_hist;    // [n_index_blocks * E] rows of each expert among a workgroup's pair ids
  int32_t* tile_expert;   // [max_tiles]
  int32_t* tile_row0;     // [max_tiles]
  int32_t* tile_rows;     // [max_tiles]
  int32_t* tile_ready;    // [max_tiles] source segment the tile waits for
  int32_t* tile_kind;     // [max_tiles] 0 / 1 / 2: the tile is computed by the 64 / 128 / 256-row kernel variant
  int32_t* tile_order;    // [max_tiles] scratch of the schedule builder: tiles sorted tallest first
  ItemRec* items0;        // [max_tiles * n_tiles_n0] layer0 schedule
  ItemRec* items1;        // [(max_tiles + 24) * n_tiles_n1] layer1 schedule, one contiguous queue per XCD
  uint32_t* panel_done;   // [n_tiles_n1] finished M-tiles per column panel of layer1
  uint32_t* arrive;       // [T * n_tiles_n1] epilogue reduction: rows of a token already written, per column panel
  uint32_t* tile_done;    // [max_tiles + 1] one-launch variant: layer0 items finished per M-tile; last: workgroups done
  uint16_t* h;            // [R,F] bf16 activation buffer
  uint16_t* Y;            // [R,H] bf16 layer1 shared tensor
};

struct Shape {
  int32_t T, H, F, E, k, S, act;
  int32_t R, F1;
};

struct IndexParams {
  Shape s;
  Workspace ws;
  const int32_t* topk_ids;
  int32_t n_blocks;
  int32_t tile_m;
  int32_t n_tiles_n0, n_tiles_n1;
  int32_t layer0_order, layer1_order;   // layer0: 0 expert-major, 1 by source segment, 2 waves of segments
  int32_t layer0_waves;                 // order 2: waves the source segments are grouped into (1..8)
  int32_t max_tiles;             // bound on the M-tiles of this plan
  int32_t force_large_schedule;  // 1: build the schedules with the one-workgroup kernel whatever the size
  int32_t block_m;               // M-tiles per block of the locality order (1..8)
  int32_t forward_serial;        // written to status[5] when an expert id is out of range
  int32_t seg_offsets[kMaxSegments + 1];
};

struct GemmParams {
  const char* A;            // x (layer0) or h (layer1), bf16
  uint32_t lda_bytes;
  const int32_t* a_rows;    // layer0: sorted row -> row of A (gather); layer1: nullptr (identity)
  const char* B;            // W1 or W2
  uint64_t b_expert_bytes;  // bytes between experts
  uint32_t ldb;             // elements per row of B
  int32_t b_packed;         // 1: B is in the packed layout of moe_pack_weights (b_expert_bytes and ldb unused)
  int32_t n_tiles_n;        // column tiles of this layer (addressing of packed B)
  int32_t handoff_fences;   // measurement aid: per-tile agent-scope release (layer0) / acquire (layer1)
  int32_t no_pre;           // 1: a tile never starts its successor's loads early (the successor's rows may not be there)
  int32_t deep_short_tiles; // 1: 64-row tiles keep five K steps of operands in flight instead of three
  int32_t n_prefetch;       // workgroups (the last of the launch, a multiple of 8) that prefetch packed weight panels
  int32_t prefetch_ahead;   // ... for the items up to this far beyond the head of their XCD's queue
  int32_t prefetch_behind;  // ... and this far before it (handed out, probably not started yet)
  uint16_t* C;              // h (layer0) or Y (layer1)
  uint32_t ldc;             // elements per row of C
  int32_t K;                // reduction length
  int32_t F;                // expert hidden size (gate/up split of W1 columns)
  const int32_t* tile_expert;
  const int32_t* tile_row0;
  const int32_t* tile_rows;
  const int32_t* tile_ready;
  const int32_t* tile_kind;
  const ItemRec* items;
  const uint32_t* seg_ready;
  uint32_t ready_epoch;
  int32_t n_segments;       // entries of seg_ready
  uint32_t spin_limit;
  int32_t* status;
  int32_t* queue_heads;     // [8] items already taken from each XCD's queue
  const int32_t* queue_len; // [8] items in each XCD's queue
  const int32_t* queue_base;// [8] list position of each queue's first item; nullptr: queue x starts at x
  int32_t queue_stride;     // list positions between consecutive items of a queue
  // layer1 only
  uint32_t* panel_done;
  const int32_t* n_tiles;   // device scalar: M-tiles in total
  int32_t n_mfma;           // workgroups doing GEMM tiles; the rest are data-movement workgroups
  int32_t fused_combine;    // 1: data-movement workgroups reduce finished panels inside this kernel
  int32_t epilogue_combine; // 1: the layer1 epilogue reduces a token once its last row has arrived (arrive[], perm)
  uint32_t* arrive;         // [T * H/256] rows of a token already written, per column panel
  const int32_t* perm;      // [R] sorted row -> pair id
  int32_t batch_publish;    // 1: no data-movement workgroups: a GEMM workgroup publishes all its tiles at its end
  // combine
  const int32_t* inv_perm;
  const float* topk_weights;
  uint16_t* out;
  int32_t T, k, H;
  int32_t* combine_counter;
};

// The two GroupGEMMs in one launch: what the hand-over of h from layer0 tiles to layer1 tiles needs.
struct FuseParams {
  uint32_t* tile_done;      // [max_tiles] layer0 items finished (and published) per M-tile
  uint32_t* wgs_done;       // [1] workgroups that have published all their layer0 tiles
  int32_t n_tiles_n0;       // layer0 items per M-tile
  int32_t publish_every;    // layer0 tiles between two publications of a workgroup
};

struct ArrivalParams {
  int32_t S;
  int32_t seg_offsets[kMaxSegments + 1];
  uint32_t row_bytes;      // bytes of one token row
  uint32_t chunk16;        // 16-byte units copied between two pacing checks
  double bytes_per_us;     // 0: as fast as one workgroup copies
  uint32_t* seg_ready;
  uint32_t* seg_arrived;   // [S] workgroups done with each segment; zero between calls
  uint32_t epoch;
};

struct CombineParams {
  const uint16_t* Y;
  const int32_t* inv_perm;
  const float* topk_weights;
  uint16_t* out;
  int32_t T, k, H;
};

// kernel launchers (defined in the .hip files)
hipError_t launch_route_topk(const float* logits, int T, int E, int k, int32_t* ids, float* w, hipStream_t st);
hipError_t launch_index_build(const IndexParams& p, hipStream_t st);
hipError_t launch_reset_counters(const Workspace& ws, int n_tiles_n1, int max_tiles, hipStream_t st);
hipError_t launch_layer0(const GemmParams& p, int act, int grid, hipStream_t st);
hipError_t launch_layer1(const GemmParams& p, int grid, hipStream_t st);
hipError_t launch_fused_layers(const GemmParams& p0, const GemmParams& p1, const FuseParams& f, int act, int grid, hipStream_t st);
hipError_t launch_combine(const CombineParams& p, hipStream_t st);
hipError_t launch_zero_u32(uint32_t* ptr, size_t n, hipStream_t st);
hipError_t launch_pack_weights(const void* B, void* out, int E, int K, int ldb, int n_tiles_n, int swiglu_F, hipStream_t st);
hipError_t launch_arrival_producer(const void* staging, void* x, const ArrivalParams& a, int n_wg, hipStream_t st);
hipError_t launch_tile_heights(const int32_t* kind, int32_t* height, int n, hipStream_t st);

}  // namespace moe
