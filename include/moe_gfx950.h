/*
 * moe_gfx950 -- C ABI of the single-GPU hot path of a Mixture-of-Experts layer on MI355X (gfx950).
 *
 * One forward of the layer (paper Section 2.1, Fig. 2): every token row of the receive buffer is
 * dispatched to its topk experts, goes through the two feed-forward GEMMs of each expert
 * (layer0: [H x F], activation, layer1: [F x H]) and the topk results are reduced back into one
 * row per token.  The two producer/consumer pipelines of Section 3 (dispatch -> GroupGEMM, and
 * GroupGEMM -> top-k reduce) meet in shared tensors of M*topk rows (Fig. 4); this library runs
 * both on one GPU, with the receive buffer split into per-source segments that stand for the
 * peers of Section 3.1.2.
 *
 * Conventions
 *   - Every pointer marked "dev" is device memory on the current HIP device, owned by the caller,
 *     16-byte aligned, row-major and contiguous.  "host" pointers are ordinary host memory.
 *   - bf16 tensors are raw 16-bit patterns (upper half of an IEEE fp32).
 *   - The library owns only the plan object.  moe_layer_forward and the other enqueueing calls
 *     allocate nothing, never synchronise the host and only enqueue work on the given stream.
 *   - Every call returns a moe_status_t (0 = OK, negative = error).  Nothing throws or aborts.
 *   - Symbols: T tokens (paper's M), H embedding size (paper's N), F expert hidden size (paper's
 *     K), E experts, k = topk, R = T*k rows of the shared tensors, S source segments.
 */
#ifndef MOE_GFX950_H
#define MOE_GFX950_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_plan moe_plan_t; /* opaque, host side, owned by the library */

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = -1,        /* NULL pointer, misaligned pointer, bad enum / key / value */
  MOE_ERR_SHAPE_MISMATCH = -2,     /* call arguments disagree with the plan (e.g. act) */
  MOE_ERR_WORKSPACE_TOO_SMALL = -3,
  MOE_ERR_UNSUPPORTED = -4,        /* shape outside what the kernels handle (see moe_plan_create) */
  MOE_ERR_HIP = -5,                /* a HIP runtime call failed; hipGetLastError has the detail */
  MOE_ERR_TIMEOUT = -6             /* a bounded wait on a ready flag expired (debug spin bound only) */
} moe_status_t;

typedef enum { MOE_ACT_GELU = 0, MOE_ACT_SWIGLU = 1 } moe_act_t;

typedef struct {
  int32_t T; /* tokens in the receive buffer */
  int32_t H; /* embedding size */
  int32_t F; /* expert hidden size */
  int32_t E; /* experts held by this GPU */
  int32_t k; /* experts per token */
  int32_t S; /* source segments of the receive buffer */
  int32_t act; /* moe_act_t */
} moe_shape_t;

/* Plan / variant selection (Section 3.2.2: the division point between data-movement and GEMM
 * workgroups and the kernel variant are chosen per shape before launch and looked up at run time).
 * seg_offsets: host, [S+1], non-decreasing, seg_offsets[0] = 0, seg_offsets[S] = T; segment s is the
 * token range [seg_offsets[s], seg_offsets[s+1]) written by source s.  Copied into the plan.
 * Supported: H % 256 == 0, F % 128 == 0 (F % 256 == 0 for GELU), 1 <= k <= E <= 256, k <= 16,
 * 1 <= S <= 64, T*k < 2^24, and T*H*2 < 2^32 and T*k*F*2 < 2^32 (row offsets inside the kernels are 32-bit byte
 * offsets); anything else is MOE_ERR_UNSUPPORTED.  Touches no GPU state.  *plan is set only on success. */
int moe_plan_create(moe_plan_t **plan, const moe_shape_t *shape, const int32_t *seg_offsets);
int moe_plan_destroy(moe_plan_t *plan);

/* Tunables.  Keys:
 *   "tile_m"       64 / 128 / 256: rows of the tallest GroupGEMM tile (default: chosen from T*k/E)
 *   "n_dm"         data-movement workgroups of the layer1 kernel (default: table lookup per shape)
 *   "layer1_order" where the top-k reduction runs: 0 = a separate combine kernel after the layer1 kernel (default:
 *                  the fastest on every workload measured, see paper_2502_19811_amd/split_sweep.py);
 *                  1 = finished column panels (Fig. 6) are reduced inside the layer1 kernel, by its n_dm
 *                  data-movement workgroups and by GEMM workgroups that ran out of tiles (Section 3.2.1's
 *                  specialised blocks); 2 = in the layer1 epilogue (the vertical fusion Section 3.2.1 weighs
 *                  against them): a tile writes its rows of Y, announces each on a counter per token and column
 *                  panel, and the row that arrives last of a token's k reduces that token.  All three give the
 *                  same bits
 *   "deep_short_tiles" 1 (default): the 64-row tiles of the ragged expert ends keep five K steps of operands in
 *                  flight instead of three (six LDS stages; their A blocks are small enough).  A K step of such a tile
 *                  is 8 MFMAs per wavefront, so with three steps of lead it spends half its time waiting for its
 *                  operands.  Same bits; 0 is kept for comparison
 *   "n_prefetch"   0, 8, ... 64 (a multiple of 8): that many of the workgroups of each GroupGEMM launch compute no
 *                  tiles but run ahead of the others of their XCD and read the packed weight panels of the items
 *                  about to be handed out, "prefetch_behind" (default 16) items before to "prefetch_ahead"
 *                  (default 16) items after the head of the XCD's queue (Section 3.2.1's specialised workgroups
 *                  with local data movement to do; Section 3.2.2's division point).  Only with packed weights and
 *                  full launches; same bits.  -1 (default) = looked up from the shape: 0 on every shape measured
 *                  (there the workgroups cost their compute units and hide nothing)
 *   "layer0_order" order of the layer0 tiles: 0 = expert-major (weight reuse first); 1 = source-segment-major (Fig. 5:
 *                  M-tiles sorted by the segment they wait for, all column tiles of an M-tile in a row);
 *                  2 = waves: the S source segments are grouped into "layer0_waves" waves, the tiles are
 *                  segment-major across waves and weight-panel-major inside a wave; -1 (default) = chosen by
 *                  every forward: 0 when seg_ready is NULL, 2 when ready flags are in use
 *   "layer0_waves" 1..8 waves of order 2 (1 is order 0); 0 (default) = looked up from the shape and
 *                  "expected_ingest_gbps" (reading the option back returns the number in effect)
 *   "expected_ingest_gbps" rate in GB/s at which the caller expects the source segments to arrive (0 = unknown,
 *                  default); with the shape it selects the number of waves, by a rule condensed from the arrival
 *                  experiment (paper_2502_19811_amd/arrival_experiment.py): more waves the longer the buffer takes
 *                  to arrive against the time layer0 takes, one wave for small experts whose buffer arrives fast
 *   "spin_limit"   >0: a wait on a ready flag gives up after that many polls (about 0.3 us each) and the forward
 *                  reports MOE_ERR_TIMEOUT through moe_last_device_status; 0 = wait for ever (a flag that never
 *                  comes then hangs the GPU: the persistent kernel owns every compute unit).  Default 2^26,
 *                  about 20 s
 *   "phases"       bit mask of the steps a forward runs: 1 index build, 2 layer0, 4 layer1, 8 combine
 *                  (default 15; used to time the phases alone).  Without bit 1 the forward runs the schedules the
 *                  last index build left in the workspace again (it resets their queue heads and counters), so
 *                  the workspace must have seen a forward with bit 1 for the same routing
 *   "n_cu"         workgroups of the persistent kernels (default: compute units of the device)
 *   "profile"      1: every forward records HIP events on its stream before and after each phase
 *                  (this call then creates the events; read them with moe_plan_phase_times).  256 forwards can
 *                  be recorded between two reads; later ones are not recorded and counted in the read-only key
 *                  "profile_dropped"
 *   "block_m"      1..8: M-tiles of one expert that form a block of the default tile order; a block's items go to
 *                  one XCD (default 4: the 32 workgroups of an XCD then work on 4 M-tiles x 8 column tiles, and
 *                  two XCDs sweep the same weight panels of an expert with 8 M-tiles at the same time, the second
 *                  finding them in the Infinity Cache)
 *   "weights_packed" 1: the W1 / W2 arguments of moe_layer_forward are buffers written by moe_pack_weights
 *                  (default 0: the plain row-major weights)
 *   "fuse_layers"  1: layer0 and layer1 run in one persistent launch (the pipelining between the two GroupGEMMs of
 *                  Fig. 3/4 without a kernel boundary): a workgroup counts the layer0 tiles it finishes per M-tile,
 *                  publishes the counts every "publish_every" tiles (default 16) behind one device-wide release, and
 *                  a layer1 tile starts once all layer0 column tiles of its M-tile are published.  Same bits.  Used
 *                  with the separate combine kernel and up to 2048 M-tiles; otherwise, and by default (0), the two
 *                  launches.  Needs every workgroup of the launch resident at once: leave compute units free with
 *                  "n_cu" for anything that runs beside the forward
 *   "handoff_fences" 1: measurement aid (results unchanged): every layer0 tile ends with an agent-scope release and
 *                  every layer1 tile starts with an agent-scope acquire, the fences a tile-granular hand-off of h
 *                  between the two GroupGEMMs inside one launch would need on a part with one L2 per XCD; the time
 *                  difference against the normal run is the price of such a hand-off (default 0)
 *   "alias_experts" 1: MEASUREMENT AID, RESULTS ARE WRONG ON PURPOSE: with plain (not packed) weights every expert
 *                  reads expert 0's W1 / W2, so the weight stream of the GroupGEMMs stays cache-resident while every
 *                  other access is unchanged and in bounds; the time difference against the normal run is what
 *                  streaming the weights from HBM costs (default 0)
 *   "large_schedule" 1: build the tile schedules with the one-workgroup kernel that has no limit on the
 *                  number of M-tiles (the default picks it only above 2048 tiles); its orders are simpler
 *                  (less operand sharing inside an XCD), the results are the same bit for bit
 * Unknown key or out-of-range value: MOE_ERR_INVALID_ARG. */
int moe_plan_set_option(moe_plan_t *plan, const char *key, int64_t value);
int moe_plan_get_option(const moe_plan_t *plan, const char *key, int64_t *value);

/* Bytes of device workspace a forward needs: index arrays, tile tables, flags and counters, the
 * activation buffer h [R,F] bf16 and the layer1 shared tensor Y [R,H] bf16 (Fig. 4). */
size_t moe_plan_workspace_bytes(const moe_plan_t *plan);

/* Size in bytes of the receive (communication) buffer for M tokens of N bf16 elements: 2*M*N
 * (Section 5.5, Table 3).  This is the x argument of moe_layer_forward. */
size_t moe_receive_buffer_bytes(int64_t M, int64_t N);

/* Gate (Section 2.1): softmax over the E logits of each token, keep the k largest, renormalise
 * the kept probabilities to sum 1.  Slot 0 is the most probable expert; equal logits go to the
 * lower expert id.  logits: dev fp32 [T,E]; topk_ids: dev int32 [T,k]; topk_weights: dev fp32 [T,k]. */
int moe_route_topk(const float *logits, int32_t T, int32_t E, int32_t k, int32_t *topk_ids, float *topk_weights,
                   void *hip_stream);

/* One forward of the layer on one GPU's share (Sections 3.1-3.2):
 *   index build   row order of the shared tensor: grouped by expert, inside an expert in source
 *                 order (Section 3.1.2, Fig. 5); tile tables and tile schedules
 *   layer0        GroupGEMM over gathered rows of x, row indices held in registers (Section 4),
 *                 activation fused, h [R,F] bf16; a tile starts once the source segment of its
 *                 last row is ready
 *   layer1        GroupGEMM h x W2 -> Y [R,H]
 *   combine       out[t] = sum_j w[t,j] * Y[row of (t,j)]: by default a kernel of its own after layer1 (the
 *                 faster choice on every workload measured on one GPU); with "layer1_order" = 1 layer1 runs
 *                 column-panel-major (Fig. 6) and finished panels are reduced inside the layer1 kernel by its
 *                 data-movement workgroups and by GEMM workgroups out of tiles (Section 3.2.1, Fig. 7)
 * x: dev bf16 [T,H] receive buffer.  topk_ids: dev int32 [T,k], values in [0,E); a value outside is routed to the
 * last expert (no access leaves a buffer) and reported by moe_last_device_status as MOE_ERR_INVALID_ARG.
 * topk_weights: dev fp32 [T,k].  W1: dev bf16 [E,H,F] (GELU) or [E,H,2F] (SwiGLU: columns [0,F)
 * gate, [F,2F) up).  W2: dev bf16 [E,F,H].  out: dev bf16 [T,H], out[t] = sum_j w[t,j] * FFN_e(t,j)(x[t]).
 * workspace: dev, >= moe_plan_workspace_bytes, 256-byte aligned; its index arrays stay readable until the
 * next forward on it.  seg_ready: dev uint32 [S] or NULL; segment s counts as arrived once
 * seg_ready[s] >= ready_epoch (written by whoever fills the segment, after the data); NULL = all
 * segments are ready.  act must equal the plan's.  Inputs are not modified. */
int moe_layer_forward(moe_plan_t *plan, const void *x, const int32_t *topk_ids, const float *topk_weights,
                      const void *W1, const void *W2, int32_t act, void *out, void *workspace,
                      size_t workspace_bytes, const uint32_t *seg_ready, uint32_t ready_epoch, void *hip_stream);

/* moe_layer_forward for callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same forward, same kernels and same results
 * bit for bit, on a workspace that is a fixed 32 MiB array inside the library's device image (one copy per GPU, held
 * until the process ends).  Allocates nothing and frees nothing.  A plan whose moe_plan_workspace_bytes exceeds
 * 32 MiB (33554432 bytes) is refused with MOE_ERR_WORKSPACE_TOO_SMALL; use moe_layer_forward with a caller-owned
 * workspace for such shapes.  All calls on one GPU share that GPU's array: a forward overwrites what the previous
 * one left there (the index build of every forward resets the counters it needs), and two forwards that overlap in
 * time on one GPU -- from different streams or threads -- race.  The array is not reachable through the getters that
 * take a workspace pointer (index outputs, tile table, device status); callers that need those use moe_layer_forward.
 * Other arguments, checks and return codes as for moe_layer_forward. */
int moe_layer_forward_static(moe_plan_t *plan, const void *x, const int32_t *topk_ids, const float *topk_weights,
                             const void *W1, const void *W2, int32_t act, void *out, const uint32_t *seg_ready,
                             uint32_t ready_epoch, void *hip_stream);

/* Plan-time re-layout of the expert weights for the GroupGEMM's operand path (Section 4: the GEMM operand pipeline;
 * Section 3.2.2: whatever is decided per shape is prepared before launch).  W1 [E,H,F1] and W2 [E,F,H] (dev bf16,
 * row-major as moe_layer_forward takes them) are rewritten into W1_packed / W2_packed (dev, same number of bytes
 * as the source, 16-byte aligned, must not overlap it): per expert, column tile of 256 and step of 32 along the
 * reduction, one contiguous 16 KiB block that is the LDS image of that operand stage in the matrix-core operand
 * order, the blocks of a tile following each other.  For SwiGLU the gate and up columns of the same 128 hidden units
 * share a tile.  A forward takes the packed buffers in place of W1 / W2 once the plan option "weights_packed" is 1;
 * its results are the same bit for bit.  Either pair may be NULL (both pointers).  Enqueues on the stream; allocates
 * nothing.  Needs to be repeated only when the weights change. */
int moe_pack_weights(const moe_plan_t *plan, const void *W1, const void *W2, void *W1_packed, void *W2_packed,
                     void *hip_stream);

/* Copies the index outputs of the last forward on this workspace into caller memory (dev pointers;
 * enqueued on the stream; any of the four may be NULL):
 * expert_counts [E], expert_offsets [E+1], perm [R] (sorted row -> pair id t*k+j), inv_perm [R]. */
int moe_get_index_outputs(const moe_plan_t *plan, const void *workspace, int32_t *expert_counts,
                          int32_t *expert_offsets, int32_t *perm, int32_t *inv_perm, void *hip_stream);

/* Tile table of the GroupGEMMs as built by the last forward (dev pointers, each [max_tiles], any may be
 * NULL, entries beyond *n_tiles untouched; n_tiles: dev int32 [1]): expert, first sorted row, rows, the
 * source segment the tile waits for, and the height (64 / 128 / 256 rows) of the kernel variant that
 * computes it.  An expert's rows are cut into tiles of "tile_m" rows; the remainder goes into shorter
 * tiles so that little of a tile is padding.  max_tiles >= moe_plan_max_tiles(plan). */
int moe_get_tile_table(const moe_plan_t *plan, const void *workspace, int32_t *n_tiles, int32_t *tile_expert,
                       int32_t *tile_row0, int32_t *tile_rows, int32_t *tile_ready_seg, int32_t *tile_height,
                       void *hip_stream);
int32_t moe_plan_max_tiles(const moe_plan_t *plan);

/* The tile schedule of layer 0 or 1 as built by the last forward on this workspace (Fig. 5 / Fig. 6: the order in
 * which GroupGEMM tiles are taken), for tests of its invariants.  items: dev int32 [moe_plan_schedule_capacity(plan,
 * layer)][8] or NULL, records {m_tile, n_tile, expert, row0, nrows, height class 0/1/2, ready_seg, 0}; only the list
 * positions named by the queues are meaningful.  queues: host int32 [24]: for XCD x the list position of its first
 * item (queues[x]), its number of items (queues[8+x]) and the distance between consecutive items (queues[16+x]); a
 * workgroup on XCD x takes its own queue front to back, then the others'.  Synchronises the stream.  The plan's
 * schedule options must be the ones the forward ran with. */
int moe_get_schedule(const moe_plan_t *plan, const void *workspace, int32_t layer, int32_t *items, int32_t *queues,
                     void *hip_stream);
int64_t moe_plan_schedule_capacity(const moe_plan_t *plan, int32_t layer);

/* Stand-in for the peers on one GPU (for tests and the arrival experiment, Section 3.1.2 / Fig. 5): n_workgroups
 * workgroups (1..64) on the given stream copy the plan's source segments, in index order, from staging into the
 * receive buffer x (both dev bf16 [T,H]) at about gbytes_per_s in total (0 = unpaced), and after each segment
 * store ready_epoch into seg_ready[s] (dev uint32 [S]) with a system-scope release.  seg_counters: dev uint32 [S],
 * zero before the first call (the call leaves it zero).  Run a forward that waits on seg_ready on another stream,
 * with "n_cu" at least n_workgroups below the device's compute units so that these workgroups find room. */
int moe_play_arrival(const moe_plan_t *plan, const void *staging, void *x, uint32_t *seg_ready, uint32_t *seg_counters,
                     uint32_t ready_epoch, double gbytes_per_s, int32_t n_workgroups, void *hip_stream);

/* Average time in ms of the four phases (index build, layer0 kernel, layer1 kernel incl. fused combine,
 * stand-alone combine) over the forwards recorded since the last call (at most 256), from the events of the
 * "profile" option.  ms: host [4]; n_steps: host [1].  Waits for the recorded forwards to finish. */
int moe_plan_phase_times(moe_plan_t *plan, float *ms, int32_t *n_steps);

/* Time in ms of each forward recorded since the last moe_plan_phase_times call (first event to last event of
 * the forward; at most 256, at most capacity), for medians and percentiles.  ms: host [capacity]; n_steps: host
 * [1].  Does not reset the recording; waits for the recorded forwards to finish. */
int moe_plan_forward_times(moe_plan_t *plan, float *ms, int32_t capacity, int32_t *n_steps);

/* Measurement aids (no part of the paper's method): ceilings of the device, measured by the library's own probe
 * kernels, to read the layer's figures against.  All create and destroy two events, enqueue on the given stream
 * and wait for their own work to finish.
 * moe_probe_mfma: a register-only loop of v_mfma_f32_32x32x16_bf16, 16 accumulator blocks per wavefront, one
 *   workgroup of 4 wavefronts per compute unit, iters x 16 instructions per wavefront; random_data != 0: random bf16
 *   operands, else zeros (zeros draw less power and clock higher); random_data == 2: random operands and the same
 *   flop as 64 accumulator blocks of v_mfma_f32_16x16x32_bf16 (half the accumulator traffic per flop).  scratch: dev, at least compute units x 1 KiB
 *   (overwritten).  tflops: host [1].
 * moe_probe_copy: plain device copy of bytes (multiple of 16, both pointers 16-byte aligned) from src to dst;
 *   gbytes_per_s: host [1], bytes read plus bytes written per second.
 * moe_probe_mix: the same MFMA loop on random data with the data movement of a GroupGEMM K step around it, arranged as
 *   the GroupGEMM's main loop is, to price each kind of traffic: mode is a bit mask -- 1: 16 ds_read_b128 per K step
 *   (32 MFMAs of a wavefront) fetch the operand fragments of the next (half) step from LDS into a second register set;
 *   2: 8 global->LDS loads of 1 KiB per K step from an L2-resident region; 4: a workgroup barrier per K step; 8 (needs
 *   2): two loads in eight stream from HBM instead; 16: the MFMAs are 64 v_mfma_f32_16x16x32_bf16 per K step instead
 *   of 32 v_mfma_f32_32x32x16_bf16.  The loop runs twice (warm-up, then timed), iters K steps each.  scratch: dev,
 *   16-byte aligned, at least 4 MiB, with bit 8 at least 4 MiB x (compute units + 1); its contents are read as
 *   operands and partly overwritten.
 *   tflops: host [1].  core_ghz: host [1] or NULL: the core clock inside the loop (cycle counter over the 100 MHz
 *   device clock, mean over the workgroups), which tells a loop that runs slower because the board clocks lower from
 *   one whose matrix cores wait: busy share = tflops / (compute units x 4 x core_ghz x 1024 flop per cycle). */
int moe_probe_mix(int32_t mode, int32_t iters, void *scratch, size_t scratch_bytes, float *tflops, float *core_ghz,
                  void *hip_stream);
int moe_probe_mfma(int32_t random_data, int32_t iters, void *scratch, size_t scratch_bytes, float *tflops,
                   void *hip_stream);
int moe_probe_copy(void *dst, const void *src, size_t bytes, float *gbytes_per_s, void *hip_stream);

/* What the kernels of the last forward reported: 0, MOE_ERR_TIMEOUT when a bounded flag wait expired, or
 * MOE_ERR_INVALID_ARG when topk_ids held a value outside [0, E) (such a pair is routed to the last expert, so that
 * nothing is accessed out of bounds; the output rows of its token are then meaningless).  Synchronises the stream. */
int moe_last_device_status(const moe_plan_t *plan, const void *workspace, void *hip_stream);

const char *moe_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* MOE_GFX950_H */
