// Internal declarations shared by the host planner, the launchers and the kernels.
// Not part of the public ABI (that is include/cronus.h).
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "cronus.h"

namespace cronus {

constexpr int kBlock = 16;          // tokens per KV block (N_size of Algorithm 1)
constexpr int kThreads = 512;       // 8 wavefronts of 64 lanes per work-group: two per SIMD
constexpr int kWaves = 8;
constexpr int kNarrowRows = 32;     // one MFMA column tile: a decode's (token, head) rows
constexpr int kWideKvTile = 64;     // keys staged in LDS per step of a wide (chunk) tile
constexpr int kNarrowKvStep = 32 * kWaves;  // keys covered by the waves of a narrow item per step
constexpr int kQueues = 8;          // work queues of a launch: one per XCD of an MI355X (each XCD has its own L2)
constexpr int kCounterStride = 16;  // int32 between the queue heads of a set: one 64-byte line each
constexpr int kQueueSetInts = (kQueues + 1) * kCounterStride;  // a set: the heads, then the count of finished work-groups
constexpr int kQueueSets = 9;       // sets of queue heads per device: one per plan buffer of the ring, one for the static entry point

// Per-sequence record of the batch (section 4.4: one iteration = chunks + decodes).
struct SeqInfo {
  int32_t prefix_len;  // keys cached before this chunk ("length already processed", section 4.2)
  int32_t chunk_len;   // query rows of this iteration (1 = decode)
  int32_t q_off;       // index of the sequence's first row in q/out
  int32_t n_blocks;    // ceil((prefix+chunk)/16): table entries that may be read
};

// One work-group's job.
struct WorkItem {
  int32_t seq;
  int32_t kv_head;
  int32_t head0;     // first q head of the group handled here
  int32_t n_heads;   // q heads handled (all read kv_head)
  int32_t q_tok0;    // first chunk token of the tile
  int32_t n_tok;     // tokens in the tile; rows = n_tok * n_heads
  int32_t kv_begin;  // keys [kv_begin, kv_end) are processed by this item
  int32_t kv_end;
  int32_t partial;   // < 0: writes final output; else index of its (wide: first of kWaves) partial-result slot(s)
  int32_t wide;      // 1: chunk tile staged through LDS; >= 2: the same, reading the bf16 copy of an fp8
                     // sequence's K/V whose first block in the copy is wide - 2; 0: narrow (<= 32 rows),
                     // waves split keys; -1: nothing to do (a work-group's "no item left" marker)
  // copy of the sequence's record, so that a work-group needs one dependent load less
  // before it can address Q and the block table
  int32_t prefix_len, chunk_len, q_off, n_blocks;
  int32_t reserved[2];  // zero
};
static_assert(sizeof(WorkItem) == 64, "one work item = one 64-byte line");

// Rows whose partial results (split over key spans) are combined by the merge kernel:
// rows row0 .. row0 + n_rows - 1 of the tile (row r = token r / n_heads, head r % n_heads);
// span s left them in partial slot first_partial + s * stride, at slot rows 0 .. n_rows - 1.
// A narrow item fills one slot (stride 1, row0 0); a split wide tile fills kWaves slots
// per span, one per wavefront (stride kWaves, row0 = 32 * wavefront).
struct MergeItem {
  int32_t first_partial;
  int32_t n_split;
  int32_t seq;
  int32_t kv_head;
  int32_t head0;
  int32_t n_heads;
  int32_t q_tok0;
  int32_t n_tok;
  int32_t row0;
  int32_t n_rows;
  int32_t stride;
  int32_t q_off;  // the sequence's first row in q/out (copy of SeqInfo::q_off: one dependent load less)
};

// A sequence of an fp8 cache whose chunk has many tiles: its K/V blocks 0 .. n_blocks - 1 are
// converted to bf16 once per launch, into blocks blk0 .. of a copy in the workspace (same
// layout as the cache, 2 bytes per element), and its wide tiles read that copy.
struct StageSeq {
  int32_t seq;
  int32_t blk0;
  int32_t n_blocks;
  int32_t pad;
};

struct Plan {
  // sizes
  int64_t n_items = 0, n_wide = 0, n_partials = 0, n_merge = 0, n_merge_rows = 0;
  int32_t n_seqs = 0;
  int32_t wide_rows = 0;  // rows per wide tile (compile-time choice of the kernel instance)
  int32_t n_stage_seqs = 0;
  int64_t n_stage_blocks = 0;
  // The work items form kQueues queues, stored one after the other: queue x is items
  // q_base[x] .. q_base[x] + q_len[x] - 1 in the order in which they should be taken.  The
  // main kernel runs n_workgroups resident work-groups that take items from the queue of the
  // XCD they run on until it is empty, then from the others.
  int32_t q_base[kQueues] = {0}, q_len[kQueues] = {0};
  int32_t n_workgroups = 0;
  // byte offsets inside the plan image (host-built metadata that the kernels read:
  // [WorkItem x n_items | MergeItem x n_merge | StageSeq x n_stage_seqs]) and its size
  size_t off_items = 0, off_merge = 0, off_stage = 0, image_bytes = 0;
  // byte offsets inside the caller's workspace (partial results; fp8: the bf16 copy) and its size
  size_t off_partials = 0, off_stage_k = 0, off_stage_v = 0, total_bytes = 0;
};

// Number of floats of one partial slot: O[32][D], m[32], l[32].
inline size_t partial_floats(int head_dim) { return (size_t)kNarrowRows * (head_dim + 2); }

// Rows per wide tile for a head shape (must match the kernel instance that is launched).
int wide_rows_for(int head_dim, int kv_dtype);

// Builds the work decomposition (sizes and offsets into *plan; the work list itself stays
// in a per-thread scratch).  write_plan() then copies that list into host_buf, which must
// hold plan->image_bytes bytes; it must follow build_plan() on the same thread.
// allow_stage = false: an fp8 cache gets no bf16 copy (every chunk tile converts codes on
// the fly), so the workspace holds partial results only.
int build_plan(const cronus_kv_cache* cache, const int32_t* prefix_lens, const int32_t* chunk_lens,
               int32_t n_seqs, int32_t max_blocks_per_seq, int n_cus, Plan* plan, bool allow_stage = true);
void write_plan(const Plan* plan, void* host_buf);

struct AttnLaunch {
  const cronus_kv_cache* cache;
  const void* q;
  void* out;
  const int32_t* block_tables;
  int32_t max_blocks_per_seq;
  float sm_scale;
  void* workspace;  // device; holds the partial results at plan->off_partials
  const void* plan_image;  // device-visible [WorkItem | MergeItem | StageSeq] image at the plan's offsets
  const Plan* plan;
  void* stream;
  int* queue_set;  // device; this call's set of queue heads (kQueueSetInts ints, all zero between launches)
  // optional hipEvent_t handles (measurement aid): [0], [1] start and stop of the main
  // kernel's dispatch; [2] start of the call's first kernel when that is another one (the
  // fp8 copy); [3] stop of its last kernel when that is another one (the merge)
  void* ev[4];
};

// One-time set-up of the attention kernels on the current device (dynamic LDS limits);
// call before the first launch_attn() there.
int prepare_attn_kernels();
int launch_attn(const AttnLaunch& a);

// The no-allocation variant's device memory: a static array in the library's device image
// (attn_mixed.hip).  static_scratch_resolve() looks up its address on the current device
// (once per device, at set-up); static_scratch_upload() enqueues the copy of `bytes` bytes of
// host data to `dst` inside it as kernel arguments (no staging buffer, nothing allocated; the
// host data may be reused as soon as the call returns).
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
int static_scratch_resolve(void** device_ptr);
// Address, on the current device, of the library's kQueueSets sets of queue heads (a small
// static device array, zero when the library is loaded; every launch leaves its set zero).
int queue_sets_resolve(int** device_ptr);
int static_scratch_upload(void* dst, const void* host_src, size_t bytes, void* stream);
int launch_kv_append(const cronus_kv_cache* cache, const void* k_src, const void* v_src,
                     const int32_t* cu_tokens, const int32_t* start_pos, const int32_t* block_tables,
                     int32_t max_blocks_per_seq, int32_t n_seqs, int32_t n_tokens, void* stream);
int launch_kv_gather(const cronus_kv_cache* cache, void* k_dst, void* v_dst, const int32_t* cu_tokens,
                     const int32_t* start_pos, const int32_t* block_tables, int32_t max_blocks_per_seq,
                     int32_t n_seqs, int32_t n_tokens, void* stream);

// mfma_probe.hip (measurement aid)
int launch_mfma_probe(int random_operands, int iters, int n_cus, float* sink, void* stream, double* flops);
int mfma_probe_sink_floats(int n_cus);

}  // namespace cronus
