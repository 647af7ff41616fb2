// C ABI entry points (include/cronus.h): argument checks, plan upload, launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "cronus_internal.h"

namespace cronus {
namespace {

int check_cache(const cronus_kv_cache* c) {
  if (!c || !c->k_cache || !c->v_cache || c->num_blocks <= 0) return CRONUS_ERR_INVALID_ARG;
  if (c->num_q_heads <= 0 || c->num_kv_heads <= 0) return CRONUS_ERR_INVALID_ARG;
  if (c->block_size != kBlock) return CRONUS_ERR_UNSUPPORTED;
  if (c->head_dim != 64 && c->head_dim != 128) return CRONUS_ERR_UNSUPPORTED;
  if (c->num_q_heads % c->num_kv_heads) return CRONUS_ERR_UNSUPPORTED;
  if (c->kv_dtype == CRONUS_KV_BF16) {
    if (c->k_scale || c->v_scale) return CRONUS_ERR_INVALID_ARG;
  } else if (c->kv_dtype == CRONUS_KV_FP8_E4M3) {
    if (!c->k_scale || !c->v_scale) return CRONUS_ERR_INVALID_ARG;
  } else {
    return CRONUS_ERR_UNSUPPORTED;
  }
  return CRONUS_OK;
}

// Shape-only variant for the size queries, which need no device pointers.
int check_shape(const cronus_kv_cache* c) {
  if (!c || c->num_q_heads <= 0 || c->num_kv_heads <= 0) return CRONUS_ERR_INVALID_ARG;
  if (c->block_size != kBlock) return CRONUS_ERR_UNSUPPORTED;
  if (c->head_dim != 64 && c->head_dim != 128) return CRONUS_ERR_UNSUPPORTED;
  if (c->num_q_heads % c->num_kv_heads) return CRONUS_ERR_UNSUPPORTED;
  if (c->kv_dtype != CRONUS_KV_BF16 && c->kv_dtype != CRONUS_KV_FP8_E4M3) return CRONUS_ERR_UNSUPPORTED;
  return CRONUS_OK;
}

// Per-device facts and one-time set-up, guarded by g_mu.  Index = HIP device ordinal.
struct DeviceState {
  int n_cus = 0;           // 0: not queried yet
  bool kernels_ready = false;
  void* static_scratch = nullptr;  // this device's address of the library's static scratch array
  int* queue_sets = nullptr;       // and of its sets of queue heads
};
constexpr int kMaxDevices = 64;
DeviceState g_dev[kMaxDevices];
std::mutex g_mu;

// CU count of the current device; 256 (MI355X) when sizes are queried without a device.
int device_cus() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return 256;
  }
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_dev[dev].n_cus) return g_dev[dev].n_cus;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
    (void)hipGetLastError();
    return 256;
  }
  g_dev[dev].n_cus = n;
  return n;
}

// Set-up that must precede the first launch on the current device (kernel attributes).
// Caller holds g_mu.
int prepare_device_locked(int* device) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CRONUS_ERR_HIP;
  *device = dev;
  if (!g_dev[dev].kernels_ready) {
    if (int rc = prepare_attn_kernels()) return rc;
    if (int rc = static_scratch_resolve(&g_dev[dev].static_scratch)) return rc;
    if (int rc = queue_sets_resolve(&g_dev[dev].queue_sets)) return rc;
    g_dev[dev].kernels_ready = true;
  }
  return CRONUS_OK;
}

// The work list is written into pinned, device-mapped host memory and the kernels read it
// from there (each work-group one 64-byte item; the merge kernel its record): no copy
// sits between the caller's previous work on the stream and the attention kernel (a
// stream-ordered copy of these few KB took about 25 us of otherwise idle stream time on
// MI355X).  A slot is reused only after the kernels of the call that used it finished.
struct Slot {
  void* host = nullptr;
  void* dev = nullptr;   // the same memory as the device sees it
  size_t cap = 0;
  hipEvent_t done = nullptr;
  bool pending = false;
};
void* g_ev[4] = {nullptr, nullptr, nullptr, nullptr};

constexpr int kSlots = 8;
static_assert(kQueueSets == kSlots + 1, "one set of queue heads per plan buffer, one for the static entry point");
Slot g_slots[kMaxDevices][kSlots];  // a ring per device: the events that guard reuse belong to a device
int g_next[kMaxDevices] = {0};

Slot* acquire_slot(int dev, size_t bytes) {
  Slot* s = &g_slots[dev][g_next[dev]];
  g_next[dev] = (g_next[dev] + 1) % kSlots;
  if (s->pending) {
    if (hipEventSynchronize(s->done) != hipSuccess) return nullptr;
    s->pending = false;
  }
  if (s->cap < bytes) {
    if (s->host) (void)hipHostFree(s->host);
    s->host = s->dev = nullptr;
    s->cap = 0;
    size_t cap = 1 << 16;
    while (cap < bytes) cap <<= 1;
    if (hipHostMalloc(&s->host, cap, hipHostMallocMapped | hipHostMallocPortable) != hipSuccess) return nullptr;
    if (hipHostGetDevicePointer(&s->dev, s->host, 0) != hipSuccess) {
      (void)hipHostFree(s->host);
      s->host = nullptr;
      return nullptr;
    }
    s->cap = cap;
  }
  if (!s->done && hipEventCreateWithFlags(&s->done, hipEventDisableTiming) != hipSuccess) return nullptr;
  return s;
}

}  // namespace
}  // namespace cronus

using namespace cronus;

extern "C" {

int cronus_kv_append(const cronus_kv_cache* cache, const void* k_src, const void* v_src,
                     const int32_t* cu_tokens, const int32_t* start_pos, const int32_t* block_tables,
                     int32_t max_blocks_per_seq, int32_t n_seqs, int32_t n_tokens, void* hip_stream) {
  if (int rc = check_cache(cache)) return rc;
  if (n_seqs < 0 || n_tokens < 0 || max_blocks_per_seq <= 0) return CRONUS_ERR_INVALID_ARG;
  if (n_tokens == 0 || n_seqs == 0) return CRONUS_OK;
  if (!k_src || !v_src || !cu_tokens || !start_pos || !block_tables) return CRONUS_ERR_INVALID_ARG;
  return launch_kv_append(cache, k_src, v_src, cu_tokens, start_pos, block_tables, max_blocks_per_seq, n_seqs,
                          n_tokens, hip_stream);
}

int cronus_kv_gather(const cronus_kv_cache* cache, void* k_dst, void* v_dst, const int32_t* cu_tokens,
                     const int32_t* start_pos, const int32_t* block_tables, int32_t max_blocks_per_seq,
                     int32_t n_seqs, int32_t n_tokens, void* hip_stream) {
  if (int rc = check_cache(cache)) return rc;
  if (n_seqs < 0 || n_tokens < 0 || max_blocks_per_seq <= 0) return CRONUS_ERR_INVALID_ARG;
  if (n_tokens == 0 || n_seqs == 0) return CRONUS_OK;
  if (!k_dst || !v_dst || !cu_tokens || !start_pos || !block_tables) return CRONUS_ERR_INVALID_ARG;
  return launch_kv_gather(cache, k_dst, v_dst, cu_tokens, start_pos, block_tables, max_blocks_per_seq, n_seqs,
                          n_tokens, hip_stream);
}

size_t cronus_probe_mfma_sink_floats(void) { return (size_t)mfma_probe_sink_floats(device_cus()); }

int cronus_probe_mfma(int random_operands, int iters, float* sink, size_t sink_floats, void* hip_stream,
                      double* flops_host) {
  if (iters < 1 || iters > (1 << 20) || !sink || !flops_host) return CRONUS_ERR_INVALID_ARG;
  const int n_cus = device_cus();
  if (sink_floats < (size_t)mfma_probe_sink_floats(n_cus)) return CRONUS_ERR_WORKSPACE;
  return launch_mfma_probe(random_operands, iters, n_cus, sink, hip_stream, flops_host);
}

size_t cronus_attn_mixed_workspace_bytes(const cronus_kv_cache* cache, const int32_t* prefix_lens,
                                         const int32_t* chunk_lens, int32_t n_seqs) {
  if (check_shape(cache) || n_seqs < 0 || (n_seqs > 0 && (!prefix_lens || !chunk_lens))) return 0;
  Plan plan;
  if (build_plan(cache, prefix_lens, chunk_lens, n_seqs, 0x7fffffff / kBlock, device_cus(), &plan)) return 0;
  return plan.total_bytes;
}

int cronus_attn_mixed_plan_stats(const cronus_kv_cache* cache, const int32_t* prefix_lens,
                                 const int32_t* chunk_lens, int32_t n_seqs, int64_t* stats) {
  if (int rc = check_shape(cache)) return rc;
  if (!stats || n_seqs < 0 || (n_seqs > 0 && (!prefix_lens || !chunk_lens))) return CRONUS_ERR_INVALID_ARG;
  Plan plan;
  if (int rc = build_plan(cache, prefix_lens, chunk_lens, n_seqs, 0x7fffffff / kBlock, device_cus(), &plan))
    return rc;
  stats[0] = plan.n_items;
  stats[1] = plan.n_wide;
  stats[2] = plan.n_partials;
  stats[3] = plan.n_merge_rows;
  stats[4] = plan.n_merge;
  stats[5] = plan.n_stage_blocks;
  return CRONUS_OK;
}

int64_t cronus_attn_mixed_plan_items(const cronus_kv_cache* cache, const int32_t* prefix_lens,
                                     const int32_t* chunk_lens, int32_t n_seqs, int32_t* items, int64_t capacity) {
  if (int rc = check_shape(cache)) return -rc;
  if (n_seqs < 0 || capacity < 0 || (n_seqs > 0 && (!prefix_lens || !chunk_lens)) || (capacity > 0 && !items))
    return -CRONUS_ERR_INVALID_ARG;
  Plan plan;
  if (int rc = build_plan(cache, prefix_lens, chunk_lens, n_seqs, 0x7fffffff / kBlock, device_cus(), &plan)) return -rc;
  std::vector<unsigned char> buf(plan.image_bytes);
  write_plan(&plan, buf.data());
  const int64_t n = std::min<int64_t>(capacity, plan.n_items);
  const WorkItem* wi = reinterpret_cast<const WorkItem*>(buf.data() + plan.off_items);
  int queue = 0;
  for (int64_t i = 0; i < n; ++i) {
    while (queue + 1 < kQueues && i >= plan.q_base[queue] + plan.q_len[queue]) ++queue;
    const WorkItem& w = wi[i];
    const int32_t row[11] = {w.seq, w.kv_head, w.head0, w.n_heads, w.q_tok0, w.n_tok, w.kv_begin, w.kv_end,
                             w.partial, w.wide, queue};
    std::memcpy(items + 11 * i, row, sizeof(row));
  }
  return plan.n_items;
}

namespace {

// Host-side checks shared by the two attention entry points; *total_q = sum of chunk_lens.
int check_attn_args(const cronus_kv_cache* cache, const void* q, const void* out, const int32_t* prefix_lens,
                    const int32_t* chunk_lens, const int32_t* block_tables, int32_t max_blocks_per_seq,
                    int32_t n_seqs, float sm_scale, long long* total_q) {
  *total_q = 0;
  if (int rc = check_cache(cache)) return rc;
  if (n_seqs < 0 || max_blocks_per_seq <= 0) return CRONUS_ERR_INVALID_ARG;
  if (!(sm_scale > 0.f) || !std::isfinite(sm_scale)) return CRONUS_ERR_INVALID_ARG;
  if (n_seqs == 0) return CRONUS_OK;
  if (!prefix_lens || !chunk_lens || !block_tables) return CRONUS_ERR_INVALID_ARG;
  long long total = 0;
  for (int s = 0; s < n_seqs; ++s) {
    if (chunk_lens[s] < 0 || prefix_lens[s] < 0) return CRONUS_ERR_INVALID_ARG;
    total += chunk_lens[s];
  }
  if (total > 0 && (total > 0x7fffffffLL || !q || !out)) return CRONUS_ERR_INVALID_ARG;
  *total_q = total;
  return CRONUS_OK;
}

}  // namespace

int cronus_attn_mixed(const cronus_kv_cache* cache, const void* q, void* out, const int32_t* prefix_lens,
                      const int32_t* chunk_lens, const int32_t* block_tables, int32_t max_blocks_per_seq,
                      int32_t n_seqs, float sm_scale, void* workspace, size_t workspace_bytes, void* hip_stream) {
  long long total_q = 0;
  if (int rc = check_attn_args(cache, q, out, prefix_lens, chunk_lens, block_tables, max_blocks_per_seq, n_seqs,
                               sm_scale, &total_q))
    return rc;
  if (total_q == 0) return CRONUS_OK;

  Plan plan;
  const int n_cus = device_cus();
  if (int rc = build_plan(cache, prefix_lens, chunk_lens, n_seqs, max_blocks_per_seq, n_cus, &plan)) return rc;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return CRONUS_ERR_WORKSPACE;
  if (workspace_bytes < plan.total_bytes) return CRONUS_ERR_WORKSPACE;
  if (plan.n_items > 0x7fffffffLL) return CRONUS_ERR_INVALID_ARG;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  std::lock_guard<std::mutex> lock(g_mu);
  // everything that can fail without a launch comes first: kernel attributes, the plan buffer
  int dev = 0;
  if (int rc = prepare_device_locked(&dev)) return rc;
  Slot* slot = acquire_slot(dev, plan.image_bytes);
  if (!slot) return CRONUS_ERR_HIP;
  write_plan(&plan, slot->host);
  // the set of queue heads that belongs to this plan buffer: free again when the buffer is
  const int set = (int)(slot - g_slots[dev]);
  AttnLaunch a{cache, q, out, block_tables, max_blocks_per_seq, sm_scale, workspace, slot->dev, &plan, hip_stream,
               g_dev[dev].queue_sets + set * kQueueSetInts, {g_ev[0], g_ev[1], g_ev[2], g_ev[3]}};
  const int rc = launch_attn(a);
  // whatever was launched may still read the slot
  if (hipEventRecord(slot->done, stream) != hipSuccess) return CRONUS_ERR_HIP;
  slot->pending = true;
  return rc;
}

int cronus_attn_mixed_static(const cronus_kv_cache* cache, const void* q, void* out, const int32_t* prefix_lens,
                             const int32_t* chunk_lens, const int32_t* block_tables, int32_t max_blocks_per_seq,
                             int32_t n_seqs, float sm_scale, void* hip_stream) {
  long long total_q = 0;
  if (int rc = check_attn_args(cache, q, out, prefix_lens, chunk_lens, block_tables, max_blocks_per_seq, n_seqs,
                               sm_scale, &total_q))
    return rc;
  if (total_q == 0) return CRONUS_OK;

  // no bf16 copy of fp8 sequences here: it can take a gigabyte; their chunk tiles convert on the fly
  Plan plan;
  if (int rc = build_plan(cache, prefix_lens, chunk_lens, n_seqs, max_blocks_per_seq, device_cus(), &plan, false))
    return rc;
  if (plan.n_items > 0x7fffffffLL) return CRONUS_ERR_INVALID_ARG;
  // scratch layout: [plan image | partial results]; both sizes are multiples of 256
  if (plan.image_bytes > kStaticScratchBytes || plan.total_bytes > kStaticScratchBytes - plan.image_bytes)
    return CRONUS_ERR_WORKSPACE;

  std::lock_guard<std::mutex> lock(g_mu);
  int dev = 0;
  if (int rc = prepare_device_locked(&dev)) return rc;  // first call on a device: looks up its scratch address
  unsigned char* base = static_cast<unsigned char*>(g_dev[dev].static_scratch);
  static thread_local std::vector<unsigned char> image;  // host memory; grows to the largest plan seen
  image.resize(plan.image_bytes);
  write_plan(&plan, image.data());
  if (int rc = static_scratch_upload(base, image.data(), plan.image_bytes, hip_stream)) return rc;
  // Nothing in the scratch has to start at zero: the kernels read the plan image that was just
  // stored and, of the partial slots, exactly the rows that items of this call write first.
  // (The heads of the work queues, which must, live in their own small array, and every
  // launch leaves them zero.)
  AttnLaunch a{cache, q, out, block_tables, max_blocks_per_seq, sm_scale, base + plan.image_bytes, base, &plan,
               hip_stream, g_dev[dev].queue_sets + kSlots * kQueueSetInts, {g_ev[0], g_ev[1], g_ev[2], g_ev[3]}};
  return launch_attn(a);
}

void cronus_profile_events(void* main_start, void* main_stop, void* first_start, void* last_stop) {
  std::lock_guard<std::mutex> lock(g_mu);
  g_ev[0] = main_start;
  g_ev[1] = main_stop;
  g_ev[2] = first_start;
  g_ev[3] = last_stop;
}

const char* cronus_status_string(int status) {
  switch (status) {
    case CRONUS_OK: return "ok";
    case CRONUS_ERR_INVALID_ARG: return "invalid argument";
    case CRONUS_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case CRONUS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case CRONUS_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int cronus_version(void) { return 504; }  // 0.5.4: resident work-groups with work queues; plan items carry their queue; MFMA probe

}  // extern "C"
