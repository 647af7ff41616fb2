// Host-side work decomposition of one mixed iteration (Cronus section 4.4: the batch
// holds continuation chunks and decodes; Eq. 3: chunk cost grows with its prefill
// context, decode cost with the summed decode contexts).  Chunks become wide tiles of
// `wide_rows` (token, head) rows; decodes and short chunks become narrow items whose
// key range is cut into spans so that long contexts spread over the chip.
#include <algorithm>
#include <cstring>
#include <vector>

#include "cronus_internal.h"

namespace cronus {
namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Costed {
  WorkItem item;
  double cost;
};

}  // namespace

int build_plan(const cronus_kv_cache* cache, const int32_t* prefix_lens, const int32_t* chunk_lens,
               int32_t n_seqs, int32_t max_blocks_per_seq, int n_cus, Plan* plan, void* host_buf) {
  const int D = cache->head_dim, Hq = cache->num_q_heads, Hkv = cache->num_kv_heads;
  const int G = Hq / Hkv;
  const int group = std::min(G, kNarrowRows);          // q heads handled together by one item
  const int n_groups = (G + group - 1) / group;        // > 1 only when G > 32
  const int wide_rows = wide_rows_for(D, cache->kv_dtype);
  const int wide_tok = std::max(1, wide_rows / group);  // tokens per wide tile

  // keys read by narrow items, to size the spans
  long long narrow_keys = 0;
  for (int s = 0; s < n_seqs; ++s) {
    const long long P = prefix_lens[s], C = chunk_lens[s];
    if (P < 0 || C < 0) return CRONUS_ERR_INVALID_ARG;
    if (P + C > (long long)max_blocks_per_seq * kBlock) return CRONUS_ERR_INVALID_ARG;
    if (C == 0) continue;
    if (C * group <= kNarrowRows) narrow_keys += (P + C) * Hkv * n_groups;
    else {
      const long long rem = C % wide_tok;
      if (rem && rem * group <= kNarrowRows) narrow_keys += (P + C) * Hkv * n_groups;
    }
  }
  const long long target_items = (long long)std::max(n_cus, 1) * 8;
  long long span = (narrow_keys + target_items - 1) / target_items;
  span = (span + kNarrowKvStep - 1) / kNarrowKvStep * kNarrowKvStep;
  span = std::min<long long>(std::max<long long>(span, 2 * kNarrowKvStep), 32 * kNarrowKvStep);

  std::vector<SeqInfo> seqs((size_t)n_seqs);
  std::vector<Costed> items;
  std::vector<MergeItem> merges;
  int64_t n_partials = 0, n_wide = 0, n_merge_rows = 0;
  int32_t q_off = 0;

  auto add_narrow = [&](int s, int kvh, int head0, int nh, int q_tok0, int n_tok, int kv_total) {
    int n_split = (int)((kv_total + span - 1) / span);
    if (n_split > 1 && kv_total - (long long)(n_split - 1) * span <= span / 4) --n_split;  // no sliver spans
    const int per = (int)(((kv_total + n_split - 1) / n_split + kNarrowKvStep - 1) / kNarrowKvStep * kNarrowKvStep);
    n_split = (kv_total + per - 1) / per;
    if (n_split > 1) {
      merges.push_back(MergeItem{(int32_t)n_partials, n_split, s, kvh, head0, nh, q_tok0, n_tok});
      n_merge_rows += (int64_t)n_tok * nh;
    }
    for (int i = 0; i < n_split; ++i) {
      WorkItem w{};
      w.seq = s; w.kv_head = kvh; w.head0 = head0; w.n_heads = nh; w.q_tok0 = q_tok0; w.n_tok = n_tok;
      w.kv_begin = i * per;
      w.kv_end = std::min(kv_total, (i + 1) * per);
      w.partial = n_split > 1 ? (int32_t)(n_partials++) : -1;
      w.wide = 0;
      items.push_back({w, 0.5 * (w.kv_end - w.kv_begin)});
    }
  };

  for (int s = 0; s < n_seqs; ++s) {
    const int P = prefix_lens[s], C = chunk_lens[s];
    seqs[(size_t)s] = SeqInfo{P, C, q_off, (P + C + kBlock - 1) / kBlock};
    q_off += C;
    if (C == 0) continue;
    for (int kvh = 0; kvh < Hkv; ++kvh) {
      for (int gidx = 0; gidx < n_groups; ++gidx) {
        const int head0 = kvh * G + gidx * group;
        const int nh = std::min(group, G - gidx * group);
        if (C * group <= kNarrowRows) {
          add_narrow(s, kvh, head0, nh, 0, C, P + C);
          continue;
        }
        for (int t0 = 0; t0 < C; t0 += wide_tok) {
          const int nt = std::min(wide_tok, C - t0);
          if (nt * group <= kNarrowRows) {
            add_narrow(s, kvh, head0, nh, t0, nt, P + t0 + nt);
            continue;
          }
          WorkItem w{};
          w.seq = s; w.kv_head = kvh; w.head0 = head0; w.n_heads = nh; w.q_tok0 = t0; w.n_tok = nt;
          w.kv_begin = 0;
          w.kv_end = P + t0 + nt;
          w.partial = -1;
          w.wide = 1;
          const double rows_frac = std::max(0.25, (double)(nt * nh) / wide_rows);
          items.push_back({w, (double)w.kv_end * (wide_rows / 128.0) * rows_frac});
          ++n_wide;
        }
      }
    }
  }
  // Order for the grid.  Work-group i runs on XCD i % 8 (each XCD has its own L2) and an
  // XCD takes its work-groups in index order.  All wide tiles of one (sequence, KV head)
  // read the same K/V blocks, so they are queued on one XCD, back to back, where the
  // 32 CUs of that XCD run them side by side and share the blocks through its L2.
  // Groups go to the least loaded XCD, longest first; narrow items (no reuse) even out
  // the queues.  Queues are padded to one length with idle items (wide = -1).
  constexpr int kXcds = 8;
  std::vector<std::vector<Costed>> queue(kXcds);
  double load[kXcds] = {0};
  {
    struct Group { double cost = 0; std::vector<Costed> items; };
    std::vector<Group> groups;
    std::vector<Costed> narrow;
    long long last_key = -1;
    for (const Costed& c : items) {  // wide tiles of a group were generated consecutively
      if (!c.item.wide) { narrow.push_back(c); continue; }
      const long long key = ((long long)c.item.seq * Hkv + c.item.kv_head) * 64 + (c.item.head0 % G) / group;
      if (key != last_key) { groups.emplace_back(); last_key = key; }
      groups.back().items.push_back(c);
      groups.back().cost += c.cost;
    }
    std::stable_sort(groups.begin(), groups.end(), [](const Group& a, const Group& b) { return a.cost > b.cost; });
    for (Group& g : groups) {
      int x = 0;
      for (int i = 1; i < kXcds; ++i) if (load[i] < load[x]) x = i;
      std::stable_sort(g.items.begin(), g.items.end(), [](const Costed& a, const Costed& b) { return a.cost > b.cost; });
      queue[x].insert(queue[x].end(), g.items.begin(), g.items.end());
      load[x] += g.cost;
    }
    std::stable_sort(narrow.begin(), narrow.end(), [](const Costed& a, const Costed& b) { return a.cost > b.cost; });
    for (const Costed& c : narrow) {
      int x = 0;
      for (int i = 1; i < kXcds; ++i) if (load[i] < load[x]) x = i;
      queue[x].push_back(c);
      load[x] += c.cost;
    }
  }
  size_t qlen = 0;
  for (const auto& q : queue) qlen = std::max(qlen, q.size());
  const size_t n_real_items = items.size();
  items.clear();
  if (n_real_items) {
    WorkItem idle{};
    idle.wide = -1;
    idle.partial = -1;
    for (size_t k = 0; k < qlen; ++k)
      for (int x = 0; x < kXcds; ++x) items.push_back(k < queue[x].size() ? queue[x][k] : Costed{idle, 0.0});
    while (!items.empty() && items.back().item.wide < 0) items.pop_back();  // trailing idle slots
  }

  plan->n_seqs = n_seqs;
  plan->wide_rows = wide_rows;
  plan->n_items = (int64_t)items.size();
  plan->n_wide = n_wide;
  plan->n_partials = n_partials;
  plan->n_merge = (int64_t)merges.size();
  plan->n_merge_rows = n_merge_rows;
  plan->off_seqs = 0;
  plan->off_items = align_up(plan->off_seqs + sizeof(SeqInfo) * (size_t)n_seqs, 256);
  plan->off_merge = align_up(plan->off_items + sizeof(WorkItem) * items.size(), 256);
  plan->upload_bytes = align_up(plan->off_merge + sizeof(MergeItem) * merges.size(), 256);
  plan->off_partials = plan->upload_bytes;
  plan->total_bytes = align_up(plan->off_partials + sizeof(float) * partial_floats(D) * (size_t)n_partials, 256);
  if (plan->total_bytes == 0) plan->total_bytes = 256;

  if (host_buf) {
    unsigned char* h = static_cast<unsigned char*>(host_buf);
    std::memset(h, 0, plan->upload_bytes);
    if (n_seqs) std::memcpy(h + plan->off_seqs, seqs.data(), sizeof(SeqInfo) * (size_t)n_seqs);
    WorkItem* wi = reinterpret_cast<WorkItem*>(h + plan->off_items);
    for (size_t i = 0; i < items.size(); ++i) wi[i] = items[i].item;
    if (!merges.empty()) std::memcpy(h + plan->off_merge, merges.data(), sizeof(MergeItem) * merges.size());
  }
  return CRONUS_OK;
}

}  // namespace cronus
