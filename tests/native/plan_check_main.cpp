// Host-only driver for the work decomposition (plan.cpp) and the balancer (balancer.cpp),
// built by tests/test_plan_sanitized_cpu.py with -fsanitize=address,undefined: it links the
// product's planner and balancer sources as they are (no HIP involved), reads cases from
// stdin and prints what they produce, so that the Python side can check the invariants of
// the plan for any CU count and compare with the shipped library, while the sanitizers
// watch every vector access, erase and thread-local reuse of the planner.
//
//   plan <Hq> <Hkv> <D> <fp8:0|1> <n_cus> <allow_stage:0|1> <n_seqs> P0 C0 P1 C1 ...
//     -> "plan <rc> <n_items> <n_wide> <n_partials> <n_merge> <n_merge_rows> <n_stage_blocks>
//              <total_bytes> <image_bytes>", then n_items lines "i" with the 11 item fields,
//        then n_merge lines "m" with the 12 merge fields
//   split <l_in> <n_d> <l_ctxd> <n_free> <k_p> <b_p> <k_ctxp> <k_ctxd> <b_c> <n_size> <B> <n_cand>
//     -> "split <rc> <l_p> <t_prefill> <t_chunked>"
#include <cinttypes>
#include <cstdio>
#include <cstring>
#include <iostream>
#include <string>
#include <vector>

#include "cronus_internal.h"

namespace cronus {
int wide_rows_for(int, int) { return kWaves * 32; }  // the kernels' tile height (attn_mixed.hip)
}  // namespace cronus

int main() {
  std::string word;
  while (std::cin >> word) {
    if (word == "plan") {
      int hq, hkv, d, fp8, n_cus, allow_stage, n;
      std::cin >> hq >> hkv >> d >> fp8 >> n_cus >> allow_stage >> n;
      std::vector<int32_t> P((size_t)n), C((size_t)n);
      for (int i = 0; i < n; ++i) std::cin >> P[(size_t)i] >> C[(size_t)i];
      cronus_kv_cache c{};
      c.num_blocks = 1 << 30;
      c.num_q_heads = hq;
      c.num_kv_heads = hkv;
      c.head_dim = d;
      c.block_size = 16;
      c.kv_dtype = fp8 ? CRONUS_KV_FP8_E4M3 : CRONUS_KV_BF16;
      cronus::Plan plan;
      const int rc = cronus::build_plan(&c, P.data(), C.data(), n, 0x7fffffff / 16, n_cus, &plan, allow_stage != 0);
      std::printf("plan %d %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %zu %zu\n", rc,
                  rc ? 0 : plan.n_items, plan.n_wide, plan.n_partials, plan.n_merge, plan.n_merge_rows,
                  plan.n_stage_blocks, plan.total_bytes, plan.image_bytes);
      if (rc) continue;
      // an exactly sized heap buffer: a write past the image is an ASan report
      std::vector<unsigned char> image(plan.image_bytes);
      cronus::write_plan(&plan, image.data());
      const auto* wi = reinterpret_cast<const cronus::WorkItem*>(image.data() + plan.off_items);
      int queue = 0;
      for (int64_t i = 0; i < plan.n_items; ++i) {
        while (queue + 1 < cronus::kQueues && i >= plan.q_base[queue] + plan.q_len[queue]) ++queue;
        const cronus::WorkItem& w = wi[i];
        std::printf("i %d %d %d %d %d %d %d %d %d %d %d\n", w.seq, w.kv_head, w.head0, w.n_heads, w.q_tok0, w.n_tok,
                    w.kv_begin, w.kv_end, w.partial, w.wide, queue);
      }
      const auto* mi = reinterpret_cast<const cronus::MergeItem*>(image.data() + plan.off_merge);
      for (int64_t i = 0; i < plan.n_merge; ++i) {
        const cronus::MergeItem& m = mi[i];
        std::printf("m %d %d %d %d %d %d %d %d %d %d %d %d\n", m.first_partial, m.n_split, m.seq, m.kv_head, m.head0,
                    m.n_heads, m.q_tok0, m.n_tok, m.row0, m.n_rows, m.stride, m.q_off);
      }
    } else if (word == "split") {
      int64_t l_in, n_d, l_ctxd, n_free, l_p = -1;
      cronus_balancer_model m{};
      std::cin >> l_in >> n_d >> l_ctxd >> n_free >> m.k_p >> m.b_p >> m.k_ctxp >> m.k_ctxd >> m.b_c >> m.block_size >>
          m.batch_tokens >> m.n_candidates;
      double tp = 0, tc = 0;
      const int rc = cronus_balancer_split(&m, l_in, n_d, l_ctxd, n_free, &l_p, &tp, &tc);
      std::printf("split %d %" PRId64 " %.17g %.17g\n", rc, l_p, tp, tc);
    } else {
      std::fprintf(stderr, "unknown command %s\n", word.c_str());
      return 2;
    }
  }
  return 0;
}
