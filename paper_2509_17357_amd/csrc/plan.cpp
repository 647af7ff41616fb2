// Host-side work decomposition of one mixed iteration (Cronus section 4.4: the batch
// holds continuation chunks and decodes; Eq. 3: chunk cost grows with its prefill
// context, decode cost with the summed decode contexts).  Chunks become wide tiles of
// `wide_rows` (token, head) rows; decodes and short chunks become narrow items whose
// key range is cut into spans so that long contexts spread over the chip.
//
// This runs on the host inside every cronus_attn_mixed call, so it is written to be a
// few tens of microseconds for thousands of items: flat arrays kept per thread, no
// comparison sorts over items (narrow items are bucketed by length, the wide tiles of a
// group are generated in cost order).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "cronus_internal.h"

namespace cronus {
namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kXcds = kQueues;

struct Group {      // the wide tiles of one (sequence, KV head, head group): items [begin, end)
  int32_t begin, end;
  float cost;
};

struct Scratch {
  std::vector<SeqInfo> seqs;
  std::vector<WorkItem> wide, narrow;
  std::vector<float> wide_cost;
  std::vector<Group> groups;
  std::vector<MergeItem> merges;
  std::vector<StageSeq> stages;
  std::vector<int32_t> queue[kXcds];  // item references: >= 0 wide index, < 0 ~narrow index
  struct Tile { int32_t t0, nt, kv_total, n_split, per, first_partial; float cost_per_key; };
  std::vector<Tile> tiles;
  std::vector<int32_t> order, bucket_start;
  struct Run { int32_t begin, len; float shortest; };  // a contiguous run of one group's tiles in a queue
  std::vector<Run> runs[kXcds];
};

Scratch& scratch() {
  static thread_local Scratch s;
  return s;
}

}  // namespace

int build_plan(const cronus_kv_cache* cache, const int32_t* prefix_lens, const int32_t* chunk_lens,
               int32_t n_seqs, int32_t max_blocks_per_seq, int n_cus, Plan* plan, bool allow_stage) {
  const int D = cache->head_dim, Hq = cache->num_q_heads, Hkv = cache->num_kv_heads;
  const int G = Hq / Hkv;
  const int group = std::min(G, kNarrowRows);          // q heads handled together by one item
  const int n_groups = (G + group - 1) / group;        // > 1 only when G > 32
  const int wide_rows = wide_rows_for(D, cache->kv_dtype);
  // Tokens per wide tile.  A launch whose items would not even fill the CUs once and whose
  // tiles are too short to be cut into key spans (one chunk of a few hundred tokens with
  // little context next to a few decodes: the iteration of section 5.1 early in a request,
  // or a short whole prompt) takes half tiles, 128 rows: four of the eight waves own rows,
  // a tile's time drops by a quarter, and twice as many CUs work.
  // (Measured on MI355X: a 512-token chunk behind 1024 cached tokens 40.6 -> 29.6 us; quarter
  // tiles are slower again, and with the CUs already filled half tiles cost 1.5x the CU time.)
  constexpr int kMinPiece = 16 * kWideKvTile;  // no key span of a wide tile is shorter
  int wide_tok = std::max(1, wide_rows / group);
  {
    long long full_tiles = 0, narrow_items = 0, longest = 0;
    for (int s = 0; s < n_seqs; ++s) {
      const long long P = prefix_lens[s], C = chunk_lens[s];
      if (C <= 0 || P < 0) continue;
      if (C * group <= kNarrowRows) { narrow_items += (long long)Hkv * n_groups; continue; }
      const long long rem = C % wide_tok, full = C / wide_tok;
      const bool wide_rem = rem && rem * group > kNarrowRows;
      full_tiles += (full + wide_rem) * Hkv * n_groups;
      narrow_items += (rem && !wide_rem) ? (long long)Hkv * n_groups : 0;
      longest = std::max(longest, P + C);
    }
    // (a tile of more than 1.5 minimum spans is cut over its keys below, which serves such a launch better)
    if (full_tiles > 0 && 2 * full_tiles + narrow_items <= std::max(n_cus, 1) && longest <= kMinPiece + kMinPiece / 2 &&
        (wide_tok / 2) * group > kNarrowRows)
      wide_tok /= 2;
  }

  // keys read by narrow items, to size the spans, and the cost of the wide tiles in the
  // planner's unit (one key of a full wide tile = wide_rows / 128, one key of a narrow
  // item = 1/2), to size the spans that long wide tiles are cut into
  long long narrow_keys = 0;
  double wide_cost_total = 0;
  long long wide_tiles = 0;
  for (int s = 0; s < n_seqs; ++s) {
    const long long P = prefix_lens[s], C = chunk_lens[s];
    if (P < 0 || C < 0) return CRONUS_ERR_INVALID_ARG;
    if (P + C > (long long)max_blocks_per_seq * kBlock) return CRONUS_ERR_INVALID_ARG;
    if (C == 0) continue;
    if (C * group <= kNarrowRows) narrow_keys += (P + C) * Hkv * n_groups;
    else {
      const long long rem = C % wide_tok;
      if (rem && rem * group <= kNarrowRows) narrow_keys += (P + C) * Hkv * n_groups;
      const long long full = C / wide_tok;  // full tiles end at P + wide_tok, P + 2 wide_tok, ...
      double keys = (double)full * P + (double)wide_tok * full * (full + 1) / 2;
      if (rem && rem * group > kNarrowRows) keys += (double)(P + C) * std::max(0.25, (double)(rem * group) / wide_rows);
      wide_cost_total += keys * (wide_rows / 128.0) * Hkv * n_groups;
      wide_tiles += (full + (rem && rem * group > kNarrowRows)) * Hkv * n_groups;
    }
  }
  // no wide item should hold a CU for much longer than three quarters of a CU's fair share
  // (measured on paper-shaped iterations: smaller spans pay more for their prologue and the
  // merge than they gain in balance), and no span is shorter than 16 K/V tiles
  int wide_piece_keys = 0;
  if (wide_cost_total > 0) {
    const double fair = (wide_cost_total + 0.5 * narrow_keys) / std::max(n_cus, 1);
    const double keys = 0.75 * fair / (wide_rows / 128.0);
    wide_piece_keys = (int)std::min<double>(std::max<double>(keys, kMinPiece), 1 << 30);
    wide_piece_keys = (wide_piece_keys + kWideKvTile - 1) / kWideKvTile * kWideKvTile;
  }
  const long long target_items = std::max(n_cus, 1);  // about one span per CU: longer spans mean fewer work-group starts and fewer partial results to merge (measured: 6 % on the Llama-3-8B-shaped batch against four per CU)
  long long span = (narrow_keys + target_items - 1) / target_items;
  span = (span + kNarrowKvStep - 1) / kNarrowKvStep * kNarrowKvStep;
  constexpr int kMaxSpanSteps = 16;  // spans are 2 .. 16 steps of kNarrowKvStep keys
  span = std::min<long long>(std::max<long long>(span, 2 * kNarrowKvStep), kMaxSpanSteps * kNarrowKvStep);

  // A launch with few wide tiles (the paper's own iteration: one chunk of at most 512 tokens
  // = 64 tiles, section 5.1) lives or dies by how its spans pack onto the CUs next to the
  // decodes: 64 tiles in five spans each are 320 items for 256 CUs, two rounds where four
  // spans each need one; next to many decodes long wide items start late and end last.
  // Such a launch therefore picks its span length by estimated duration: for every way of
  // cutting the longest tile into 1 .. 8 equal spans (of at least 12 K/V tiles), the items
  // and their times under a model fitted to measured launches on MI355X (D = 128, bf16: 47
  // paper-shaped iterations of 1 k .. 64 k context with 0 .. 200 decodes of up to 1 M keys in
  // total, each with every cut that gives a distinct plan; the model's choice is the measured
  // best or within 3 % of it on all of them).  Two regimes, by the narrow items' share of the
  // work:
  //  * chunk-dominated (estimated narrow time under 0.3 of the wide tiles'): the wide items
  //    run in rounds over the CUs; the CUs that the last round leaves free take narrow items
  //    meanwhile, the narrow items left after that follow in rounds of their own.  A wide item
  //    takes 8 us + 23.7 ns per key at 256 rows (three quarters of that per key at half
  //    height), a narrow span 6 us + 12 ns per key, the merge 13 us + 3 ns per partial slot.
  //  * decode-rich: the launch cannot end before the items' times summed over the CUs, before
  //    the wide items alone have run in rounds, or before the narrow items' K/V has streamed at
  //    5.2 TB/s; the queues alternate the two kinds with the wide list running ahead, so the
  //    last wide item starts at about 0.77 of that time and the launch ends when it does.
  //    Next to streaming CUs a wide item takes 10 us + 16 ns per key (the clock is higher than
  //    under a chip-wide MFMA load), a narrow span 8 us + 6.7 ns per key, and a partial slot
  //    costs 21 ns (its traffic competes with the decodes'), the merge launch 4 us.
  if (wide_cost_total > 0 && wide_tiles <= 2LL * std::max(n_cus, 1)) {
    const int cus = std::max(n_cus, 1);
    struct Costs { double wide_us0, wide_us_key, narrow_us0, narrow_us_key, slot_us, merge_us0; };
    const Costs chunk_dominated{8.0, 0.0237, 6.0, 0.012, 0.003, 13.0}, decode_rich{10.0, 0.016, 8.0, 0.0067, 0.0206, 4.0};
    const double hbm_bytes_per_us = 5.24e6, last_wide_start = 0.77;
    constexpr int kMinCutPiece = 12 * kWideKvTile;
    long long longest = 0, n_narrow = 0;
    for (int s = 0; s < n_seqs; ++s) {
      const long long P = prefix_lens[s], C = chunk_lens[s];
      if (C <= 0) continue;
      const long long copies = (long long)Hkv * n_groups;
      if (C * group > kNarrowRows) {
        longest = std::max(longest, P + C);
        const long long rem = C % wide_tok;
        if (rem && rem * group <= kNarrowRows) n_narrow += std::max<long long>(1, (P + C + span - 1) / span) * copies;
      } else {
        n_narrow += std::max<long long>(1, (P + C + span - 1) / span) * copies;
      }
    }
    const double kv_elem_bytes = cache->kv_dtype == CRONUS_KV_FP8_E4M3 ? 1.0 : 2.0;
    const double hbm_us = (double)narrow_keys * 2.0 * D * kv_elem_bytes / hbm_bytes_per_us;  // K and V of every narrow key
    // items, summed and longest time of the wide items, and partial slots for a span length
    struct WideSide { long long items, slots; double total_us, longest_us; };
    auto wide_side = [&](int piece, const Costs& c) {
      WideSide w{0, 0, 0.0, 0.0};
      for (int s = 0; s < n_seqs; ++s) {
        const long long P = prefix_lens[s], C = chunk_lens[s];
        if (C * group <= kNarrowRows) continue;
        for (long long t0 = 0; t0 < C; t0 += wide_tok) {
          const long long nt = std::min<long long>(wide_tok, C - t0);
          if (nt * group <= kNarrowRows) continue;
          const long long kv_total = P + t0 + nt;
          long long n_split = kv_total > piece + piece / 2 ? (kv_total + piece - 1) / piece : 1;
          const long long per = ((kv_total + n_split - 1) / n_split + kWideKvTile - 1) / kWideKvTile * kWideKvTile;
          n_split = (kv_total + per - 1) / per;
          const double height = nt * group * 2 <= wide_rows ? 0.75 : 1.0;
          const double us = c.wide_us0 + c.wide_us_key * height * (double)per;
          const long long copies = (long long)Hkv * n_groups;
          w.items += n_split * copies;
          w.total_us += us * (double)(n_split * copies);
          w.longest_us = std::max(w.longest_us, us);
          if (n_split > 1) w.slots += n_split * copies * kWaves;
        }
      }
      return w;
    };
    auto narrow_item_us = [&](const Costs& c) {
      return n_narrow > 0 ? c.narrow_us0 + c.narrow_us_key * (double)narrow_keys / (double)n_narrow : 0.0;
    };
    const WideSide whole = wide_side(1 << 30, chunk_dominated);  // no tile cut
    const bool few_decodes =
        whole.items == 0 || (double)n_narrow * narrow_item_us(chunk_dominated) < 0.3 * whole.total_us;
    const Costs& c = few_decodes ? chunk_dominated : decode_rich;
    const double narrow_us = narrow_item_us(c), narrow_total_us = (double)n_narrow * narrow_us;
    double best_us = 0;
    int best_piece = 0;
    for (int cut = 1; cut <= 8; ++cut) {
      int piece = (int)((longest + cut - 1) / cut);
      piece = (piece + kWideKvTile - 1) / kWideKvTile * kWideKvTile;
      if (cut > 1 && piece < kMinCutPiece) break;
      const WideSide w = wide_side(piece, c);
      if (w.items == 0) break;
      const long long rounds = (w.items + cus - 1) / cus;
      const double mean_us = w.total_us / (double)w.items;
      const double wide_alone_us = (double)(rounds - 1) * mean_us + w.longest_us;
      // narrow items that the CUs left free by the last round of wide items take meanwhile
      auto trailing_us = [&]() {
        if (n_narrow == 0) return 0.0;
        const long long last_round = w.items - (rounds - 1) * cus;
        const long long absorbed = (cus - last_round) * (long long)(mean_us / narrow_us);
        const long long left = std::max<long long>(0, n_narrow - absorbed);
        return (double)((left + cus - 1) / cus) * narrow_us;
      };
      double us;
      if (few_decodes) {
        us = wide_alone_us + trailing_us();
      } else {
        const double floor_us = std::max(std::max((w.total_us + narrow_total_us) / cus, hbm_us), wide_alone_us);
        const double ratio = narrow_total_us / w.total_us;
        if (ratio < 0.3) us = wide_alone_us + trailing_us();
        else if (ratio <= 10.0) us = std::max(floor_us, last_wide_start * floor_us + w.longest_us);
        else us = std::max(floor_us, w.longest_us);
      }
      us += c.slot_us * (double)w.slots + (w.slots ? c.merge_us0 : 0.0);
      if (best_piece == 0 || us < best_us) {
        best_us = us;
        best_piece = piece;
      }
    }
    if (best_piece > 0) wide_piece_keys = best_piece;
  }

  Scratch& sc = scratch();
  sc.seqs.resize((size_t)n_seqs);
  sc.wide.clear();
  sc.narrow.clear();
  sc.wide_cost.clear();
  sc.groups.clear();
  sc.merges.clear();
  sc.stages.clear();
  int64_t n_partials = 0, n_merge_rows = 0, n_stage_blocks = 0;
  // fp8 cache: a chunk of many tiles reads each key of its sequence that many times; its
  // K/V is then converted to bf16 once (into the workspace) and the tiles run on the bf16
  // pipeline (measured on the chunks of the 70B-shaped batch: 7.66 -> 6.6 ms of attention).
  // (measured on 70B-shaped iterations, whole call: 16 tiles gain 5 % behind 2 k cached tokens and 14 %
  // behind 32 k; 8 tiles lose 2 % behind 2 k and gain 10 % behind 32 k)
  constexpr int kStageMinTiles = 16, kStageMinTilesLong = 8, kStageLongKeys = 8192;
  constexpr long long kStageMaxBytes = 1LL << 30;  // of workspace for the copy; later sequences convert on the fly
  const long long stage_block_bytes = 2LL * Hkv * kBlock * D * 2;  // K and V of one block, bf16
  const bool fp8 = cache->kv_dtype == CRONUS_KV_FP8_E4M3 && allow_stage;  // candidates for the bf16 copy
  int32_t q_off = 0;

  auto add_narrow = [&](int s, int kvh, int head0, int nh, int q_tok0, int n_tok, int kv_total) {
    int n_split = (int)((kv_total + span - 1) / span);
    if (n_split > 1 && kv_total - (long long)(n_split - 1) * span <= span / 4) --n_split;  // no sliver spans
    const int per = (int)(((kv_total + n_split - 1) / n_split + kNarrowKvStep - 1) / kNarrowKvStep * kNarrowKvStep);
    n_split = (kv_total + per - 1) / per;
    if (n_split > 1) {
      sc.merges.push_back(MergeItem{(int32_t)n_partials, n_split, s, kvh, head0, nh, q_tok0, n_tok, 0, n_tok * nh, 1, 0});
      n_merge_rows += (int64_t)n_tok * nh;
    }
    for (int i = 0; i < n_split; ++i) {
      WorkItem w{};
      w.seq = s; w.kv_head = kvh; w.head0 = head0; w.n_heads = nh; w.q_tok0 = q_tok0; w.n_tok = n_tok;
      w.kv_begin = i * per;
      w.kv_end = std::min(kv_total, (i + 1) * per);
      w.partial = n_split > 1 ? (int32_t)(n_partials++) : -1;
      w.wide = 0;
      sc.narrow.push_back(w);
    }
  };

  for (int s = 0; s < n_seqs; ++s) {
    const int P = prefix_lens[s], C = chunk_lens[s];
    sc.seqs[(size_t)s] = SeqInfo{P, C, q_off, (P + C + kBlock - 1) / kBlock};
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
        int32_t wide_tag = 1;
        const int seq_tiles = (C + wide_tok - 1) / wide_tok;
        if (fp8 && (seq_tiles >= kStageMinTiles || (seq_tiles >= kStageMinTilesLong && P + C >= kStageLongKeys))) {
          const int32_t nb = (P + C + kBlock - 1) / kBlock;
          const bool listed = !sc.stages.empty() && sc.stages.back().seq == s;
          if (!listed && (n_stage_blocks + nb) * stage_block_bytes <= kStageMaxBytes) {
            sc.stages.push_back(StageSeq{s, (int32_t)n_stage_blocks, nb, 0});
            n_stage_blocks += nb;
          }
          if (!sc.stages.empty() && sc.stages.back().seq == s) wide_tag = 2 + sc.stages.back().blk0;
        }
        // the tiles of this (sequence, KV head, head group), shortest first
        sc.tiles.clear();
        int max_split = 0;
        for (int t0 = 0; t0 < C; t0 += wide_tok) {
          const int nt = std::min(wide_tok, C - t0);
          if (nt * group <= kNarrowRows) {
            add_narrow(s, kvh, head0, nh, t0, nt, P + t0 + nt);
            continue;
          }
          // A tile whose keys alone would keep one CU busy for much longer than a CU's fair
          // share of the whole launch is cut into spans of whole K/V tiles;
          // each span leaves partial results (one slot per wavefront) for the merge.
          const int kv_total = P + t0 + nt;
          const float rows_frac = std::max(0.25f, (float)(nt * nh) / wide_rows);
          int n_split = 1;
          if (wide_piece_keys > 0 && kv_total > wide_piece_keys + wide_piece_keys / 2)
            n_split = (kv_total + wide_piece_keys - 1) / wide_piece_keys;
          const int per = ((kv_total + n_split - 1) / n_split + kWideKvTile - 1) / kWideKvTile * kWideKvTile;
          n_split = (kv_total + per - 1) / per;
          const int rows = nt * nh;
          int32_t first_partial = -1;
          if (n_split > 1) {
            first_partial = (int32_t)n_partials;
            for (int wv = 0; wv * kNarrowRows < rows; ++wv)
              sc.merges.push_back(MergeItem{first_partial + wv, n_split, s, kvh, head0, nh, t0, nt,
                                            wv * kNarrowRows, std::min(kNarrowRows, rows - wv * kNarrowRows), kWaves, 0});
            n_merge_rows += rows;
            n_partials += (int64_t)n_split * kWaves;
          }
          sc.tiles.push_back(Scratch::Tile{t0, nt, kv_total, n_split, per, first_partial, (wide_rows / 128.0f) * rows_frac});
          max_split = std::max(max_split, n_split);
        }
        // One group per span index: the spans i of all tiles of this (sequence, KV head) cover
        // nearly the same keys, so they are queued together (on one XCD, whose L2 then serves
        // the K/V blocks to all of them); different spans share nothing and may go elsewhere.
        for (int i = 0; i < max_split; ++i) {
          Group g{(int32_t)sc.wide.size(), 0, 0.f};
          for (const Scratch::Tile& t : sc.tiles) {
            if (i >= t.n_split) continue;
            WorkItem w{};
            w.seq = s; w.kv_head = kvh; w.head0 = head0; w.n_heads = nh; w.q_tok0 = t.t0; w.n_tok = t.nt;
            w.kv_begin = i * t.per;
            w.kv_end = std::min(t.kv_total, (i + 1) * t.per);
            w.partial = t.n_split > 1 ? t.first_partial + i * kWaves : -1;
            w.wide = wide_tag;
            const float cost = (float)(w.kv_end - w.kv_begin) * t.cost_per_key;
            sc.wide.push_back(w);
            sc.wide_cost.push_back(cost);
            g.cost += cost;
          }
          g.end = (int32_t)sc.wide.size();
          if (g.end > g.begin) sc.groups.push_back(g);
        }
      }
    }
  }

  // Order of the work.  The main kernel's work-groups stay resident (one per CU) and take
  // items from the queue of the XCD they run on, in queue order, and from the other queues
  // once their own is empty (each XCD has its own L2).  The wide tiles of one (sequence, KV
  // head, span) read the same K/V blocks, so they are queued on one XCD, back to back,
  // longest first (they were generated shortest first), where the 32 CUs of that XCD run
  // them side by side and share the blocks through its L2.  Groups go to the least loaded
  // queue, longest group first; narrow items (no reuse), longest first, even out the queues;
  // the two kinds may then be interleaved (below).
  double load[kXcds] = {0};
  for (auto& q : sc.queue) q.clear();
  for (auto& r : sc.runs) r.clear();
  auto least_loaded = [&]() {
    int x = 0;
    for (int i = 1; i < kXcds; ++i) if (load[i] < load[x]) x = i;
    return x;
  };
  std::sort(sc.groups.begin(), sc.groups.end(), [](const Group& a, const Group& b) { return a.cost > b.cost; });
  double wide_total = 0;
  for (const Group& g : sc.groups) wide_total += g.cost;
  const double piece_max = wide_total / (2 * kXcds);  // balance before locality: no piece above half a fair share
  for (const Group& g : sc.groups) {
    const int n_tiles = g.end - g.begin;
    int pieces = piece_max > 0 ? (int)(g.cost / piece_max) + 1 : 1;
    pieces = std::max(1, std::min(pieces, n_tiles));
    for (int pc = 0; pc < pieces; ++pc) {  // contiguous runs of tiles, longest keys first
      const int hi = g.end - (int)((long long)n_tiles * pc / pieces);
      const int lo = g.end - (int)((long long)n_tiles * (pc + 1) / pieces);
      const int x = least_loaded();
      sc.runs[x].push_back(Scratch::Run{(int32_t)sc.queue[x].size(), hi - lo, sc.wide_cost[(size_t)lo]});
      for (int i = hi - 1; i >= lo; --i) {
        sc.queue[x].push_back(i);
        load[x] += sc.wide_cost[(size_t)i];
      }
    }
  }
  // Within a queue the runs are taken in the order of their shortest tile, longest first: the
  // run that ends with the queue's shortest tiles comes last, so the wide items that start
  // last, and decide when the launch ends, are short ones (runs were dealt by total cost, and
  // a run of many medium tiles would otherwise precede one of few long tiles).  Measured on
  // the prefill-heavy batch: 1 % shorter launch, the other batches unchanged.
  for (int x = 0; x < kXcds; ++x) {
    auto& runs = sc.runs[x];
    if (runs.size() < 2) continue;
    std::stable_sort(runs.begin(), runs.end(), [](const Scratch::Run& a, const Scratch::Run& b) { return a.shortest > b.shortest; });
    sc.order.assign(sc.queue[x].begin(), sc.queue[x].end());
    size_t k = 0;
    for (const Scratch::Run& r : runs)
      for (int32_t j = 0; j < r.len; ++j) sc.queue[x][k++] = sc.order[(size_t)(r.begin + j)];
  }
  {  // narrow items by length, longest first: bucket sort on the number of kNarrowKvStep steps
    const size_t n = sc.narrow.size();
    sc.bucket_start.assign(kMaxSpanSteps + 2, 0);
    auto steps_of = [&](const WorkItem& w) {
      return std::min(kMaxSpanSteps, (w.kv_end - w.kv_begin + kNarrowKvStep - 1) / kNarrowKvStep);
    };
    for (const WorkItem& w : sc.narrow) ++sc.bucket_start[(size_t)(kMaxSpanSteps - steps_of(w)) + 1];
    for (int b = 0; b <= kMaxSpanSteps; ++b) sc.bucket_start[(size_t)b + 1] += sc.bucket_start[(size_t)b];
    sc.order.resize(n);
    for (size_t i = 0; i < n; ++i) sc.order[(size_t)sc.bucket_start[(size_t)(kMaxSpanSteps - steps_of(sc.narrow[i]))]++] = (int32_t)i;
    for (size_t k = 0; k < n; ++k) {
      const int32_t i = sc.order[k];
      const WorkItem& w = sc.narrow[(size_t)i];
      const int x = least_loaded();
      sc.queue[x].push_back(~i);
      load[x] += 0.5 * (w.kv_end - w.kv_begin);
    }
  }
  // Where decode spans are a large part of a queue's work but not nearly all of it (estimated
  // time at least 0.3 of its wide tiles' and at most ten times theirs), the two kinds alternate in proportion to their estimated times, each
  // kind keeping its order: while some CUs of the XCD compute wide tiles (little HBM
  // traffic), the others stream decode spans, and a CU that streams next to computing CUs
  // gets a larger share of the memory system than one that streams next to 255 others.
  // The wide list runs ahead (its share of time emitted is 1 / kWideLead of the spans'), so
  // that it is used up at about three quarters of the queue and only spans, the short
  // items, are left for the tail.  Measured on the Llama-3-8B-shaped batch: 12 % shorter
  // step than with the spans last.  Where wide tiles dominate, the spans stay at the end
  // of the queue anyway.
  constexpr double kWideLead = 0.75;
  for (auto& q : sc.queue) {
    // microseconds per item, fitted to per-work-group timestamps of the Llama-3-8B-shaped
    // batch on MI355X (D = 128, bf16; only the ratio of the two kinds matters here)
    auto time_of = [&](int32_t ref) {
      if (ref >= 0) {
        const WorkItem& w = sc.wide[(size_t)ref];
        return 5.0 + 0.0286 * (w.kv_end - w.kv_begin);
      }
      const WorkItem& w = sc.narrow[(size_t)~ref];
      return 9.6 + 0.0141 * (w.kv_end - w.kv_begin);
    };
    double total[2] = {0, 0}, done[2] = {0, 0};
    size_t n_wide_q = 0;
    for (int32_t ref : q) {
      total[ref < 0] += time_of(ref);
      n_wide_q += ref >= 0;
    }
    if (n_wide_q == 0 || n_wide_q == q.size() || total[1] < 0.3 * total[0] || total[0] < 0.1 * total[1]) continue;
    sc.order.assign(q.begin(), q.end());  // wide refs first, then narrow refs
    size_t iw = 0, in = n_wide_q, k = 0;
    while (iw < n_wide_q || in < sc.order.size()) {
      const bool take_narrow =
          iw == n_wide_q || (in < sc.order.size() && done[1] * total[0] < kWideLead * done[0] * total[1]);
      const int32_t ref = take_narrow ? sc.order[in++] : sc.order[iw++];
      done[take_narrow] += time_of(ref);
      q[k++] = ref;
    }
  }
  const size_t n_slots = sc.wide.size() + sc.narrow.size();
  {
    int32_t base = 0;
    for (int x = 0; x < kQueues; ++x) {
      plan->q_base[x] = base;
      plan->q_len[x] = (int32_t)sc.queue[x].size();
      base += plan->q_len[x];
    }
  }
  plan->n_workgroups = (int32_t)std::min<size_t>(n_slots, (size_t)std::max(n_cus, 1));

  plan->n_seqs = n_seqs;
  plan->wide_rows = wide_rows;
  plan->n_items = (int64_t)n_slots;
  plan->n_wide = (int64_t)sc.wide.size();
  plan->n_partials = n_partials;
  plan->n_merge = (int64_t)sc.merges.size();
  plan->n_merge_rows = n_merge_rows;
  plan->off_items = 0;
  plan->off_merge = align_up(plan->off_items + sizeof(WorkItem) * n_slots, 256);
  plan->n_stage_seqs = (int32_t)sc.stages.size();
  plan->n_stage_blocks = n_stage_blocks;
  plan->off_stage = align_up(plan->off_merge + sizeof(MergeItem) * sc.merges.size(), 256);
  plan->image_bytes = align_up(plan->off_stage + sizeof(StageSeq) * sc.stages.size(), 256);
  plan->off_partials = 0;
  plan->off_stage_k = align_up(plan->off_partials + sizeof(float) * partial_floats(D) * (size_t)n_partials, 256);
  const size_t stage_bytes = (size_t)n_stage_blocks * Hkv * kBlock * D * 2;  // bf16 copy of K (and of V)
  plan->off_stage_v = align_up(plan->off_stage_k + stage_bytes, 256);
  plan->total_bytes = align_up(plan->off_stage_v + stage_bytes, 256);
  if (plan->total_bytes == 0) plan->total_bytes = 256;

  return CRONUS_OK;
}

void write_plan(const Plan* plan, void* host_buf) {
  // copies the work list that the last build_plan() of this thread left in its scratch
  Scratch& sc = scratch();
  unsigned char* h = static_cast<unsigned char*>(host_buf);
  // (the per-sequence records travel inside the work and merge items; the kernels read nothing else)
  WorkItem* wi = reinterpret_cast<WorkItem*>(h + plan->off_items);
  size_t i = 0;
  for (int x = 0; x < kQueues; ++x) {
    for (const int32_t ref : sc.queue[x]) {
      WorkItem w = ref >= 0 ? sc.wide[(size_t)ref] : sc.narrow[(size_t)~ref];
      const SeqInfo& si = sc.seqs[(size_t)w.seq];
      w.prefix_len = si.prefix_len;
      w.chunk_len = si.chunk_len;
      w.q_off = si.q_off;
      w.n_blocks = si.n_blocks;
      wi[i++] = w;
    }
  }
  if (!sc.merges.empty()) {
    for (MergeItem& mi : sc.merges) mi.q_off = sc.seqs[(size_t)mi.seq].q_off;
    std::memcpy(h + plan->off_merge, sc.merges.data(), sizeof(MergeItem) * sc.merges.size());
  }
  if (!sc.stages.empty()) std::memcpy(h + plan->off_stage, sc.stages.data(), sizeof(StageSeq) * sc.stages.size());
}

}  // namespace cronus
