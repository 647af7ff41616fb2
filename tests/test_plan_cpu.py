"""The host-side work decomposition (no GPU): every (sequence, q head, chunk token)
must be covered by exactly one chain of items whose key ranges partition [0, prefix +
token + 1) up to the tile's own causal end, spans must be aligned to what the kernel
assumes, and the items must be listed queue by queue."""
import numpy as np
import pytest

from paper_2509_17357_amd import binding as B
from paper_2509_17357_amd import workloads as W

F = {n: i for i, n in enumerate(B.PLAN_ITEM_FIELDS)}


def plan_for(shape, P, C):
    c = B.make_cache(0, 0, 1 << 20, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                     B.CRONUS_KV_FP8_E4M3 if shape.kv_dtype == "fp8" else B.CRONUS_KV_BF16)
    items = B.cronus_attn_mixed_plan_items(c, P, C)
    stats = B.cronus_attn_mixed_plan_stats(c, P, C)
    return items, stats


def check_plan(shape, P, C):
    P, C = np.asarray(P), np.asarray(C)
    items, stats = plan_for(shape, P, C)
    assert len(items) == stats["items"]
    verify_items(shape, P, C, items, stats)
    return items, stats


def verify_items(shape, P, C, items, stats):
    """The invariants of a work list (whatever planner options or CU count produced it)."""
    G = shape.n_q_heads // shape.n_kv_heads
    real = items
    assert (items[:, F["wide"]] >= 0).all()                       # every listed item is work
    assert (np.diff(items[:, F["queue"]]) >= 0).all() and items[:, F["queue"]].min(initial=0) >= 0 \
        and items[:, F["queue"]].max(initial=0) <= 7                # queue by queue
    assert (real[:, F["wide"]] >= 1).sum() == stats["wide_items"]
    # coverage[s][head, token] = list of (kv_begin, kv_end, partial)
    cover = {}
    tiles = []
    for it in real:
        s, kvh, h0, nh, t0, nt, kb, ke, part, wide = (int(x) for x in it[:10])
        tiles.append((s, kvh, h0, nh, t0, nt, kb, ke, part, wide))
    for s, kvh, h0, nh, t0, nt, kb, ke, part, wide in tiles:
        assert 0 <= s < len(P) and C[s] > 0 and 0 <= kvh < shape.n_kv_heads
        assert h0 // G == kvh and (h0 + nh - 1) // G == kvh and nh >= 1   # heads of one KV head
        assert 0 <= t0 and nt >= 1 and t0 + nt <= C[s]
        assert nt * nh <= (256 if wide else 32)
        if wide:
            assert kb % 64 == 0 and kb < ke <= P[s] + t0 + nt   # whole K/V tiles of 64 keys
        else:
            assert kb % 256 == 0 and kb < ke <= P[s] + t0 + nt
        for h in range(h0, h0 + nh):
            for t in range(t0, t0 + nt):
                cover.setdefault((s, h, t), []).append((kb, ke, part, t0 + nt))
    n_partial = 0
    for s in range(len(P)):
        for h in range(shape.n_q_heads):
            for t in range(int(C[s])):
                spans = sorted(cover.pop((s, h, t)))
                tile_end = spans[0][3]
                assert spans[0][0] == 0 and spans[-1][1] == P[s] + tile_end   # whole visible range of the tile
                for a, b in zip(spans, spans[1:]):
                    assert a[1] == b[0]                                        # no gap, no overlap
                if len(spans) > 1:
                    assert all(sp[2] >= 0 for sp in spans)                     # merged through partial slots
                else:
                    assert spans[0][2] == -1
    assert not cover
    # each partial slot belongs to one item: a narrow item owns one, a split wide tile one per wavefront
    slots = []
    for it in real[real[:, F["partial"]] >= 0]:
        slots += list(range(int(it[F["partial"]]), int(it[F["partial"]]) + (8 if it[F["wide"]] >= 1 else 1)))
    assert sorted(slots) == list(range(stats["partials"]))


@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_plan_covers_benchmark_batches(cid):
    b = W.draw_batch(cid, scale=1.0 if cid in (1, 2) else 0.25)
    check_plan(b.shape, b.prefix_lens, b.chunk_lens)


def test_plan_edge_cases():
    sh = W.SHAPE_8B
    check_plan(sh, [0], [1])                       # a single key
    check_plan(sh, [0, 5, 0], [0, 0, 3])           # empty sequences are skipped
    check_plan(sh, [100000], [1])                  # long decode: many spans
    check_plan(sh, [7], [65])                      # one wide tile and a one-token narrow tail
    check_plan(W.HeadShape(28, 4, 128), [10, 129, 0], [50, 1, 260])   # G = 7
    check_plan(W.HeadShape(64, 1, 128), [33], [40])                    # G = 64 > 32: two head groups
    check_plan(W.HeadShape(4, 4, 64), [5, 0, 63], [40, 200, 1])        # MHA
    items, stats = plan_for(sh, [], [])
    assert stats["items"] == 0 and len(items) == 0


def test_plan_queues_follow_xcd_order():
    """One queue per XCD: the wide tiles of one (sequence, KV head) sit in few queues, and
    within a queue they come longest first."""
    b = W.draw_batch(3)
    items, _ = plan_for(b.shape, b.prefix_lens, b.chunk_lens)
    wide = [(int(it[F["queue"]]) % 8, it) for it in items if it[F["wide"]] >= 1]
    queues_of = {}
    for x, it in wide:
        queues_of.setdefault((int(it[F["seq"]]), int(it[F["kv_head"]])), set()).add(x)
    assert max(len(v) for v in queues_of.values()) <= 2
    for x in range(8):
        last = {}
        for xx, it in wide:
            if xx != x or it[F["kv_begin"]] > 0:
                continue
            key = (int(it[F["seq"]]), int(it[F["kv_head"]]))
            if key in last:
                assert it[F["q_tok0"]] < last[key]        # the latest tile (the most keys) first
            last[key] = int(it[F["q_tok0"]])
    # a queue's runs (tiles of one (sequence, KV head), back to back) come in the order of their
    # shortest tile, longest first: the wide items that start last are the queue's shortest
    for x in range(8):
        runs = []   # [key, fewest keys of the run]
        for xx, it in wide:
            if xx != x:
                continue
            key = (int(it[F["seq"]]), int(it[F["kv_head"]]))
            n_keys = int(it[F["kv_end"]] - it[F["kv_begin"]])
            if runs and runs[-1][0] == key:
                runs[-1][1] = min(runs[-1][1], n_keys)
            else:
                runs.append([key, n_keys])
        assert len(runs) >= 2
        shortest = [r[1] for r in runs]
        assert shortest == sorted(shortest, reverse=True), shortest
    # the eight queues carry similar amounts of work
    load = np.zeros(8)
    for it in items:
        if it[F["wide"]] >= 1:
            load[it[F["queue"]] % 8] += 2.0 * (it[F["kv_end"]] - it[F["kv_begin"]])
        elif it[F["wide"]] == 0:
            load[it[F["queue"]] % 8] += 0.5 * (it[F["kv_end"]] - it[F["kv_begin"]])
    assert load.max() <= 1.1 * load.mean()


def test_few_long_wide_tiles_are_split_over_keys():
    """A paper-shaped iteration (one chunk of at most 512 tokens against a long prefix) has
    only 64 wide tiles for 256 CUs: each is cut into key spans so that every CU gets work,
    while a batch with many tiles per CU is left alone."""
    sh = W.SHAPE_8B
    items, stats = check_plan(sh, [32768] + [999] * 16, [496] + [1] * 16)
    wide = items[items[:, F["wide"]] >= 1]
    tiles = {(int(i[F["kv_head"]]), int(i[F["q_tok0"]])) for i in wide}
    assert len(tiles) == 8 * 8 and len(wide) >= 4 * len(tiles)
    span = wide[:, F["kv_end"]] - wide[:, F["kv_begin"]]
    assert span.max() <= 2 * span[span > 256].min() + 64   # spans of one size, up to the tail
    b = W.draw_batch(3)
    items3, _ = plan_for(b.shape, b.prefix_lens, b.chunk_lens)
    w3 = items3[items3[:, F["wide"]] >= 1]
    assert (w3[:, F["kv_begin"]] == 0).all() and (w3[:, F["partial"]] == -1).all()


def test_whole_prompts_with_many_tiles_per_cu():
    """Whole prompts (prefix 0) with 16 tiles per CU: one item per tile, none cut into spans;
    a (sequence, KV head)'s tiles sit in one run, longest first."""
    sh = W.HeadShape(32, 8, 128)
    P, C = [0] * 8, [4096] * 8                      # 8 x 64 tiles x 8 KV heads = 4096 tiles, 16 per CU
    items, stats = plan_for(sh, P, C)
    wide = items[items[:, F["wide"]] >= 1]
    assert stats["wide_items"] == 4096 and len(wide) == 4096 == len(items)
    assert (wide[:, F["partial"]] == -1).all() and (wide[:, F["kv_begin"]] == 0).all()
    key = (wide[:, F["seq"]] * 8 + wide[:, F["kv_head"]]) * 64 + wide[:, F["q_tok0"]] // 64
    assert len(np.unique(key)) == 4096
    assert (wide[:, F["kv_end"]] == wide[:, F["q_tok0"]] + wide[:, F["n_tok"]]).all()
    check_plan(sh, [0] * 16, [64 * 33] * 16)


def test_small_launches_take_half_tiles():
    """A launch that cannot fill the CUs once, with tiles too short for key spans, uses
    tiles of 128 rows; with more decodes, more chunks or a long context it keeps 256."""
    sh = W.SHAPE_8B
    tok = lambda items: set(int(n) for n in items[items[:, F["wide"]] >= 1][:, F["n_tok"]])
    items, _ = check_plan(sh, [1024] + [999] * 8, [512] + [1] * 8)      # 2*64 + 64 items <= 256 CUs
    assert tok(items) == {32}
    items, _ = check_plan(sh, [0], [1010])                               # a short whole prompt, ragged end
    assert tok(items) == {32, 18}
    items, _ = check_plan(sh, [1024] + [999] * 32, [512] + [1] * 32)    # 2*64 + 256 items: CUs are busy anyway
    assert tok(items) == {64}
    items, _ = check_plan(sh, [1024] * 3, [512] * 3)                    # 192 full tiles
    assert tok(items) == {64}
    items, stats = check_plan(sh, [2048], [512])                         # tiles long enough for two key spans
    assert tok(items) == {64} and stats["partials"] > 0
    items, stats = check_plan(sh, [16384], [512])                        # long context: key spans instead
    assert tok(items) == {64} and stats["partials"] > 0
    items, _ = check_plan(W.HeadShape(64, 8, 128, "fp8"), [300], [200])  # G = 8: 16-token half tiles
    assert tok(items) == {16, 8}


def test_fp8_chunks_of_many_tiles_read_a_bf16_copy():
    """fp8 cache: a sequence whose chunk has 16 or more tiles gets blocks in the launch's bf16
    copy (wide = 2 + its first block there, blocks dealt in batch order); shorter chunks,
    decodes and bf16 caches do not; the workspace grows by the copy."""
    sh = W.HeadShape(64, 8, 128, "fp8")                      # G = 8: 32 tokens per tile
    P, C = [1000, 0, 5000, 77, 40], [600, 100, 513, 1, 2048]
    items, stats = check_plan(sh, P, C)
    wide = items[items[:, F["wide"]] >= 1]
    by_seq = {s: set(int(w) for w in wide[wide[:, F["seq"]] == s][:, F["wide"]]) for s in range(5)}
    blocks = lambda s: (P[s] + C[s] + 15) // 16
    assert by_seq[0] == {2}                                   # 19 tiles: first in the copy
    assert by_seq[1] == {1}                                   # 4 tiles: staged through registers
    assert by_seq[2] == {2 + blocks(0)}                       # 17 tiles (the last one partial)
    assert by_seq[3] == set()                                 # a decode
    assert by_seq[4] == {2 + blocks(0) + blocks(2)}
    c = B.make_cache(0, 0, 1 << 20, 64, 8, 128, B.CRONUS_KV_FP8_E4M3)
    need = B.cronus_attn_mixed_workspace_bytes(c, P, C)
    copy_bytes = 2 * (blocks(0) + blocks(2) + blocks(4)) * 8 * 16 * 128 * 2
    assert need >= copy_bytes and need < copy_bytes + (64 << 20)
    # the same lengths on a bf16 cache: nothing is copied
    items, _ = check_plan(W.HeadShape(64, 8, 128), P, C)
    assert set(int(w) for w in items[:, F["wide"]]) <= {-1, 0, 1}
    cb = B.make_cache(0, 0, 1 << 20, 64, 8, 128)
    assert B.cronus_attn_mixed_workspace_bytes(cb, P, C) < copy_bytes
    # the copy is bounded (1 GiB of workspace): sequences past the bound convert on the fly
    P, C = [200000, 200000, 100], [1024, 1024, 1024]
    items, _ = plan_for(sh, P, C)
    wide = items[items[:, F["wide"]] >= 1]
    tags = [set(int(w) for w in wide[wide[:, F["seq"]] == s][:, F["wide"]]) for s in range(3)]
    assert tags[0] == {2} and tags[1] == {1} and tags[2] == {2 + (200000 + 1024 + 15) // 16}
    assert B.cronus_attn_mixed_workspace_bytes(c, P, C) < (1 << 30) + (256 << 20)


@pytest.mark.parametrize("seed", range(12))
def test_plan_random_batches_cover_every_row_once(seed):
    """Seeded random batches over head shapes, cache types and length mixes (empty sequences,
    decodes, short and long chunks, long prefixes): the coverage and alignment invariants of
    check_plan hold whatever mix of tile sizes, key spans and copies the planner picks."""
    rng = np.random.default_rng([seed, 0x91A])
    shape = [W.HeadShape(32, 8, 128), W.HeadShape(28, 4, 128), W.HeadShape(8, 2, 64), W.HeadShape(64, 8, 128, "fp8"),
             W.HeadShape(16, 16, 64), W.HeadShape(64, 1, 128), W.HeadShape(16, 2, 128, "fp8")][seed % 7]
    n = int(rng.integers(1, 12))
    kind = rng.integers(0, 4, n)                   # empty, decode, short chunk, long chunk
    C = np.where(kind == 0, 0, np.where(kind == 1, 1, np.where(kind == 2, rng.integers(2, 70, n), rng.integers(70, 900, n))))
    P = np.where(rng.random(n) < 0.3, 0, rng.integers(0, 6000, n))
    if seed % 3 == 0:                              # one long context
        P[int(rng.integers(0, n))] = int(rng.integers(20000, 40000))
    if C.sum() == 0:
        C[0] = 1
    check_plan(shape, P.astype(np.int64), C.astype(np.int64))
