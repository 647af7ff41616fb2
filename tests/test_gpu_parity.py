"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by
element, on the same seeded inputs.  Scatter must be bit-exact; attention within
max-abs 2e-2 and relative L2 1e-2 (overall, per sequence, chunk rows, decode rows)."""
import numpy as np
import pytest
import torch

from paper_2509_17357_amd import binding as B
from paper_2509_17357_amd import workloads as W
from paper_2509_17357_amd.runtime import DeviceIteration, bits_from_bf16_tensor

import parity_util as U

pytestmark = pytest.mark.gpu


def run_batch(batch, poison=True, check_pools=True, scales=None):
    """Full hot path on the GPU + oracle on the host; returns the error report."""
    fill = 0x7FC1 if batch.shape.kv_dtype == "bf16" else 0x7F  # NaN patterns in unused slots
    it = DeviceIteration(batch, pool_fill=(fill if fill < 0x8000 else fill - 0x10000) if poison else 0)
    kv_bits = it.load_host_inputs()
    ks = vs = None
    if it.fp8:
        ks, vs = scales if scales is not None else it.amax_scales()
        it.set_fp8_scales(ks, vs)
    it.setup_decode_context()
    it.step()
    torch.cuda.synchronize()
    if check_pools:
        kp, vp = U.oracle_pools(batch, kv_bits, fill=fill, k_scale=ks, v_scale=vs)
        view = (lambda t: t.cpu().numpy()) if it.fp8 else (lambda t: t.cpu().numpy().view(np.uint16))
        assert np.array_equal(view(it.k_pool), kp), "K pool differs from the reference scatter"
        assert np.array_equal(view(it.v_pool), vp), "V pool differs from the reference scatter"
    ref = U.oracle_attention(batch, bits_from_bf16_tensor(it.q), U.oracle_kv_values(batch, kv_bits, ks, vs),
                             it.sm_scale)
    rep = U.error_report(batch, bits_from_bf16_tensor(it.out), ref)
    print(batch.name, rep)
    return rep


def test_config1_tiny():
    rep = run_batch(W.draw_batch(1))
    U.assert_within_tolerance(rep)


RAGGED = [
    # (Hq, Hkv, D, prefix_lens, chunk_lens)
    (8, 2, 64, [0, 3, 17, 100, 31], [1, 5, 33, 70, 129]),
    (32, 8, 128, [0, 0, 15, 16, 255, 1000], [1, 130, 1, 17, 64, 3]),
    (4, 4, 128, [5, 0, 63], [40, 200, 1]),          # MHA (G = 1)
    (16, 2, 128, [77, 300], [9, 1]),                 # G = 8
    (28, 4, 128, [10, 129, 0], [50, 1, 260]),        # G = 7 (Qwen2-7B-like grouping)
    (8, 8, 64, [0], [1]),                            # a single key
    (64, 1, 128, [33, 200], [40, 1]),                # G = 64 > 32: two head groups per KV head
    (8, 1, 64, [100, 5, 900], [70, 1, 1]),           # multi-query attention, D = 64
]


@pytest.mark.parametrize("case", range(len(RAGGED)))
def test_ragged_small_batches(case):
    Hq, Hkv, D, P, C = RAGGED[case]
    batch = W.custom_batch(W.HeadShape(Hq, Hkv, D), P, C, seed=4200 + case)
    U.assert_within_tolerance(run_batch(batch))


def test_long_decode_is_split_and_merged():
    batch = W.custom_batch(W.SHAPE_8B, [8191, 4097, 700, 12000], [1, 1, 1, 1], seed=4300)
    it = DeviceIteration(batch)
    stats = B.cronus_attn_mixed_plan_stats(it.cache, batch.prefix_lens, batch.chunk_lens)
    assert stats["partials"] > 0
    U.assert_within_tolerance(run_batch(batch))


SPLIT_WIDE = [
    # (shape, prefix_lens, chunk_lens): few wide tiles with many keys -> key spans + merge
    (W.SHAPE_8B, [3000, 40], [100, 1]),                       # last span holds the causal edge
    (W.SHAPE_8B, [2500], [130]),                              # two wide tiles and a narrow tail of two tokens
    (W.HeadShape(8, 2, 64), [2500, 777], [70, 1]),            # D = 64
    (W.HeadShape(28, 4, 128), [1900], [80]),                  # G = 7: wavefronts start inside a token
    (W.HeadShape(16, 2, 128, "fp8"), [2100, 300], [64, 1]),   # fp8 cache (register-staged wide path)
    (W.SHAPE_8B, [6000, 1999, 1999], [512 - 2, 1, 1]),        # a paper-shaped iteration: 512 batched tokens
]


@pytest.mark.parametrize("case", range(len(SPLIT_WIDE)))
def test_split_wide_tiles(case):
    shape, P, C = SPLIT_WIDE[case]
    batch = W.custom_batch(shape, P, C, seed=4350 + case)
    it = DeviceIteration(batch)
    items = B.cronus_attn_mixed_plan_items(it.cache, batch.prefix_lens, batch.chunk_lens)
    f = {n: i for i, n in enumerate(B.PLAN_ITEM_FIELDS)}
    wide = items[items[:, f["wide"]] == 1]
    assert (wide[:, f["partial"]] >= 0).any() and (wide[:, f["kv_begin"]] > 0).any()
    del it
    U.assert_within_tolerance(run_batch(batch))


def test_full_prompt_prefill_without_prefix():
    """prefix_len = 0: the whole prompt is one chunk (what the partial prefill instance runs
    on its side of the hand-over, section 4.2), here 1500 tokens = 23 full tiles and a
    28-token remainder, next to a second, short prompt."""
    batch = W.custom_batch(W.SHAPE_8B, [0, 0], [1500, 77], seed=4360)
    U.assert_within_tolerance(run_batch(batch))


def test_many_short_decodes_and_empty_sequences():
    """600 decodes with contexts of 1 .. 300 keys, every fifth sequence empty (chunk_len 0)."""
    rng = np.random.default_rng(4370)
    P = rng.integers(0, 300, 600)
    C = np.where(np.arange(600) % 5 == 4, 0, 1)
    batch = W.custom_batch(W.HeadShape(16, 4, 64), P.tolist(), C.tolist(), seed=4370)
    U.assert_within_tolerance(run_batch(batch))


def test_very_long_decode_context():
    """One decode over 131072 keys (32 spans merged) next to a short one."""
    batch = W.custom_batch(W.HeadShape(8, 2, 128), [131071, 40], [1, 1], seed=4380)
    it = DeviceIteration(batch)
    stats = B.cronus_attn_mixed_plan_stats(it.cache, batch.prefix_lens, batch.chunk_lens)
    assert stats["partials"] >= 2 * 32
    del it
    U.assert_within_tolerance(run_batch(batch))


SHAPES = [W.HeadShape(32, 8, 128), W.HeadShape(8, 2, 64), W.HeadShape(28, 4, 128), W.HeadShape(16, 16, 64),
          W.HeadShape(8, 1, 128), W.HeadShape(16, 2, 128, "fp8"), W.HeadShape(8, 4, 64, "fp8")]


@pytest.mark.parametrize("seed", range(24))
def test_random_small_batches(seed):
    """Seeded random mixes of prompts without prefix, continuation chunks of every size class
    (a few tokens, part of a tile, several tiles) and decodes, over several head shapes: the
    planner's thresholds (narrow / wide, spans, interleaving) are hit in combinations that
    the hand-written cases do not list."""
    rng = np.random.default_rng(97000 + seed)
    shape = SHAPES[seed % len(SHAPES)]
    n = int(rng.integers(1, 13))
    P, C = [], []
    for _ in range(n):
        kind = rng.integers(0, 5)
        if kind == 0:      # decode
            P.append(int(rng.integers(0, 4000))); C.append(1)
        elif kind == 1:    # short chunk (narrow item)
            P.append(int(rng.integers(0, 2500))); C.append(int(rng.integers(2, 9)))
        elif kind == 2:    # part of a tile
            P.append(int(rng.integers(0, 3000))); C.append(int(rng.integers(9, 70)))
        elif kind == 3:    # several tiles
            P.append(int(rng.integers(0, 2000))); C.append(int(rng.integers(70, 400)))
        else:              # prompt without prefix
            P.append(0); C.append(int(rng.integers(1, 300)))
    batch = W.custom_batch(shape, P, C, seed=97000 + seed)
    U.assert_within_tolerance(run_batch(batch))


@pytest.mark.parametrize("seed", range(8))
def test_random_long_context_batches(seed):
    """Few chunks against long prefixes (their wide tiles are cut into key spans and merged)
    next to decodes of very different lengths (spans, merges, interleaved queues)."""
    rng = np.random.default_rng(98000 + seed)
    shape = [W.SHAPE_8B, W.HeadShape(28, 4, 128), W.HeadShape(16, 2, 128, "fp8"), W.HeadShape(8, 2, 64)][seed % 4]
    P = [int(rng.integers(2000, 24000)) for _ in range(int(rng.integers(1, 4)))]
    C = [int(rng.integers(64, 512)) for _ in P]
    n_dec = int(rng.integers(0, 21))
    P += [int(rng.integers(100, 20000)) for _ in range(n_dec)]
    C += [1] * n_dec
    batch = W.custom_batch(shape, P, C, seed=98000 + seed)
    U.assert_within_tolerance(run_batch(batch))


def test_config2_scaled_down():
    U.assert_within_tolerance(run_batch(W.draw_batch(2, scale=0.25)))


def test_fp8_chunks_of_many_tiles_over_the_bf16_copy():
    """fp8 cache, chunks of 16 or more tiles: their sequences are converted to bf16 once and
    the tiles read that copy.  One chunk sits behind a long prefix (its tiles are cut into key
    spans and merged: partial results carry the K scale in their exponents, the merge applies
    the V scale), one behind a short prefix with a ragged last tile, one chunk is too short
    for the copy and converts on the fly, and decodes read codes."""
    shape = W.HeadShape(16, 2, 128, "fp8")                       # G = 8: 32 tokens per tile
    P, C = [20000, 300, 77, 9000, 4000], [600, 530, 100, 1, 1]
    batch = W.custom_batch(shape, P, C, seed=4420)
    from paper_2509_17357_amd import binding as B
    c = B.make_cache(0, 0, 1 << 20, 16, 2, 128, B.CRONUS_KV_FP8_E4M3)
    items = B.cronus_attn_mixed_plan_items(c, P, C)
    F = {n: i for i, n in enumerate(B.PLAN_ITEM_FIELDS)}
    copy = items[items[:, F["wide"]] >= 2]
    assert set(int(x) for x in copy[:, F["seq"]]) == {0, 1} and (copy[:, F["partial"]] >= 0).any()
    real = items[items[:, F["wide"]] >= 0]
    assert set(int(x) for x in real[real[:, F["seq"]] == 2][:, F["wide"]]) == {0, 1}   # three tiles and a narrow tail
    U.assert_within_tolerance(run_batch(batch))
    # D = 64 and MQA: other strides in the copy
    U.assert_within_tolerance(run_batch(W.custom_batch(W.HeadShape(8, 1, 64, "fp8"), [5000, 0], [640, 520], seed=4421)))


def test_fp8_cache_head_dim_64():
    batch = W.custom_batch(W.HeadShape(8, 2, 64, "fp8"), [300, 20, 1500], [140, 1, 1], seed=4410)
    U.assert_within_tolerance(run_batch(batch))


def test_fp8_cache_small():
    batch = W.custom_batch(W.HeadShape(16, 2, 128, "fp8"), [40, 0, 500, 1300], [90, 33, 1, 1], seed=4400)
    U.assert_within_tolerance(run_batch(batch))
    # power-of-two scales
    ks = np.full(2, 2.0 ** -9, dtype=np.float32)
    vs = np.full(2, 2.0 ** -10, dtype=np.float32)
    U.assert_within_tolerance(run_batch(batch, scales=(ks, vs)))


@pytest.mark.parametrize("kind", ["peaky", "outlier", "monotone", "equal"])
def test_stress_distributions(kind):
    shape = W.HeadShape(8, 2, 128)
    P, C = 150, 100
    batch = W.custom_batch(shape, [P, P + C - 1], [C, 1], seed=4500)
    qb, kb, vb = W.stress_qkv(kind, 4500, C, P + C, shape)
    it = DeviceIteration(batch, pool_fill=0x7FC1)
    it.load_host_inputs()
    from paper_2509_17357_amd.runtime import bf16_tensor_from_bits
    # both sequences share the same K/V; the decode row is the chunk's last row
    it.prefix_k, it.ctx_k = bf16_tensor_from_bits(kb[:P], it.device), bf16_tensor_from_bits(kb[:P + C - 1], it.device)
    it.prefix_v, it.ctx_v = bf16_tensor_from_bits(vb[:P], it.device), bf16_tensor_from_bits(vb[:P + C - 1], it.device)
    it.new_k = bf16_tensor_from_bits(np.concatenate([kb[P:], kb[P + C - 1:]]), it.device)
    it.new_v = bf16_tensor_from_bits(np.concatenate([vb[P:], vb[P + C - 1:]]), it.device)
    it.q = bf16_tensor_from_bits(np.concatenate([qb, qb[C - 1:]]), it.device)
    it.setup_decode_context()
    it.step()
    torch.cuda.synchronize()
    import oracle.cronus_oracle as orc
    q, k, v = (orc.bf16_bits_to_f64(x) for x in (qb, kb, vb))
    ref = np.concatenate([orc.attn_rows(q, k, v, P, it.sm_scale), orc.attn_rows(q[C - 1:], k, v, P + C - 1, it.sm_scale)])
    rep = U.error_report(batch, bits_from_bf16_tensor(it.out), ref)
    print(kind, rep)
    U.assert_within_tolerance(rep)
    got = bits_from_bf16_tensor(it.out)
    # decode == chunk of one: same keys, same query -> rows agree to bf16 rounding of different summation orders
    d = np.abs(orc.bf16_bits_to_f64(got[C - 1]) - orc.bf16_bits_to_f64(got[C]))
    assert d.max() <= 2e-2


def test_error_codes():
    batch = W.draw_batch(1)
    it = DeviceIteration(batch)
    it.load_host_inputs()
    it.ensure_workspace()
    c = it.cache
    args = (it.q, it.out, batch.prefix_lens, batch.chunk_lens, it.block_tables, batch.max_blocks, it.sm_scale)
    assert B.cronus_attn_mixed(c, *args, it.workspace, 16, check=False) == B.CRONUS_ERR_WORKSPACE
    assert B.cronus_attn_mixed(c, *args, None, 1 << 20, check=False) == B.CRONUS_ERR_WORKSPACE
    assert B.cronus_attn_mixed(c, None, it.out, *args[2:], it.workspace, it.workspace_bytes,
                               check=False) == B.CRONUS_ERR_INVALID_ARG
    too_long = batch.prefix_lens.copy()
    too_long[0] = 16 * batch.max_blocks
    assert B.cronus_attn_mixed(c, it.q, it.out, too_long, *args[3:], it.workspace, it.workspace_bytes,
                               check=False) == B.CRONUS_ERR_INVALID_ARG
    bad = B.make_cache(it.k_pool, it.v_pool, batch.num_blocks, 8, 2, 96)
    assert B.cronus_attn_mixed(bad, *args, it.workspace, it.workspace_bytes, check=False) == B.CRONUS_ERR_UNSUPPORTED
    assert B.cronus_kv_append(bad, it.new_k, it.new_v, it.cu_new, it.prefix_pos, it.block_tables, batch.max_blocks,
                              batch.n_seqs, it.n_new_tokens, check=False) == B.CRONUS_ERR_UNSUPPORTED
    assert B.cronus_kv_append(c, None, it.new_v, it.cu_new, it.prefix_pos, it.block_tables, batch.max_blocks,
                              batch.n_seqs, it.n_new_tokens, check=False) == B.CRONUS_ERR_INVALID_ARG
    # empty batch and zero-length chunks are no-ops
    assert B.cronus_attn_mixed(c, it.q, it.out, batch.prefix_lens, np.zeros_like(batch.chunk_lens), it.block_tables,
                               batch.max_blocks, it.sm_scale, it.workspace, it.workspace_bytes) == B.CRONUS_OK
    torch.cuda.synchronize()
