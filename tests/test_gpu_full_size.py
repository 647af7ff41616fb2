"""The five benchmark batches at FULL size, in the launch configuration bench.py times.
Configs 1-4: every output row against the oracle.  Config 5: every decode row, and a
stratified sample of the chunk rows (first and last tile, tile boundaries, a uniform
sample): its two chunks alone are 8.2 TFLOP of fp64 work for the oracle."""
import numpy as np
import pytest
import torch

from oracle import cronus_oracle as orc
from paper_2509_17357_amd import binding as B
from paper_2509_17357_amd import workloads as W
from paper_2509_17357_amd.runtime import DeviceIteration, bf16_tensor_from_bits, bits_from_bf16_tensor

import parity_util as U

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid", [2, 3])
def test_full_batch_every_row(cid):
    batch = W.draw_batch(cid)
    it = DeviceIteration(batch, pool_fill=0x7FC1)
    kv_bits = it.load_host_inputs()
    it.setup_decode_context()
    it.step()
    torch.cuda.synchronize()
    ref = U.oracle_attention(batch, bits_from_bf16_tensor(it.q), U.oracle_kv_values(batch, kv_bits), it.sm_scale)
    rep = U.error_report(batch, bits_from_bf16_tensor(it.out), ref)
    print(batch.name, rep)
    U.assert_within_tolerance(rep)


def test_paper_shaped_iteration_long_context_every_row():
    """One iteration as the paper runs them (section 5.1: 512 batched tokens): a chunk of
    496 tokens whose request already has 16384 tokens of context, next to 16 decodes.
    Its 64 wide tiles are cut into key spans and merged (the planner's answer to a launch
    with fewer tiles than CUs); every output row is checked."""
    rng = np.random.default_rng(515)
    P = [16384] + rng.integers(1500, 6000, 16).tolist()
    C = [496] + [1] * 16
    batch = W.custom_batch(W.SHAPE_8B, P, C, seed=5150)
    it = DeviceIteration(batch, pool_fill=0x7FC1)
    kv_bits = it.load_host_inputs()
    it.setup_decode_context()
    it.step()
    torch.cuda.synchronize()
    stats = B.cronus_attn_mixed_plan_stats(it.cache, batch.prefix_lens, batch.chunk_lens)
    assert stats["wide_items"] >= 3 * 64
    ref = U.oracle_attention(batch, bits_from_bf16_tensor(it.q), U.oracle_kv_values(batch, kv_bits), it.sm_scale)
    rep = U.error_report(batch, bits_from_bf16_tensor(it.out), ref)
    print(batch.name, rep)
    U.assert_within_tolerance(rep)


@pytest.mark.parametrize("kind", ["bf16", "fp8", "bf16_prefix"])
def test_whole_prompts_every_row(kind):
    """Whole prompts (prefix 0; the prefill that precedes the hand-over of section 4.2) with
    16 tiles per CU, none of them cut into spans: a resident work-group runs sixteen tiles, from
    the longest of a (sequence, KV head) to the shortest, one after the other.  Prompt lengths
    leave whole, nearly whole and tiny last tiles; every output row is checked."""
    if kind == "bf16":
        shape, C = W.SHAPE_8B, [4096, 4100, 4031, 4160, 3900, 4200, 4097, 4223, 1500]
        P = [0] * len(C)
    elif kind == "fp8":
        shape, C = W.SHAPE_70B, [4096, 4100, 4031, 4223, 720]
        P = [0] * len(C)
    else:  # long continuation chunks behind prefixes that are, and are not, multiples of the tile
        shape, C, P = W.SHAPE_8B, [5500, 5440, 5503, 5567, 5500, 5570], [0, 64, 1000, 37, 500, 2049]
    batch = W.custom_batch(shape, P, C, seed=4242)
    it = DeviceIteration(batch, pool_fill=0x7F if kind == "fp8" else 0x7FC1)
    kv_bits = it.load_host_inputs()
    ks = vs = None
    if it.fp8:
        ks, vs = it.amax_scales()
        it.set_fp8_scales(ks, vs)
    it.setup_decode_context()
    it.step()
    torch.cuda.synchronize()
    items = B.cronus_attn_mixed_plan_items(it.cache, batch.prefix_lens, batch.chunk_lens)
    F = {n: i for i, n in enumerate(B.PLAN_ITEM_FIELDS)}
    wide = items[items[:, F["wide"]] >= 1]
    assert len(wide) >= 12 * 256 and (wide[:, F["partial"]] == -1).all()   # many whole tiles per CU
    ref = U.oracle_attention(batch, bits_from_bf16_tensor(it.q), U.oracle_kv_values(batch, kv_bits, ks, vs),
                             it.sm_scale)
    rep = U.error_report(batch, bits_from_bf16_tensor(it.out), ref)
    print(batch.name, kind, rep)
    U.assert_within_tolerance(rep)


def _full_size_check(cid, chunk_rows_of):
    """A benchmark batch at full size with every tensor drawn on the host (so that the oracle
    sees the same bits): the whole hot path on the GPU, then, sequence by sequence, every
    decode row and the chunk rows that chunk_rows_of selects against the oracle, and the
    cache blocks of a sample of sequences against the reference scatter, bit for bit."""
    batch = W.draw_batch(cid)
    sh = batch.shape
    it = DeviceIteration(batch)
    kv = U.draw_all_kv(batch)
    it.load_host_inputs(kv)
    ks = vs = None
    if it.fp8:
        ks, vs = it.amax_scales()
        it.set_fp8_scales(ks, vs)
    it.setup_decode_context()
    it.step()
    torch.cuda.synchronize()
    out_bits, q_bits = bits_from_bf16_tensor(it.out), bits_from_bf16_tensor(it.q)
    rep = U.check_rows_by_sequence(batch, out_bits, q_bits, lambda s: kv[s], it.sm_scale, ks, vs,
                                   rows_of=lambda s, C: np.arange(C) if C == 1 else chunk_rows_of(s, C))
    print(batch.name, rep)
    assert rep["seqs"] == batch.n_seqs
    # scatter: the cache blocks of these sequences hold exactly their rows (bit-exact)
    P, C = batch.prefix_lens.astype(np.int64), batch.chunk_lens.astype(np.int64)
    rng = np.random.default_rng([batch.seed, 0x5A])
    dec_ids = np.flatnonzero(C == 1)
    sample = sorted(set(np.flatnonzero(C > 1).tolist()) | set(rng.choice(dec_ids, size=12, replace=False).tolist()) |
                    {int(dec_ids[np.argmax(P[dec_ids])]), int(dec_ids[np.argmin(P[dec_ids])])})
    for s in sample:
        k, v = kv[s]
        nb = int(batch.blocks_needed()[s])
        ids = torch.from_numpy(batch.block_tables[s, :nb].astype(np.int64)).to(it.device)
        per_blk = sh.n_kv_heads * 16 * sh.head_dim
        kblk = it.k_pool.view(batch.num_blocks, per_blk)[ids].cpu().numpy()
        vblk = it.v_pool.view(batch.num_blocks, per_blk)[ids].cpu().numpy()
        view = (lambda a: a) if it.fp8 else (lambda a: a.view(np.uint16))
        local = W.custom_batch(sh, [P[s]], [C[s]], seed=1)
        local.block_tables = np.arange(nb, dtype=np.int32)[None, :]
        local.num_blocks = nb
        kp, vp = U.oracle_pools(local, [(k, v)], fill=0, k_scale=ks, v_scale=vs)
        L = int(P[s] + C[s])
        gk, gv = orc.kv_gather(view(kblk).reshape(-1), view(vblk).reshape(-1), np.arange(nb), L, sh.n_kv_heads, sh.head_dim)
        ek, ev = orc.kv_gather(kp, vp, np.arange(nb), L, sh.n_kv_heads, sh.head_dim)
        assert np.array_equal(gk, ek) and np.array_equal(gv, ev), s


def test_config4_decode_heavy_every_row():
    """All 257 sequences: the 256 decode rows and the 256 chunk rows, each against the oracle."""
    _full_size_check(4, lambda s, C: np.arange(C))


def test_config5_fp8_long_context_every_decode_row():
    """All 128 decode rows against the oracle; of the two chunks of 4096 tokens a stratified
    sample of rows: the first and the last tile, the rows on both sides of every eighth tile
    boundary, and a uniform sample of 1 in 64."""
    def rows(s, c):
        rng = np.random.default_rng([5000, 0x5B, s])
        tile = 32  # tokens per wide tile at 8 heads per KV head
        edges = np.concatenate([np.arange(0, tile), np.arange(c - tile, c),
                                (np.arange(tile, c, 256)[:, None] + np.array([-1, 0])).ravel()])
        uni = rng.choice(c, size=c // 64, replace=False)
        return np.unique(np.clip(np.concatenate([edges, uni]), 0, c - 1))
    _full_size_check(5, rows)
