"""The five benchmark batches at FULL size, in the launch configuration bench.py times.
Configs 1-3: every output row against the oracle.  Configs 4-5: the bulk of the K/V is
drawn on the device; every chunk sequence and a seeded sample of decode sequences get
host-drawn tensors and are checked row by row (config 5: a stratified sample of chunk
rows: first and last tile, tile boundaries, and a uniform sample)."""
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
def test_whole_prompts_paired_tiles_every_row(kind):
    """Whole prompts (prefix 0; the prefill that precedes the hand-over of section 4.2) with
    16 tiles per CU: the planner gives each work-group an early and a late tile of one
    (sequence, KV head).  Prompt lengths leave whole, nearly whole and tiny last tiles, and
    odd tile counts (a single middle tile); every output row is checked."""
    if kind == "bf16":
        shape, C = W.SHAPE_8B, [4096, 4100, 4031, 4160, 3900, 4200, 4097, 4223, 1500]
        P = [0] * len(C)
    elif kind == "fp8":
        shape, C = W.SHAPE_70B, [4096, 4100, 4031, 4223, 720]
        P = [0] * len(C)
    else:  # long continuation chunks pair the same way: the second tile starts at key 0 of a non-empty prefix
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
    assert (wide[:, F["pair_tok1"]] > 0).sum() > 0.9 * len(wide)      # the paired path is what runs
    assert (wide[:, F["pair_tok1"]] == 0).sum() > 0                    # and some single middle tiles
    ref = U.oracle_attention(batch, bits_from_bf16_tensor(it.q), U.oracle_kv_values(batch, kv_bits, ks, vs),
                             it.sm_scale)
    rep = U.error_report(batch, bits_from_bf16_tensor(it.out), ref)
    print(batch.name, kind, rep)
    U.assert_within_tolerance(rep)


def _sampled_check(cid, n_decode_samples, chunk_row_sample):
    batch = W.draw_batch(cid)
    sh = batch.shape
    it = DeviceIteration(batch)
    it.load_device_inputs()
    P, C = batch.prefix_lens.astype(np.int64), batch.chunk_lens.astype(np.int64)
    dec = C == 1
    rng = np.random.default_rng([batch.seed, 0x5A])
    dec_ids = np.flatnonzero(dec)
    sample = sorted(set(np.flatnonzero(~dec).tolist()) |
                    set(rng.choice(dec_ids, size=min(n_decode_samples, dec_ids.size), replace=False).tolist()) |
                    {int(dec_ids[np.argmax(P[dec_ids])]), int(dec_ids[np.argmin(P[dec_ids])])})
    # overwrite the device-drawn rows of the sampled sequences with host-drawn ones
    cu_prefix = np.concatenate([[0], np.cumsum(np.where(dec, 0, P))])
    cu_ctx = np.concatenate([[0], np.cumsum(np.where(dec, P, 0))])
    cu_new = batch.cu_q
    q_bits_host = {}
    kv_host = {}
    for s in sample:
        k, v = batch.gen_kv(s)
        kv_host[s] = (k, v)
        dst_k, dst_v, off = (it.ctx_k, it.ctx_v, cu_ctx[s]) if dec[s] else (it.prefix_k, it.prefix_v, cu_prefix[s])
        dst_k[off:off + P[s]] = bf16_tensor_from_bits(k[:P[s]], it.device)
        dst_v[off:off + P[s]] = bf16_tensor_from_bits(v[:P[s]], it.device)
        it.new_k[cu_new[s]:cu_new[s + 1]] = bf16_tensor_from_bits(k[P[s]:], it.device)
        it.new_v[cu_new[s]:cu_new[s + 1]] = bf16_tensor_from_bits(v[P[s]:], it.device)
        q_bits_host[s] = bits_from_bf16_tensor(it.q[cu_new[s]:cu_new[s + 1]])
    ks = vs = None
    if it.fp8:
        ks, vs = it.amax_scales()
        it.set_fp8_scales(ks, vs)
    it.setup_decode_context()
    it.step()
    torch.cuda.synchronize()
    out = it.out
    worst = 0.0
    for s in sample:
        k, v = kv_host[s]
        sub = W.custom_batch(sh, [P[s]], [C[s]], seed=1)
        (kf, vf), = U.oracle_kv_values(sub, [(k, v)], ks, vs)
        q = orc.bf16_bits_to_f64(q_bits_host[s])
        rows = np.arange(C[s]) if C[s] <= 512 else chunk_row_sample(int(C[s]), rng)
        ref = orc.attn_rows(q, kf, vf, int(P[s]), it.sm_scale, rows=rows)
        got = orc.bf16_bits_to_f64(bits_from_bf16_tensor(out[cu_new[s]:cu_new[s + 1]]))[rows]
        assert not np.isnan(got).any(), s
        err = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        worst = max(worst, err)
        assert err <= U.REL_L2_TOL, (s, err)
        assert np.abs(got - ref).max() <= U.MAX_ABS_TOL, s
        # scatter: the cache blocks of this sequence hold exactly its rows (bit-exact)
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
    print(batch.name, "sampled sequences", len(sample), "worst rel L2", worst)
    # every output row of the batch is finite and of plausible size (properties that hold at any size)
    o = out.float()
    assert torch.isfinite(o).all()
    assert float(o.abs().max()) < 1.0


def test_config4_decode_heavy_sampled():
    _sampled_check(4, 24, lambda c, rng: np.arange(c))


def test_config5_fp8_long_context_sampled():
    def rows(c, rng):
        tile = 32  # tokens per wide tile at 8 heads per KV head
        edges = np.concatenate([np.arange(0, tile), np.arange(c - tile, c),
                                (np.arange(tile, c, 256)[:, None] + np.array([-1, 0])).ravel()])
        uni = rng.choice(c, size=c // 64, replace=False)
        return np.unique(np.clip(np.concatenate([edges, uni]), 0, c - 1))
    _sampled_check(5, 12, rows)
