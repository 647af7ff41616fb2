"""CPU-side checks of the C ABI: the library loads, exports every symbol that
include/cronus.h declares, and its host logic (argument checks, work decomposition
sizes) behaves; no kernel is launched."""
import os
import re

import numpy as np

from paper_2509_17357_amd import binding as B
from paper_2509_17357_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cronus.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cronus_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(B.EXPORTS) <= set(names)
    L = B.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert B.version() >= 100
    assert B.status_string(B.CRONUS_OK) == "ok"
    assert "workspace" in B.status_string(B.CRONUS_ERR_WORKSPACE)


def test_workspace_and_plan_sizes_for_the_five_configs():
    for cid in range(1, 6):
        b = W.draw_batch(cid)
        sh = b.shape
        c = B.make_cache(0, 0, b.num_blocks, sh.n_q_heads, sh.n_kv_heads, sh.head_dim,
                         B.CRONUS_KV_FP8_E4M3 if sh.kv_dtype == "fp8" else B.CRONUS_KV_BF16)
        st = B.cronus_attn_mixed_plan_stats(c, b.prefix_lens, b.chunk_lens)
        ws = B.cronus_attn_mixed_workspace_bytes(c, b.prefix_lens, b.chunk_lens)
        assert st["items"] >= sh.n_kv_heads * int((b.chunk_lens > 0).sum())
        # the workspace holds the partial results (and, for fp8, the bf16 copy), not the work list
        copy = 2 * st["copy_blocks"] * sh.n_kv_heads * 16 * sh.head_dim * 2
        partials = 4 * 32 * (sh.head_dim + 2) * st["partials"]
        assert partials + copy <= ws <= partials + copy + 1024 and ws % 256 == 0 and ws > 0
        assert (st["merge_groups"] > 0) == (st["partials"] > 0)


def test_argument_checks_without_a_device():
    c = B.make_cache(0, 0, 10, 8, 3, 64)  # Hq % Hkv != 0
    assert B.cronus_attn_mixed_workspace_bytes(c, [1], [1]) == 0
    c = B.make_cache(0, 0, 10, 8, 2, 64, block_size=32)
    assert B.cronus_attn_mixed_workspace_bytes(c, [1], [1]) == 0
    c = B.make_cache(0, 0, 10, 8, 2, 64)
    assert B.cronus_attn_mixed_workspace_bytes(c, [-1], [1]) == 0
    assert B.cronus_attn_mixed_workspace_bytes(c, [5], [0]) > 0
    # null cache pointers are rejected before anything touches a device
    assert B.cronus_attn_mixed(c, 0, 0, [1], [1], 0, 1, 0.125, 0, 0, check=False) == B.CRONUS_ERR_INVALID_ARG
    assert B.cronus_kv_append(c, 0, 0, 0, 0, 0, 1, 1, 1, check=False) == B.CRONUS_ERR_INVALID_ARG
    # the MFMA rate probe: iteration count, null sink, a sink that is too small (made-up address, never used)
    need = B.cronus_probe_mfma_sink_floats()
    assert need == 256 * 512  # without a device the library assumes MI355X's 256 CUs
    assert B.cronus_probe_mfma(True, 0, 0x1000, need, check=False) == B.CRONUS_ERR_INVALID_ARG
    assert B.cronus_probe_mfma(True, (1 << 20) + 1, 0x1000, need, check=False) == B.CRONUS_ERR_INVALID_ARG
    assert B.cronus_probe_mfma(True, 10, 0, need, check=False) == B.CRONUS_ERR_INVALID_ARG
    assert B.cronus_probe_mfma(False, 10, 0x1000, need - 1, check=False) == B.CRONUS_ERR_WORKSPACE


def test_workload_recipes():
    b1 = W.draw_batch(1)
    assert b1.prefix_lens.tolist() == [192, 255, 255, 255, 255] and b1.chunk_lens.tolist() == [64, 1, 1, 1, 1]
    assert b1.visible_pairs() * 8 == 15392 * 8 and b1.flops() == 31522816
    b2 = W.draw_batch(2)
    assert (b2.chunk_lens[:4] == 512).all() and ((b2.prefix_lens[:4] >= 512) & (b2.prefix_lens[:4] <= 2048)).all()
    assert ((b2.kv_lens[4:] >= 256) & (b2.kv_lens[4:] <= 4096)).all() and b2.n_seqs == 68
    b3 = W.draw_batch(3)
    assert (b3.chunk_lens[:8] <= 2048).all() and (b3.kv_lens[:8] <= 8192).all() and b3.n_seqs == 24
    b4 = W.draw_batch(4)
    assert b4.n_seqs == 257 and b4.total_q == 512 and ((b4.kv_lens[1:] >= 1024) & (b4.kv_lens[1:] <= 8192)).all()
    b5 = W.draw_batch(5)
    assert b5.shape.kv_dtype == "fp8" and b5.total_q == 8320 and (b5.kv_lens[:2] == 32768).all()
    for b in (b1, b2, b3, b4, b5):
        ids = b.block_tables[b.block_tables >= 0]
        assert ids.size == len(set(ids.tolist())) == int(b.blocks_needed().sum())  # no block shared
        assert b.num_blocks >= 1.25 * ids.size - 1 and ids.max() < b.num_blocks
        for s in range(b.n_seqs):
            n = int(b.blocks_needed()[s])
            assert (b.block_tables[s, :n] >= 0).all() and (b.block_tables[s, n:] == -1).all()
    # same seed, same draw; different trial, different draw
    assert np.array_equal(W.draw_batch(2).prefix_lens, b2.prefix_lens)
    assert not np.array_equal(W.draw_batch(2, trial=1).prefix_lens, b2.prefix_lens)
    # bf16 helper: round to nearest even
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5], dtype=np.float32)  # 1+2^-8 is a tie -> 1.0
    assert W.f32_to_bf16_bits(x).tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020]


def test_error_paths_forced_from_the_host():
    """Every error that the header promises 'before anything is launched' is returned with
    made-up device addresses (nothing may touch them), and on a machine without a GPU a call
    with valid arguments ends in CRONUS_ERR_HIP at the device set-up, again before a launch."""
    fake = 0x7F0000001000  # never dereferenced: all of these calls return from the host-side checks
    c = B.make_cache(fake, fake, 100, 8, 2, 64)
    ok = dict(max_blocks_per_seq=4, sm_scale=0.125)
    call = lambda cache, q, out, P, C, bt, ws, ws_bytes, **kw: B.cronus_attn_mixed(
        cache, q, out, P, C, bt, kw.get("max_blocks_per_seq", 4), kw.get("sm_scale", 0.125), ws, ws_bytes, check=False)
    need = B.cronus_attn_mixed_workspace_bytes(c, [40], [3])
    assert need >= 256
    assert call(c, fake, fake, [40], [3], fake, None, need) == B.CRONUS_ERR_WORKSPACE        # no workspace
    assert call(c, fake, fake, [40], [3], fake, fake + 8, need) == B.CRONUS_ERR_WORKSPACE    # misaligned
    assert call(c, fake, fake, [40], [3], fake, fake, need - 1) == B.CRONUS_ERR_WORKSPACE    # too small
    assert call(c, fake, fake, [62], [3], fake, fake, need) == B.CRONUS_ERR_INVALID_ARG      # 65 keys > 4 blocks
    assert call(c, fake, fake, [-1], [3], fake, fake, need) == B.CRONUS_ERR_INVALID_ARG
    assert call(c, fake, fake, [40], [-3], fake, fake, need) == B.CRONUS_ERR_INVALID_ARG
    assert call(c, None, fake, [40], [3], fake, fake, need) == B.CRONUS_ERR_INVALID_ARG      # q
    assert call(c, fake, None, [40], [3], fake, fake, need) == B.CRONUS_ERR_INVALID_ARG      # out
    assert call(c, fake, fake, [40], [3], None, fake, need) == B.CRONUS_ERR_INVALID_ARG      # block tables
    for bad_scale in (0.0, -1.0, float("nan"), float("inf")):
        assert call(c, fake, fake, [40], [3], fake, fake, need, sm_scale=bad_scale) == B.CRONUS_ERR_INVALID_ARG
    assert call(c, fake, fake, [40], [3], fake, fake, need, max_blocks_per_seq=0) == B.CRONUS_ERR_INVALID_ARG
    assert call(c, fake, fake, [40, 7], [0, 0], fake, None, 0) == B.CRONUS_OK                # nothing to do
    for bad in (B.make_cache(fake, fake, 100, 8, 2, 96), B.make_cache(fake, fake, 100, 8, 2, 64, kv_dtype=7),
                B.make_cache(fake, fake, 100, 8, 3, 64), B.make_cache(fake, fake, 100, 8, 2, 64, block_size=32)):
        assert call(bad, fake, fake, [40], [3], fake, fake, need) == B.CRONUS_ERR_UNSUPPORTED
    for bad in (B.make_cache(None, fake, 100, 8, 2, 64), B.make_cache(fake, fake, 0, 8, 2, 64),
                B.make_cache(fake, fake, 100, 8, 2, 64, k_scale=fake, v_scale=fake),           # scales on a bf16 cache
                B.make_cache(fake, fake, 100, 8, 2, 64, kv_dtype=B.CRONUS_KV_FP8_E4M3)):       # fp8 without scales
        assert call(bad, fake, fake, [40], [3], fake, fake, need) == B.CRONUS_ERR_INVALID_ARG
    # the scatter and the gather: counts and pointers
    for fn in (B.cronus_kv_append, B.cronus_kv_gather):
        assert fn(c, fake, fake, fake, fake, fake, 4, -1, 5, check=False) == B.CRONUS_ERR_INVALID_ARG
        assert fn(c, fake, fake, fake, fake, fake, 4, 1, -5, check=False) == B.CRONUS_ERR_INVALID_ARG
        assert fn(c, fake, fake, fake, fake, fake, 0, 1, 5, check=False) == B.CRONUS_ERR_INVALID_ARG
        assert fn(c, fake, fake, None, fake, fake, 4, 1, 5, check=False) == B.CRONUS_ERR_INVALID_ARG
        assert fn(c, fake, fake, fake, fake, fake, 4, 1, 0, check=False) == B.CRONUS_OK       # no rows: no-op
    import torch
    if not torch.cuda.is_available():
        # valid arguments, no device: the set-up that precedes the first launch reports it
        assert call(c, fake, fake, [40], [3], fake, fake, need) == B.CRONUS_ERR_HIP
        assert B.cronus_kv_append(c, fake, fake, fake, fake, fake, 4, 1, 5, check=False) == B.CRONUS_ERR_HIP
