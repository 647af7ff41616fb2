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
        assert ws >= 16 * b.n_seqs + 48 * st["items"] + 4 * 32 * (sh.head_dim + 2) * st["partials"]
        assert ws % 256 == 0


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
