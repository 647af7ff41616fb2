"""cronus_kv_gather through the C ABI: the paged -> contiguous export must be bit-exact.
It is checked against the oracle's gather of the oracle's pool image, as the inverse of
cronus_kv_append (the source comes back), and on ranges that start and end inside blocks;
rows outside the call keep their contents."""
import numpy as np
import pytest
import torch

from oracle import cronus_oracle as orc
from paper_2509_17357_amd import binding as B
from paper_2509_17357_amd import workloads as W
from paper_2509_17357_amd.runtime import DeviceIteration

import parity_util as U

pytestmark = pytest.mark.gpu

CASES = [
    # (Hq, Hkv, D, kv dtype, prefix_lens, chunk_lens)
    (8, 2, 64, "bf16", [0, 3, 17, 100, 31], [1, 5, 33, 70, 129]),
    (32, 8, 128, "bf16", [0, 0, 15, 16, 255, 1000], [1, 130, 1, 17, 64, 3]),
    (28, 4, 128, "bf16", [10, 129, 0], [50, 1, 260]),
    (16, 8, 128, "fp8", [33, 0, 500], [31, 1, 77]),
    (8, 2, 64, "fp8", [5, 64], [12, 1]),
]


def filled(case, seed):
    Hq, Hkv, D, dt, P, C = CASES[case]
    batch = W.custom_batch(W.HeadShape(Hq, Hkv, D, dt), P, C, seed=seed)
    fill = 0x7FC1 if dt == "bf16" else 0x7F
    it = DeviceIteration(batch, pool_fill=fill)
    kv_bits = it.load_host_inputs()
    ks = vs = None
    if it.fp8:
        ks, vs = it.amax_scales()
        it.set_fp8_scales(ks, vs)
    it.setup_decode_context()
    it.ingest_prefix()
    it.append_new()
    torch.cuda.synchronize()
    return batch, it, kv_bits, fill, ks, vs


def gather(it, batch, start, count, sentinel):
    """Run the export of positions [start[s], start[s] + count[s]); returns host arrays."""
    sh = batch.shape
    dt = torch.uint8 if it.fp8 else torch.int16
    n_tok = int(np.sum(count))
    pad = 3  # rows after the last one must stay untouched
    kd = torch.full((n_tok + pad, sh.n_kv_heads, sh.head_dim), sentinel, dtype=dt, device=it.device)
    vd = torch.full_like(kd, sentinel)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(it.device)
    cu = i32(np.concatenate([[0], np.cumsum(count)]))
    B.cronus_kv_gather(it.cache, kd, vd, cu, i32(start), it.block_tables, batch.max_blocks, batch.n_seqs, n_tok,
                       torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    view = (lambda t: t.cpu().numpy()) if it.fp8 else (lambda t: t.cpu().numpy().view(np.uint16))
    return view(kd), view(vd), n_tok


@pytest.mark.parametrize("case", range(len(CASES)))
def test_whole_sequences_equal_the_oracle_gather_and_the_source(case):
    batch, it, kv_bits, fill, ks, vs = filled(case, 7300 + case)
    sh = batch.shape
    L = (batch.prefix_lens + batch.chunk_lens).astype(np.int64)
    k, v, n_tok = gather(it, batch, np.zeros_like(L), L, 0x55 if it.fp8 else 0x5555)
    kp, vp = U.oracle_pools(batch, kv_bits, fill=fill, k_scale=ks, v_scale=vs)
    off = 0
    for s in range(batch.n_seqs):
        ek, ev = orc.kv_gather(kp, vp, batch.block_tables[s], int(L[s]), sh.n_kv_heads, sh.head_dim)
        assert np.array_equal(k[off:off + L[s]], ek) and np.array_equal(v[off:off + L[s]], ev), s
        if not it.fp8:  # bf16: the scatter's source comes back bit for bit
            assert np.array_equal(k[off:off + L[s]], kv_bits[s][0]) and np.array_equal(v[off:off + L[s]], kv_bits[s][1])
        off += int(L[s])
    sent = 0x55 if it.fp8 else 0x5555
    assert (k[n_tok:] == sent).all() and (v[n_tok:] == sent).all()


@pytest.mark.parametrize("case", [0, 1, 3])
def test_ranges_inside_blocks_and_empty_ranges(case):
    batch, it, kv_bits, fill, ks, vs = filled(case, 7400 + case)
    sh = batch.shape
    L = (batch.prefix_lens + batch.chunk_lens).astype(np.int64)
    rng = np.random.default_rng(case)
    start = np.array([rng.integers(0, l) for l in L])
    count = np.array([rng.integers(0, l - st + 1) for l, st in zip(L, start)])
    count[0] = 0  # an empty range
    k, v, n_tok = gather(it, batch, start, count, 0x55 if it.fp8 else 0x5555)
    kp, vp = U.oracle_pools(batch, kv_bits, fill=fill, k_scale=ks, v_scale=vs)
    off = 0
    for s in range(batch.n_seqs):
        ek, ev = orc.kv_gather(kp, vp, batch.block_tables[s], int(L[s]), sh.n_kv_heads, sh.head_dim)
        a, b = int(start[s]), int(start[s] + count[s])
        assert np.array_equal(k[off:off + b - a], ek[a:b]) and np.array_equal(v[off:off + b - a], ev[a:b]), s
        off += b - a
    assert off == n_tok


def test_gather_error_codes():
    batch, it, *_ = filled(0, 7500)
    st = torch.cuda.current_stream().cuda_stream
    d = torch.zeros(16, dtype=torch.int16, device=it.device)
    ok = lambda **kw: B.cronus_kv_gather(it.cache, kw.get("k", d), kw.get("v", d), kw.get("cu", it.cu_new),
                                         it.zero_pos, it.block_tables, kw.get("mb", batch.max_blocks),
                                         kw.get("ns", batch.n_seqs), kw.get("nt", 1), st, check=False)
    assert ok(k=None) == B.CRONUS_ERR_INVALID_ARG
    assert ok(cu=None) == B.CRONUS_ERR_INVALID_ARG
    assert ok(nt=-1) == B.CRONUS_ERR_INVALID_ARG
    assert ok(mb=0) == B.CRONUS_ERR_INVALID_ARG
    assert ok(nt=0) == B.CRONUS_OK and ok(ns=0) == B.CRONUS_OK
    torch.cuda.synchronize()
