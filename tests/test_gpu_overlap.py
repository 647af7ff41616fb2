"""Prefix ingest on a side stream while the attention of other requests runs (section 4.2,
steps 6-7: the transferred KV cache is stored while the instance keeps computing).  The
attention output must match the fp64 oracle and be bit-identical to the one computed with
nothing else running; afterwards both pools must equal the reference scatter's image bit for
bit (the running requests' rows, the newcomers' prefixes, untouched slots), and the gather
must return the newcomers' prefixes."""
import numpy as np
import pytest
import torch

from paper_2509_17357_amd import binding as B
from paper_2509_17357_amd import workloads as W
from paper_2509_17357_amd.overlap import OverlapRun
from paper_2509_17357_amd.runtime import bits_from_bf16_tensor

import parity_util as U

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("source", ["device", "pinned"])
def test_overlapped_ingest_leaves_attention_untouched(source):
    run = OverlapRun(W.SHAPE_8B, [700, 300, 2047, 90], [200, 1, 1, 1], [513, 1999, 64], seed=8200, source=source,
                     host_inputs=True, pool_fill=0x7FC1)
    it, batch = run.it, run.batch
    main = torch.cuda.current_stream(it.device)
    run.attention(main)
    torch.cuda.synchronize()
    ref = run.out_run.clone()
    # the reference run itself against the oracle (the running requests only)
    sub = W.custom_batch(batch.shape, run.P_run, run.C_run, seed=1)
    want = U.oracle_attention(sub, bits_from_bf16_tensor(run.q_run), U.oracle_kv_values(sub, run.kv_bits[:run.n_run]),
                              it.sm_scale)
    rep = U.error_report(sub, bits_from_bf16_tensor(ref), want)
    print(source, rep)
    U.assert_within_tolerance(rep)
    # wipe the newcomers' blocks, then ingest them again while the attention runs (several rounds)
    ids = torch.from_numpy(np.concatenate([batch.block_tables[s][:(batch.prefix_lens[s] + 16) // 16]
                                           for s in range(run.n_run, batch.n_seqs)]).astype(np.int64)).to(it.device)
    for pool in (it.k_pool, it.v_pool):
        pool.view(batch.num_blocks, -1)[ids] = 0x7FC1
    torch.cuda.synchronize()
    for _ in range(3):
        run.out_run.zero_()
        torch.cuda.synchronize()
        run.side.wait_stream(main)
        run.ingest(run.side)
        run.attention(main)
        torch.cuda.synchronize()
        assert torch.equal(run.out_run, ref)
    # both pools against the reference scatter: the running requests hold prefix + new rows,
    # the newcomers their prefix rows only (their blocks were wiped with the fill pattern)
    import dataclasses
    C_after = batch.chunk_lens.copy()
    C_after[run.n_run:] = 0
    after = dataclasses.replace(batch, chunk_lens=C_after)
    kv_after = [(k, v) if s < run.n_run else (k[:batch.prefix_lens[s]], v[:batch.prefix_lens[s]])
                for s, (k, v) in enumerate(run.kv_bits)]
    kp, vp = U.oracle_pools(after, kv_after, fill=0x7FC1)
    assert np.array_equal(it.k_pool.cpu().numpy().view(np.uint16), kp), "K pool differs from the reference scatter"
    assert np.array_equal(it.v_pool.cpu().numpy().view(np.uint16), vp), "V pool differs from the reference scatter"
    # and the prefixes come back through the gather, bit for bit
    P_new = batch.prefix_lens[run.n_run:].astype(np.int64)
    n = int(P_new.sum())
    sh = batch.shape
    kd = torch.zeros((n, sh.n_kv_heads, sh.head_dim), dtype=torch.int16, device=it.device)
    vd = torch.zeros_like(kd)
    B.cronus_kv_gather(it.cache, kd, vd, run.cu_ingest, run.zero, run.bt_new, batch.max_blocks, run.n_new, n,
                       main.cuda_stream)
    torch.cuda.synchronize()
    want_k = np.concatenate([run.kv_bits[s][0][:P_new[i]] for i, s in enumerate(range(run.n_run, batch.n_seqs))])
    want_v = np.concatenate([run.kv_bits[s][1][:P_new[i]] for i, s in enumerate(range(run.n_run, batch.n_seqs))])
    assert np.array_equal(kd.cpu().numpy().view(np.uint16), want_k)
    assert np.array_equal(vd.cpu().numpy().view(np.uint16), want_v)
