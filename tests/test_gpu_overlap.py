"""Prefix ingest on a side stream while the attention of other requests runs (section 4.2):
the attention output must be bit-identical to the one computed with nothing else running,
and the newcomers' prefixes must sit in their blocks bit for bit afterwards."""
import numpy as np
import pytest
import torch

from paper_2509_17357_amd import binding as B
from paper_2509_17357_amd import workloads as W
from paper_2509_17357_amd.overlap import OverlapRun
from paper_2509_17357_amd.runtime import bits_from_bf16_tensor

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
    # the prefixes are back: export them through the gather and compare with the source bits
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
