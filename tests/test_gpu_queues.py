"""The work queues of the main kernel (resident work-groups take their items through queue
heads that live in a small device array of the library, one set per plan buffer of the
ring, and every launch leaves its set zero): many calls in a row that wrap the ring of plan
buffers several times, calls of different batches alternating, and calls on two streams whose
kernels overlap on the device, must each give the bits that the same call gives alone."""
import numpy as np
import pytest
import torch

from paper_2509_17357_amd import binding as B
from paper_2509_17357_amd import workloads as W
from paper_2509_17357_amd.runtime import DeviceIteration

import parity_util as U

pytestmark = pytest.mark.gpu


def prepared(shape, P, C, seed):
    batch = W.custom_batch(shape, P, C, seed=seed)
    it = DeviceIteration(batch)
    it.load_host_inputs()
    if it.fp8:
        it.set_fp8_scales(*it.amax_scales())
    it.setup_decode_context()
    it.ingest_prefix()
    it.append_new()
    it.ensure_workspace()
    it.attention()
    torch.cuda.synchronize()
    return batch, it, it.out.clone()


def call(it, batch, stream):
    return B.cronus_attn_mixed(it.cache, it.q, it.out, batch.prefix_lens, batch.chunk_lens, it.block_tables,
                               batch.max_blocks, it.sm_scale, it.workspace, it.workspace_bytes, stream.cuda_stream)


def test_many_calls_wrap_the_ring_and_two_streams_overlap():
    # a: chunk tiles (some cut into spans), decodes cut into spans; b: many short items; c: fp8 with a bf16 copy
    a, it_a, ref_a = prepared(W.SHAPE_8B, [9000, 700, 0, 4095, 33, 12000], [1, 200, 130, 1, 1, 300], seed=9300)
    rng = np.random.default_rng(9301)
    b, it_b, ref_b = prepared(W.HeadShape(16, 4, 64), rng.integers(0, 600, 300).tolist(), [1] * 300, seed=9301)
    c, it_c, ref_c = prepared(W.HeadShape(16, 2, 128, "fp8"), [5000, 77, 3000], [600, 1, 1], seed=9302)
    # the first call on a. is checked against the oracle once, so that "the same bits" below means "right"
    kv = [a.gen_kv(s) for s in range(a.n_seqs)]
    rep = U.check_rows_by_sequence(a, ref_a.cpu().view(torch.int16).numpy().view(np.uint16), a.gen_q(), lambda s: kv[s], it_a.sm_scale)
    assert rep["rows"] == a.total_q
    main = torch.cuda.current_stream()
    # 1. 45 calls in a row on one stream, batches alternating: the ring of 8 plan buffers wraps five times
    for i in range(45):
        batch, it, ref = ((a, it_a, ref_a), (b, it_b, ref_b), (c, it_c, ref_c))[i % 3]
        if i % 9 == 0:
            it.out.zero_()
        call(it, batch, main)
    torch.cuda.synchronize()
    for it, ref in ((it_a, ref_a), (it_b, ref_b), (it_c, ref_c)):
        assert torch.equal(it.out.view(torch.int16), ref.view(torch.int16))
    # 2. two streams: calls of a and b go out back to back without waiting, their kernels share the device
    side = torch.cuda.Stream()
    for rnd in range(6):
        it_a.out.zero_()
        it_b.out.zero_()
        it_c.out.zero_()
        torch.cuda.synchronize()
        for _ in range(3):
            call(it_a, a, main)
            call(it_b, b, side)
            call(it_c, c, main)
        torch.cuda.synchronize()
        assert torch.equal(it_a.out.view(torch.int16), ref_a.view(torch.int16)), rnd
        assert torch.equal(it_b.out.view(torch.int16), ref_b.view(torch.int16)), rnd
        assert torch.equal(it_c.out.view(torch.int16), ref_c.view(torch.int16)), rnd
    # 3. the static entry point afterwards (its own set of queue heads)
    it_a.out.zero_()
    B.cronus_attn_mixed_static(it_a.cache, it_a.q, it_a.out, a.prefix_lens, a.chunk_lens, it_a.block_tables, a.max_blocks,
                               it_a.sm_scale, main.cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(it_a.out.view(torch.int16), ref_a.view(torch.int16))
