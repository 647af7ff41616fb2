"""cronus_profile_events: a launch timed through the caller's events computes the same
output, bit for bit, as an untimed one; the main pair brackets the main kernel (a positive
duration, shorter than the wall-clock time of the call plus synchronisation), and the outer
pair the whole attention of the call: from the fp8 copy kernel, if the plan has one, to the
merge kernel, if it has one."""
import time

import pytest
import torch

from paper_2509_17357_amd import binding as B
from paper_2509_17357_amd import workloads as W
from paper_2509_17357_amd.runtime import DeviceIteration

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
def test_timed_launch_matches_untimed(dtype):
    # chunks (wide tiles), decodes long enough to be split (merge kernel), an empty sequence
    # (fp8: the chunk of 1100 tokens spans 18 tiles, so its sequence gets a bf16 copy: three kernels)
    batch = W.custom_batch(W.HeadShape(32, 8, 128, dtype), [700, 0, 9000, 4095, 33, 5, 300],
                           [200, 130, 1, 1, 1, 0, 1100], seed=77)
    it = DeviceIteration(batch)
    it.load_host_inputs()
    if it.fp8:
        it.set_fp8_scales(*it.amax_scales())
    it.setup_decode_context()
    it.ingest_prefix()
    it.append_new()
    it.attention()
    torch.cuda.synchronize()
    plain = it.out.clone()

    stats = B.cronus_attn_mixed_plan_stats(it.cache, batch.prefix_lens, batch.chunk_lens)
    assert stats["merge_groups"] > 0 and (stats["copy_blocks"] > 0) == (dtype == "fp8")
    ev = B.HipEvents()
    start, stop, first, last = ev.create(), ev.create(), ev.create(), ev.create()
    try:
        for _ in range(2):  # the second use of the same pair must work too
            it.out.fill_(0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            B.cronus_profile_events(start, stop, first, last)
            it.attention()
            B.cronus_profile_events(None, None)
            torch.cuda.synchronize()
            wall_ms = (time.perf_counter() - t0) * 1e3
            ms = ev.elapsed_ms(start, stop)
            span = ev.elapsed_ms(first if stats["copy_blocks"] else start, last)
            assert 0.0 < ms < span <= wall_ms
            assert torch.equal(it.out.view(torch.int16), plain.view(torch.int16))
        # switched off again: an ordinary launch
        it.out.fill_(0)
        it.attention()
        torch.cuda.synchronize()
        assert torch.equal(it.out.view(torch.int16), plain.view(torch.int16))
    finally:
        B.cronus_profile_events(None, None)
        for e in (start, stop, first, last):
            ev.destroy(e)
