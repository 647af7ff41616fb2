"""cronus_profile_events: a launch timed through the caller's events computes the same
output, bit for bit, as an untimed one, and the events bracket that one kernel (a positive
duration, shorter than the wall-clock time of the call plus synchronisation)."""
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
    batch = W.custom_batch(W.HeadShape(32, 8, 128, dtype), [700, 0, 9000, 4095, 33, 5], [200, 130, 1, 1, 1, 0], seed=77)
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

    ev = B.HipEvents()
    start, stop = ev.create(), ev.create()
    try:
        for _ in range(2):  # the second use of the same pair must work too
            it.out.fill_(0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            B.cronus_profile_events(start, stop)
            it.attention()
            B.cronus_profile_events(None, None)
            torch.cuda.synchronize()
            wall_ms = (time.perf_counter() - t0) * 1e3
            ms = ev.elapsed_ms(start, stop)
            assert 0.0 < ms <= wall_ms
            assert torch.equal(it.out.view(torch.int16), plain.view(torch.int16))
        # switched off again: an ordinary launch
        it.out.fill_(0)
        it.attention()
        torch.cuda.synchronize()
        assert torch.equal(it.out.view(torch.int16), plain.view(torch.int16))
    finally:
        B.cronus_profile_events(None, None)
        ev.destroy(start)
        ev.destroy(stop)
