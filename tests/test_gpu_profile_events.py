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


def test_mfma_probe_runs_and_reports_its_work():
    """The MFMA rate probe (measurement aid): the reported operation count is that of the launch,
    the accumulators come back finite (zero for the constant bit patterns, which are bf16
    denormals; non-zero for random operands), and the rate lies below the published peak."""
    need = B.cronus_probe_mfma_sink_floats()
    n_cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert need == n_cus * 512
    sink = torch.full((need,), float("nan"), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    iters = 200
    for rnd in (False, True):
        sink.fill_(float("nan"))
        flops = B.cronus_probe_mfma(rnd, iters, sink, stream=stream)
        assert flops == 2.0 * 32 * 32 * 16 * 32 * iters * 8 * n_cus
        torch.cuda.synchronize()
        assert bool(torch.isfinite(sink).all())
        assert bool((sink != 0).any()) == rnd
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.cronus_probe_mfma(rnd, 2000, sink, stream=stream)
        e1.record()
        torch.cuda.synchronize()
        tflops = flops * 10 / 1e12 / (e0.elapsed_time(e1) * 1e-3)
        assert 200.0 < tflops < 2600.0, tflops
