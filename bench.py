#!/usr/bin/env python3
"""Benchmark of the mixed-iteration attention hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: ingest of the
transferred prefixes of the continuation chunks (cronus_kv_append), append of the
iteration's new K/V rows (cronus_kv_append), and the mixed attention
(cronus_attn_mixed: work decomposition, chunk tiles, decode spans, merge).  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-extra]
                  [--no-cpu-baseline]

The headline workload is the prefill-heavy batch (benchmark configs[2]): the largest
bf16 batch and the one that carries the MFMA roofline target.  Every other workload is
timed with the same K and W and reported under "other_workloads", each with its own
roofline and cpu_baseline: the Llama-3-8B-shaped batch, the decode-heavy batch (HBM
roofline target), the 70B-shaped batch with the fp8 cache, and two iterations shaped like
the paper's own (section 5.1: 512 batched tokens = one chunk behind 16384 cached tokens +
16 decodes), one per head grouping of the two models of section 5.1.  "scatter_gather" has
cronus_kv_append / cronus_kv_gather as pure data movement.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {"tiny": 1, "llama3_8b": 2, "prefill_heavy": 3, "decode_heavy": 4, "llama_70b_fp8": 5,
             "paper_iteration_16k": "paper:32/8/128", "paper_iteration_16k_g7": "paper:28/4/128"}
HEADLINE = "prefill_heavy"
CLOCK_SETTLE_MS = 150.0        # untimed work before the warm-up steps: the clocks of a GPU that idled take tens of ms of load to settle
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
# which roofline bounds the attention kernel on each workload (KV bytes vs visible-pair flops)
BOUND = {"tiny": "hbm", "llama3_8b": "hbm", "prefill_heavy": "mfma", "decode_heavy": "hbm", "llama_70b_fp8": "mfma",
         "paper_iteration_16k": "mfma", "paper_iteration_16k_g7": "mfma"}
# HBM bytes per launch of the main attention kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this file, scaled by what the same counters read for a plain 1 GiB copy (FETCH_SIZE x
# 2.000, WRITE_SIZE x 1.000).  These are STATIC figures copied from the summary named below, taken
# with the library version named below; with any other library version the line carries null.
TRAFFIC_SOURCE = "profiles/attn_mixed_kernel_benchmark_batches_rocprofv3.md"
TRAFFIC_LIB_VERSION = 504
MEASURED_TRAFFIC_BYTES = {"llama3_8b": 624168265, "prefill_heavy": 612655156, "decode_heavy": 4868695611,
                          "llama_70b_fp8": 4032754278, "paper_iteration_16k": 273880466}


def make_batch(name, trial=0):
    from paper_2509_17357_amd import workloads as W
    cfg = WORKLOADS[name]
    if isinstance(cfg, int):
        return W.draw_batch(cfg, trial)
    # the paper's own iteration (section 5.1: at most 512 batched tokens): one continuation chunk
    # behind 16384 cached tokens + 16 decodes with contexts uniform in [512, 4096]
    hq, hkv, d = (int(x) for x in cfg.split(":")[1].split("/"))
    rng = __import__("numpy").random.default_rng([5100 + trial, hq])
    b = W.paper_iteration(16384, rng.integers(512, 4096, size=16, endpoint=True), budget=512, seed=5100 + trial,
                          shape=W.HeadShape(hq, hkv, d))
    b.name = name
    return b


def time_workload(name, steps, warmup, trial=0):
    import torch
    from paper_2509_17357_amd import binding as B
    from paper_2509_17357_amd.runtime import DeviceIteration

    batch = make_batch(name, trial)
    it = DeviceIteration(batch, device="cuda:0")
    it.load_device_inputs()
    if it.fp8:
        it.set_fp8_scales(*it.amax_scales())
    it.setup_decode_context()
    it.ensure_workspace()
    torch.cuda.synchronize()
    stats = B.cronus_attn_mixed_plan_stats(it.cache, batch.prefix_lens, batch.chunk_lens)

    # The interpreter's cyclic garbage collector stays out of everything from here to the end of
    # the timed region: with torch imported one full collection takes 30-40 ms of host time during
    # which the GPU idles and its clocks drop; the launches that follow then run up to 20 % slower
    # and take some twenty launches to recover (a collection between warm-up and timed steps was
    # what made short runs of this file read 5-10 % below long ones).
    gc.collect()
    gc.disable()
    try:
        # four events per timed step: start/stop of the main kernel's own dispatch, start of the
        # call's first kernel if that is the fp8 copy, stop of its last if that is the merge
        ev = B.HipEvents()
        quads = [tuple(ev.create() for _ in range(4)) for _ in range(steps)]
        for q in quads:  # first use of an event is slow (lazy allocation): keep it out of the timed region
            B.cronus_profile_events(*q)
            it.attention()
        B.cronus_profile_events(None, None)
        torch.cuda.synchronize()
        # let the clocks settle under this workload (untimed, not counted as warm-up steps),
        # then the W warm-up steps, then, with nothing but a synchronisation between, the K timed steps
        t_settle = time.perf_counter()
        while (time.perf_counter() - t_settle) * 1e3 < CLOCK_SETTLE_MS:
            for _ in range(8):
                it.step()
            torch.cuda.synchronize()
        for _ in range(warmup):
            it.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for q in quads:
            B.cronus_profile_events(*q)
            it.step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    finally:
        gc.enable()
    B.cronus_profile_events(None, None)
    main_ms = np.array([ev.elapsed_ms(q[0], q[1]) for q in quads])
    span_ms = np.array([ev.elapsed_ms(q[2] if stats["copy_blocks"] else q[0], q[3] if stats["merge_groups"] else q[1])
                        for q in quads])
    for q in quads:
        for e in q:
            ev.destroy(e)

    ms_per_step = (t1 - t0) * 1e3 / steps
    flops, abytes = batch.flops(), batch.attn_bytes()
    bound = BOUND[name]
    work, peak, unit = (flops / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s") if bound == "mfma" else (abytes / 1e9, PEAK_HBM_GBS, "GB/s")
    rate = lambda ms: work / (ms * 1e-3)
    sh = batch.shape
    append_bytes = (it.n_prefix_tokens + it.n_new_tokens) * sh.n_kv_heads * sh.head_dim * 2 * (2 + (1 if it.fp8 else 2))
    traffic = MEASURED_TRAFFIC_BYTES.get(name) if B.version() == TRAFFIC_LIB_VERSION else None
    span_mean, main_mean = float(span_ms.mean()), float(main_ms.mean())
    res = {
        "workload": name,
        "heads": f"{sh.n_q_heads}/{sh.n_kv_heads}/{sh.head_dim}", "kv_dtype": sh.kv_dtype,
        "tokens_per_s": batch.total_q / (ms_per_step * 1e-3),
        "kv_tokens_per_s": int(batch.kv_lens.sum()) / (ms_per_step * 1e-3),
        "ms_per_step": ms_per_step,
        # the whole attention of a call on the device: first kernel's start to last kernel's end
        # (fp8 copy, main kernel, merge, and the gaps between them)
        "attn_ms": span_mean, "attn_ms_median": float(np.median(span_ms)), "attn_ms_min": float(span_ms.min()),
        # the main kernel alone (what a profiler's kernel trace lists as attn_mixed_kernel)
        "attn_kernel_ms": main_mean, "attn_kernel_ms_median": float(np.median(main_ms)),
        "attn_kernel_ms_min": float(main_ms.min()),
        "attn_ms_first_to_last": [round(float(x), 4) for x in (span_ms if steps <= 40 else span_ms[:: max(1, steps // 40)])],
        "attn_tflops": flops / 1e12 / (span_mean * 1e-3),
        "attn_gbs": abytes / 1e9 / (span_mean * 1e-3),
        "pct_mfma_peak": 100.0 * flops / 1e12 / (span_mean * 1e-3) / PEAK_BF16_TFLOPS,
        "pct_hbm_peak": 100.0 * abytes / 1e9 / (span_mean * 1e-3) / PEAK_HBM_GBS,
        "q_tokens": batch.total_q,
        "kv_tokens": int(batch.kv_lens.sum()),
        "n_seqs": batch.n_seqs,
        "algorithmic_flops": flops,
        "algorithmic_bytes": abytes,
        "append_tokens": it.n_prefix_tokens + it.n_new_tokens,
        "append_algorithmic_bytes": append_bytes,
        "plan": stats,
        # achieved = the call's algorithmic work / mean duration of ALL its attention kernels (span
        # above), so the copy and merge kernels are charged; frac_main_kernel_only divides by the
        # main kernel's own duration, the figure a kernel trace's average reproduces
        "roofline": {"bound": bound, "kernel": "attn_mixed_kernel (+ kv_stage_kernel, attn_merge_kernel of the same call)",
                     "achieved": rate(span_mean), "peak": peak, "unit": unit, "frac": rate(span_mean) / peak,
                     "frac_median": rate(float(np.median(span_ms))) / peak,
                     "frac_main_kernel_only": rate(main_mean) / peak,
                     "timed_launches": int(steps), "traffic": traffic,
                     "traffic_source": (f"{TRAFFIC_SOURCE} (static: rocprofv3 --pmc of library version {TRAFFIC_LIB_VERSION})"
                                        if traffic is not None else None)},
    }
    del it
    torch.cuda.empty_cache()
    return res, batch


def time_mfma_probe(iters=4000, reps=5):
    """What rate of v_mfma_f32_32x32x16_bf16 this GPU sustains when every CU issues nothing else
    (cronus_probe_mfma): with operand registers that hold small constants, and with random bf16
    values.  Context for the MFMA roofline fractions: the published peak assumes the nominal
    clock, which the GPU does not hold under a chip-wide MFMA load on real data."""
    import torch
    from paper_2509_17357_amd import binding as B
    sink = torch.empty(B.cronus_probe_mfma_sink_floats(), dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    out = {"instruction": "v_mfma_f32_32x32x16_bf16", "wavefronts_per_cu": 8, "mfma_per_wavefront": 32 * iters}
    for name, rnd in (("constant_operands", False), ("random_operands", True)):
        for _ in range(3):
            flops = B.cronus_probe_mfma(rnd, iters, sink, stream=stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            B.cronus_probe_mfma(rnd, iters, sink, stream=stream)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out[name] = {"ms": ms, "tflops": flops / 1e12 / (ms * 1e-3), "frac_of_peak": flops / 1e12 / (ms * 1e-3) / PEAK_BF16_TFLOPS}
    return out


def time_scatter_gather(reps=5):
    """cronus_kv_append and cronus_kv_gather as pure data movement: the decode contexts of
    the decode-heavy batch (about 1.2 M tokens, 4.8 GB of K+V) scattered into the paged pool
    and exported again.  GB/s counts what the call must move: source read + destination write."""
    import torch
    from paper_2509_17357_amd import binding as B
    from paper_2509_17357_amd import workloads as W
    from paper_2509_17357_amd.runtime import DeviceIteration

    batch = make_batch("decode_heavy")
    it = DeviceIteration(batch, device="cuda:0")
    it.load_device_inputs()
    sh = batch.shape
    n = it.n_ctx_tokens
    kd, vd = torch.empty_like(it.ctx_k), torch.empty_like(it.ctx_v)
    stream = torch.cuda.current_stream().cuda_stream
    gather = lambda: B.cronus_kv_gather(it.cache, kd, vd, it.cu_ctx, it.zero_pos, it.block_tables, batch.max_blocks,
                                        batch.n_seqs, n, stream)
    out = {}
    for name, fn in (("kv_append", it.setup_decode_context), ("kv_gather", gather)):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        nbytes = 2 * n * sh.n_kv_heads * sh.head_dim * 2 * 2  # K and V, read + write, bf16
        out[name] = {"tokens": n, "ms": ms, "algorithmic_bytes": nbytes, "gbs": nbytes / (ms * 1e-3) / 1e9,
                     "pct_hbm_peak": 100.0 * nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
    assert torch.equal(kd, it.ctx_k) and torch.equal(vd, it.ctx_v), "gather(append(x)) != x"
    del it, kd, vd
    torch.cuda.empty_cache()
    return out


def cpu_baseline(batch, budget_s=12.0, min_s=10.0):
    """The fp64 oracle, untuned, on a bounded stratified sample of the same batch:
    chunk sequences and decode sequences are sampled separately (whole sequences, in
    batch order, until each group has used its share of the time budget) and each
    group's time is scaled to the whole batch by its visible (query, key) pairs.  A batch
    the oracle finishes sooner is passed over again until about min_s seconds of CPU work
    have been timed, so that the figure is not a cold first call."""
    import threadpoolctl

    from oracle import cronus_oracle as orc

    sh = batch.shape
    P, C = batch.prefix_lens.astype(np.int64), batch.chunk_lens.astype(np.int64)
    cu = batch.cu_q
    sm_scale = 1.0 / float(np.sqrt(sh.head_dim))
    q_bits = batch.gen_q()
    pairs = C * P + C * (C + 1) // 2
    groups = {"chunk": [s for s in range(batch.n_seqs) if C[s] > 1], "decode": [s for s in range(batch.n_seqs) if C[s] == 1]}
    t_used = {g: 0.0 for g in groups}
    done = {g: 0 for g in groups}
    seqs_seen, rows_seen = set(), 0
    passes, t_total = 0, 0.0
    inputs = {}
    while passes == 0 or (t_total < min_s and passes < 64):
        passes += 1
        for name, ids in groups.items():
            t_pass = 0.0
            for s in ids:
                if t_pass > budget_s:
                    break
                if s not in inputs:
                    k_bits, v_bits = batch.gen_kv(s)
                    inputs[s] = (orc.bf16_bits_to_f64(q_bits[cu[s]:cu[s + 1]]), orc.bf16_bits_to_f64(k_bits),
                                 orc.bf16_bits_to_f64(v_bits))
                q, k, v = inputs[s]
                t0 = time.perf_counter()
                orc.attn_rows(q, k, v, int(P[s]), sm_scale)
                dt = time.perf_counter() - t0
                t_pass += dt
                done[name] += int(pairs[s])
                if s not in seqs_seen:
                    seqs_seen.add(s)
                    rows_seen += int(C[s])
            t_used[name] += t_pass
            t_total += t_pass
    est_full_s = sum(t_used[g] * int(pairs[ids].sum()) / max(done[g], 1) for g, ids in groups.items() if ids)
    pairs_done = sum(done.values())
    threads = max((i.get("num_threads", 1) for i in threadpoolctl.threadpool_info()), default=1)
    return {"value": batch.total_q / est_full_s, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{rows_seen} query rows of {len(seqs_seen)} whole sequences, {passes} pass(es): {pairs_done} "
                      f"visible (query,key) pairs per head timed in {t_total:.2f} s (the batch has {int(pairs.sum())}); "
                      f"chunk and decode groups scaled separately to the whole batch by pairs",
            "oracle_seconds_full_batch_extrapolated": est_full_s,
            "oracle_gflops": 4 * sh.head_dim * sh.n_q_heads * pairs_done / max(t_total, 1e-9) / 1e9}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: the clocks of an idle MI355X take some tens of milliseconds of work to settle
    # (10 warm-up steps of this 0.2 ms step measured 9 % slower than 100)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default=HEADLINE, choices=sorted(WORKLOADS))
    ap.add_argument("--no-extra", action="store_true", help="time the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mfma-probe", action="store_true", help="run only the MFMA rate probe (cronus_probe_mfma)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB device copy (reference for the FETCH_SIZE/WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)

    if args.calibrate_copy:
        n = 1 << 30
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(max(1, args.steps)):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "launches": max(1, args.steps)}))
        return

    if args.mfma_probe:
        print(json.dumps({"mfma_probe": time_mfma_probe()}))
        return

    main_res, batch = time_workload(args.workload, args.steps, args.warmup)
    if not args.no_cpu_baseline:
        main_res["cpu_baseline"] = cpu_baseline(batch)
    others = {}
    scatter_gather = None
    mfma_probe = None
    if not args.no_extra:
        mfma_probe = time_mfma_probe()
        # every workload with the same K timed launches after the same settle phase and W warm-up steps
        for name in ("llama3_8b", "prefill_heavy", "decode_heavy", "llama_70b_fp8", "paper_iteration_16k",
                     "paper_iteration_16k_g7"):
            if name == args.workload:
                continue
            others[name], b = time_workload(name, args.steps, args.warmup)
            if not args.no_cpu_baseline:
                others[name]["cpu_baseline"] = cpu_baseline(b, budget_s=3.0, min_s=2.5)
            del b
        scatter_gather = time_scatter_gather()
    if mfma_probe is not None:
        # context, not the roofline: the fraction of what plain MFMA issue sustains on this GPU, on random data
        for res in [main_res, *others.values()]:
            if res["roofline"]["bound"] == "mfma":
                res["roofline"]["mfma_probe_tflops"] = mfma_probe["random_operands"]["tflops"]
                res["roofline"]["frac_of_mfma_probe"] = res["roofline"]["achieved"] / mfma_probe["random_operands"]["tflops"]
    sh = batch.shape
    line = {
        "metric": "mixed-batch attention tokens/s; TFLOP/s and HBM GB/s as % of MI355X peak",
        "value": main_res["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "clock_settle_ms": CLOCK_SETTLE_MS,
        "config": {"workload": args.workload, "q_heads": sh.n_q_heads, "kv_heads": sh.n_kv_heads,
                   "head_dim": sh.head_dim, "kv_dtype": sh.kv_dtype, "block_size": 16,
                   "n_seqs": batch.n_seqs, "q_tokens": batch.total_q, "kv_tokens": int(batch.kv_lens.sum()),
                   "step": "kv_append(prefix of chunks) + kv_append(new tokens) + attn_mixed"},
        "detail": main_res,
        "roofline": main_res["roofline"],
        "other_workloads": others,
        "scatter_gather": scatter_gather,
        "mfma_probe": mfma_probe,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = main_res["cpu_baseline"]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
