#!/usr/bin/env python3
"""Benchmark of the mixed-iteration attention hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: ingest of the
transferred prefixes of the continuation chunks (cronus_kv_append), append of the
iteration's new K/V rows (cronus_kv_append), and the mixed attention
(cronus_attn_mixed: work decomposition, chunk tiles, decode spans, merge).  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-extra]
                  [--no-cpu-baseline]

The headline workload is the Llama-3-8B-shaped batch (benchmark configs[1]); the
prefill-heavy and decode-heavy batches, which carry the MFMA and HBM roofline targets, and
the 70B-shaped batch with the fp8 cache are timed as well and reported under
"other_workloads"; "scatter_gather" has cronus_kv_append / cronus_kv_gather as pure
data movement.
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

WORKLOADS = {"tiny": 1, "llama3_8b": 2, "prefill_heavy": 3, "decode_heavy": 4, "llama_70b_fp8": 5}
CLOCK_SETTLE_MS = 60.0         # untimed work before the warm-up steps: clocks of an idle GPU rise over tens of ms
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
# which roofline bounds the attention kernel on each workload (KV bytes vs visible-pair flops)
BOUND = {"tiny": "hbm", "llama3_8b": "hbm", "prefill_heavy": "mfma", "decode_heavy": "hbm", "llama_70b_fp8": "mfma"}
# HBM bytes per attention-kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled
# by what the same counters read for a plain 1 GiB copy (FETCH_SIZE x 2.000, WRITE_SIZE x 1.000):
# profiles/attn_mixed_kernel_benchmark_batches_rocprofv3.md.  None where not measured.
MEASURED_TRAFFIC_BYTES = {"tiny": None, "llama3_8b": 624460157, "prefill_heavy": 568301344,
                          "decode_heavy": 4868596580, "llama_70b_fp8": 3998651460}


def time_workload(name, steps, warmup, trial=0):
    import torch
    from paper_2509_17357_amd import binding as B
    from paper_2509_17357_amd import workloads as W
    from paper_2509_17357_amd.runtime import DeviceIteration

    batch = W.draw_batch(WORKLOADS[name], trial)
    it = DeviceIteration(batch, device="cuda:0")
    it.load_device_inputs()
    if it.fp8:
        it.set_fp8_scales(*it.amax_scales())
    it.setup_decode_context()
    it.ensure_workspace()
    torch.cuda.synchronize()

    # let the clocks of an idle GPU settle (untimed, not counted as warm-up steps), then the W warm-up steps
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < CLOCK_SETTLE_MS:
        for _ in range(8):
            it.step()
        torch.cuda.synchronize()
    for _ in range(warmup):
        it.step()
    torch.cuda.synchronize()

    ev = B.HipEvents()
    pairs = [(ev.create(), ev.create()) for _ in range(steps)]
    for a, b in pairs:  # first use of an event is slow (lazy allocation): keep it out of the timed region
        B.cronus_profile_events(a, b)
        it.attention()
    B.cronus_profile_events(None, None)
    torch.cuda.synchronize()
    # The interpreter's cyclic garbage collector stays out of the timed region: with torch
    # imported one full collection takes 30-40 ms, twice the 100 timed steps of the default
    # run, and whether one falls into them changed from run to run (0.18 or 0.5 ms/step).
    gc.collect()
    gc.disable()
    try:
        t0 = time.perf_counter()
        for a, b in pairs:
            B.cronus_profile_events(a, b)
            it.step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    finally:
        gc.enable()
    B.cronus_profile_events(None, None)
    kern_ms = [ev.elapsed_ms(a, b) for a, b in pairs]
    for a, b in pairs:
        ev.destroy(a)
        ev.destroy(b)

    ms_per_step = (t1 - t0) * 1e3 / steps
    kernel_ms = float(np.mean(kern_ms))
    flops, abytes = batch.flops(), batch.attn_bytes()
    bound = BOUND[name]
    if bound == "mfma":
        achieved, peak, unit = flops / (kernel_ms * 1e-3) / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s"
    else:
        achieved, peak, unit = abytes / (kernel_ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
    stats = B.cronus_attn_mixed_plan_stats(it.cache, batch.prefix_lens, batch.chunk_lens)
    sh = batch.shape
    append_bytes = (it.n_prefix_tokens + it.n_new_tokens) * sh.n_kv_heads * sh.head_dim * 2 * (2 + (1 if it.fp8 else 2))
    res = {
        "workload": name,
        "tokens_per_s": batch.total_q / (ms_per_step * 1e-3),
        "kv_tokens_per_s": int(batch.kv_lens.sum()) / (ms_per_step * 1e-3),
        "ms_per_step": ms_per_step,
        "attn_kernel_ms": kernel_ms,
        "attn_kernel_ms_min": float(np.min(kern_ms)),
        "attn_tflops": flops / (kernel_ms * 1e-3) / 1e12,
        "attn_gbs": abytes / (kernel_ms * 1e-3) / 1e9,
        "pct_mfma_peak": 100.0 * flops / (kernel_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "pct_hbm_peak": 100.0 * abytes / (kernel_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "q_tokens": batch.total_q,
        "kv_tokens": int(batch.kv_lens.sum()),
        "n_seqs": batch.n_seqs,
        "algorithmic_flops": flops,
        "algorithmic_bytes": abytes,
        "append_tokens": it.n_prefix_tokens + it.n_new_tokens,
        "append_algorithmic_bytes": append_bytes,
        "plan": stats,
        "roofline": {"bound": bound, "kernel": "attn_mixed_kernel", "achieved": achieved, "peak": peak, "unit": unit,
                     "frac": achieved / peak, "traffic": MEASURED_TRAFFIC_BYTES.get(name)},
    }
    del it
    torch.cuda.empty_cache()
    return res, batch


def time_scatter_gather(reps=5):
    """cronus_kv_append and cronus_kv_gather as pure data movement: the decode contexts of
    the decode-heavy batch (about 1.2 M tokens, 4.8 GB of K+V) scattered into the paged pool
    and exported again.  GB/s counts what the call must move: source read + destination write."""
    import torch
    from paper_2509_17357_amd import binding as B
    from paper_2509_17357_amd import workloads as W
    from paper_2509_17357_amd.runtime import DeviceIteration

    batch = W.draw_batch(WORKLOADS["decode_heavy"])
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
    ap.add_argument("--workload", default="llama3_8b", choices=sorted(WORKLOADS))
    ap.add_argument("--no-extra", action="store_true", help="skip the prefill-heavy / decode-heavy runs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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

    main_res, batch = time_workload(args.workload, args.steps, args.warmup)
    others = {}
    scatter_gather = None
    if not args.no_extra:
        for name in ("prefill_heavy", "decode_heavy"):
            if name != args.workload:
                others[name], _ = time_workload(name, max(5, args.steps // 2), max(2, args.warmup // 2))
        if args.workload != "llama_70b_fp8":
            others["llama_70b_fp8"], _ = time_workload("llama_70b_fp8", max(5, args.steps // 10), max(2, args.warmup // 10))
        scatter_gather = time_scatter_gather()
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
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(batch)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
