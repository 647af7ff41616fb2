#!/usr/bin/env python3
"""Profile the chunked prefill iteration of this library on the GPU it runs on and fit the
balancer's iteration-time model (Cronus section 4.4, Eq. 3):

    t_chunked = k_ctxp * L_ctxp + k_ctxd * sum(L_ctxd) + b_c

Each sample is one paper-shaped iteration (section 5.1: at most `--budget` batched tokens):
one prefill request that already has L_ctxp tokens of context and contributes
n_p = budget - n_d chunk tokens, next to n_d decode requests whose contexts add up to a
chosen total.  What is timed is this library's part of the iteration: the attention kernels
on the device (events on the dispatches themselves; the main fit), and append of the new K/V
rows + mixed attention by the host's clock (second fit); the MLP and projection time of a real
model is a constant at a fixed token budget and would only add to b_c.  Prints one JSON object with the
coefficients (milliseconds per token / milliseconds), R^2 and the mean absolute percentage
error, ready for cronus_balancer_model; `--table` also lists every sample.

    python -m paper_2509_17357_amd.fit_eq3 [--budget 512] [--steps 20] [--table]
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def sample_grid(budget):
    ctxp = [0, 1024, 2048, 4096, 8192, 16384, 32768]
    dec = [(0, 0), (16, 32768), (64, 131072), (64, 524288), (128, 262144), (128, 1048576)]  # (n_d, sum of contexts)
    return [(lp, nd, tot) for lp in ctxp for nd, tot in dec if nd < budget]


def make_batch(W, lp, n_d, total_ctx, budget, seed):
    n_p = budget - n_d
    rng = np.random.default_rng(seed)
    if n_d:
        # contexts that differ from request to request and add up to total_ctx (each >= 2)
        w = rng.uniform(0.5, 1.5, n_d)
        ctx = np.maximum(2, np.floor(w / w.sum() * total_ctx).astype(np.int64))
        ctx[0] += total_ctx - int(ctx.sum())
    else:
        ctx = np.zeros(0, dtype=np.int64)
    P = [lp] + [int(c) - 1 for c in ctx]  # a decode with context c attends c keys, its own included
    C = [n_p] + [1] * n_d
    return W.custom_batch(W.HeadShape(32, 8, 128), P, C, seed=seed)


def time_batch(batch, steps, warmup):
    """(attention ms, wall ms) per iteration.  Attention: the device time of the call's kernels,
    from the first one's start to the last one's end, taken with HIP events on the dispatches
    themselves (cronus_profile_events), median over the iterations.  Wall: host clock around
    append + attention, fastest of four groups of iterations (a stall of the host does not count)."""
    import torch
    from . import binding as B
    from .runtime import DeviceIteration
    it = DeviceIteration(batch, device="cuda:0")
    it.load_device_inputs()
    it.setup_decode_context()
    it.ingest_prefix()
    it.ensure_workspace()
    stats = B.cronus_attn_mixed_plan_stats(it.cache, batch.prefix_lens, batch.chunk_lens)
    ev = B.HipEvents()
    quads = [tuple(ev.create() for _ in range(4)) for _ in range(steps)]
    for q in quads[:max(warmup, 1)]:
        B.cronus_profile_events(*q)
        it.append_new()
        it.attention()
    for q in quads:  # every event has been used once before it counts
        B.cronus_profile_events(*q)
        it.attention()
    torch.cuda.synchronize()
    groups = []
    per_group = max(1, steps // 4)
    k = 0
    for _ in range(4):
        t0 = time.perf_counter()
        for _ in range(per_group):
            B.cronus_profile_events(*quads[k])
            k += 1
            it.append_new()
            it.attention()
        torch.cuda.synchronize()
        groups.append((time.perf_counter() - t0) * 1e3 / per_group)
    B.cronus_profile_events(None, None)
    span = [ev.elapsed_ms(q[2] if stats["copy_blocks"] else q[0], q[3] if stats["merge_groups"] else q[1]) for q in quads[:k]]
    for q in quads:
        for e in q:
            ev.destroy(e)
    del it
    torch.cuda.empty_cache()
    return float(np.median(span)), min(groups)


def fit(rows, key="ms"):
    a = np.array([[r["l_ctxp"], r["l_ctxd"], 1.0] for r in rows], dtype=np.float64)
    t = np.array([r[key] for r in rows], dtype=np.float64)
    coef, *_ = np.linalg.lstsq(a, t, rcond=None)
    pred = a @ coef
    ss_res, ss_tot = float(((t - pred) ** 2).sum()), float(((t - t.mean()) ** 2).sum())
    return {"k_ctxp_ms_per_token": float(coef[0]), "k_ctxd_ms_per_token": float(coef[1]), "b_c_ms": float(coef[2]),
            "r2": 1.0 - ss_res / ss_tot, "mape_percent": float(np.mean(np.abs(pred - t) / t) * 100.0),
            "samples": len(rows)}, pred


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--budget", type=int, default=512, help="batched tokens per iteration")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--table", action="store_true")
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        print("fit_eq3: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    from . import workloads as W
    # let the clocks of an idle GPU settle before the first sample (untimed)
    time_batch(make_batch(W, 8192, 64, 262144, args.budget, seed=8999), 200, 50)
    rows = []
    for i, (lp, nd, tot) in enumerate(sample_grid(args.budget)):
        batch = make_batch(W, lp, nd, tot, args.budget, seed=9000 + i)
        ms, wall = time_batch(batch, args.steps, args.warmup)
        rows.append({"l_ctxp": lp, "n_d": nd, "l_ctxd": int(tot), "n_p": args.budget - nd, "ms": ms, "wall_ms": wall})
        print(f"fit_eq3: sample {i + 1}: L_ctxp {lp} n_d {nd} sum L_ctxd {tot}: attention {ms:.4f} ms, append + attention "
              f"wall {wall:.4f} ms", file=sys.stderr, flush=True)
    res, pred = fit(rows)
    res_wall, _ = fit(rows, "wall_ms")
    res.update({"model": "t_chunked = k_ctxp * L_ctxp + k_ctxd * sum(L_ctxd) + b_c (Eq. 3)", "budget_tokens": args.budget,
                "timed": "the kernels of cronus_attn_mixed, first start to last end (HIP events on the dispatches), median",
                "wall_fit": {**res_wall, "timed": "cronus_kv_append of the iteration's tokens + cronus_attn_mixed, host clock"},
                "head_shape": "Hq 32 / Hkv 8 / D 128 / bf16"})
    if args.table:
        for r, p in zip(rows, pred):
            r["model_ms"] = float(p)
        res["table"] = rows
    print(json.dumps(res))


if __name__ == "__main__":
    main()
