#!/usr/bin/env python3
"""Prefix ingest overlapped with the attention of other requests (Cronus section 4.2: the
KV cache of a partially prefilled request arrives while the chunked prefill instance keeps
computing decodes and chunks of the requests it already has).

The running requests and the newcomers share one paged pool.  The running batch's
cronus_attn_mixed goes to one stream, the newcomers' cronus_kv_append to a second stream
(default priority both); the source of the append is a device buffer standing in for the
receive buffer, or pinned host memory copied to such a buffer on the same side stream.
`measure()` times each call alone and both together.

    python -m paper_2509_17357_amd.overlap [--source device|pinned] [--steps 20]
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np
import torch

from . import binding as B
from . import workloads as W
from .runtime import DeviceIteration


class OverlapRun:
    def __init__(self, shape, run_prefix, run_chunk, new_prefix, seed, source="device", host_inputs=False,
                 pool_fill=None):
        self.n_run, self.n_new = len(run_prefix), len(new_prefix)
        # newcomers go last, typed like decodes so that their prefix rows are the tail of the context rows
        self.batch = W.custom_batch(shape, list(run_prefix) + list(new_prefix), list(run_chunk) + [1] * self.n_new, seed)
        it = self.it = DeviceIteration(self.batch, pool_fill=pool_fill)
        self.kv_bits = it.load_host_inputs() if host_inputs else it.load_device_inputs()
        if it.fp8:
            it.set_fp8_scales(*it.amax_scales())
        it.setup_decode_context()
        it.ingest_prefix()
        it.append_new()
        dev = it.device
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
        P, C = self.batch.prefix_lens.astype(np.int64), self.batch.chunk_lens.astype(np.int64)
        self.P_run, self.C_run = P[:self.n_run].astype(np.int32), C[:self.n_run].astype(np.int32)
        nq = int(C[:self.n_run].sum())
        self.q_run, self.out_run = it.q[:nq], it.out[:nq]
        self.bt_run, self.bt_new = it.block_tables[:self.n_run], it.block_tables[self.n_run:]
        need = B.cronus_attn_mixed_workspace_bytes(it.cache, self.P_run, self.C_run)
        self.workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
        self.workspace_bytes = need
        off = int(P[:self.n_run][C[:self.n_run] == 1].sum())  # context rows of the running decodes come first
        self.n_ingest = int(P[self.n_run:].sum())
        self.src_k, self.src_v = it.ctx_k[off:off + self.n_ingest], it.ctx_v[off:off + self.n_ingest]
        self.cu_ingest = i32(np.concatenate([[0], np.cumsum(P[self.n_run:])]))
        self.zero = i32(np.zeros(self.n_new))
        self.source = source
        if source == "pinned":
            self.host_k = torch.empty(self.src_k.shape, dtype=self.src_k.dtype, pin_memory=True)
            self.host_v = torch.empty(self.src_v.shape, dtype=self.src_v.dtype, pin_memory=True)
            self.host_k.copy_(self.src_k)
            self.host_v.copy_(self.src_v)
            self.stage_k, self.stage_v = torch.empty_like(self.src_k), torch.empty_like(self.src_v)
        elif source != "device":
            raise ValueError(source)
        self.side = torch.cuda.Stream(device=dev)  # default priority
        torch.cuda.synchronize()

    def attention(self, stream):
        it = self.it
        return B.cronus_attn_mixed(it.cache, self.q_run, self.out_run, self.P_run, self.C_run, self.bt_run,
                                   self.batch.max_blocks, it.sm_scale, self.workspace, self.workspace_bytes,
                                   stream.cuda_stream)

    def ingest(self, stream):
        it = self.it
        k, v = self.src_k, self.src_v
        if self.source == "pinned":
            with torch.cuda.stream(stream):
                self.stage_k.copy_(self.host_k, non_blocking=True)
                self.stage_v.copy_(self.host_v, non_blocking=True)
            k, v = self.stage_k, self.stage_v
        return B.cronus_kv_append(it.cache, k, v, self.cu_ingest, self.zero, self.bt_new, self.batch.max_blocks,
                                  self.n_new, self.n_ingest, stream.cuda_stream)

    def _timed(self, fn_main, fn_side, steps):
        main = torch.cuda.current_stream(self.it.device)
        ev = lambda: torch.cuda.Event(enable_timing=True)
        m0, m1, s0, s1 = ev(), ev(), ev(), ev()
        torch.cuda.synchronize()
        self.side.wait_stream(main)
        t0 = time.perf_counter()
        if fn_main:
            m0.record(main)
        if fn_side:
            s0.record(self.side)
        for _ in range(steps):
            if fn_side:
                fn_side(self.side)
            if fn_main:
                fn_main(main)
        if fn_main:
            m1.record(main)
        if fn_side:
            s1.record(self.side)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        return (wall, m0.elapsed_time(m1) / steps if fn_main else None, s0.elapsed_time(s1) / steps if fn_side else None)

    def measure(self, steps=20, warmup=3):
        for _ in range(warmup):
            self.attention(torch.cuda.current_stream(self.it.device))
            self.ingest(self.side)
        torch.cuda.synchronize()
        _, attn_alone, _ = self._timed(self.attention, None, steps)
        _, _, ingest_alone = self._timed(None, self.ingest, steps)
        wall, attn_both, ingest_both = self._timed(self.attention, self.ingest, steps)
        sh = self.batch.shape
        esz = 1 if self.it.fp8 else 2
        ingest_bytes = self.n_ingest * sh.n_kv_heads * sh.head_dim * 2 * (2 + esz)  # bf16 source read + cache write, K and V
        return {"attn_alone_ms": attn_alone, "ingest_alone_ms": ingest_alone, "attn_overlapped_ms": attn_both,
                "ingest_overlapped_ms": ingest_both, "both_wall_ms": wall, "serial_sum_ms": attn_alone + ingest_alone,
                "ingest_tokens": self.n_ingest, "ingest_gbs_alone": ingest_bytes / (ingest_alone * 1e-3) / 1e9,
                "source": self.source, "running_q_tokens": int(self.C_run.sum()),
                "running_kv_tokens": int((self.P_run + self.C_run).sum())}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--source", default="device", choices=["device", "pinned"])
    ap.add_argument("--steps", type=int, default=20)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("overlap: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    out = {}
    # running batch shaped like the Llama-3-8B benchmark batch; newcomers: 4 prefixes of about 2k tokens
    b = W.draw_batch(2)
    rng = np.random.default_rng(77)
    for name, new in (("4x2k", rng.integers(1500, 2500, 4).tolist()), ("16x4k", rng.integers(3000, 5000, 16).tolist())):
        run = OverlapRun(b.shape, b.prefix_lens.tolist(), b.chunk_lens.tolist(), new, seed=8100, source=args.source)
        out[name] = run.measure(steps=args.steps)
        del run
        torch.cuda.empty_cache()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
