"""Device-side plumbing for one mixed iteration: torch tensors for memory and streams,
every computation through the C ABI (binding.py).  No oracle, no fallback.

The hot path of one iteration (Cronus section 4.2 and 4.4) is, in order:
  1. ingest_prefix  - cronus_kv_append of the transferred prefix KV of the continuation
                      chunks (start_pos = 0)
  2. append_new     - cronus_kv_append of this iteration's K/V rows (start_pos = prefix)
  3. attention      - cronus_attn_mixed over chunks and decodes
The contexts of the decode requests were cached by earlier iterations; here they are
placed by setup_decode_context(), which is set-up, not part of the iteration.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from .workloads import Batch


def bf16_tensor_from_bits(bits: np.ndarray, device) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def bits_from_bf16_tensor(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class DeviceIteration:
    """Device buffers of one batch and the three calls of the hot path."""

    def __init__(self, batch: Batch, device="cuda:0", pool_fill: int | None = None):
        self.batch = batch
        self.device = torch.device(device)
        sh = batch.shape
        self.fp8 = sh.kv_dtype == "fp8"
        self.elems_per_block = sh.n_kv_heads * 16 * sh.head_dim
        pool_dtype = torch.uint8 if self.fp8 else torch.int16
        n = batch.num_blocks * self.elems_per_block
        if pool_fill is None:
            self.k_pool = torch.empty(n, dtype=pool_dtype, device=self.device)
            self.v_pool = torch.empty(n, dtype=pool_dtype, device=self.device)
        else:
            self.k_pool = torch.full((n,), pool_fill, dtype=pool_dtype, device=self.device)
            self.v_pool = torch.full((n,), pool_fill, dtype=pool_dtype, device=self.device)
        self.block_tables = torch.from_numpy(np.ascontiguousarray(batch.block_tables)).to(self.device)
        self.k_scale = self.v_scale = None
        self.q = self.out = None
        self.prefix_k = self.prefix_v = self.new_k = self.new_v = None
        P, C = batch.prefix_lens.astype(np.int64), batch.chunk_lens.astype(np.int64)
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(self.device)
        is_dec = C == 1
        self.cu_prefix = i32(np.concatenate([[0], np.cumsum(np.where(is_dec, 0, P))]))  # chunk sequences only
        self.cu_ctx = i32(np.concatenate([[0], np.cumsum(np.where(is_dec, P, 0))]))     # decode sequences only
        self.n_ctx_tokens = int(P[is_dec].sum())
        self.ctx_k = self.ctx_v = None
        self.cu_new = i32(np.concatenate([[0], np.cumsum(C)]))
        self.zero_pos = i32(np.zeros(batch.n_seqs))
        self.prefix_pos = i32(P)
        self.n_prefix_tokens = int(P[~is_dec].sum())
        self.n_new_tokens = int(C.sum())
        self.sm_scale = 1.0 / float(np.sqrt(sh.head_dim))
        self._cache = None
        self.workspace = None
        self.workspace_bytes = 0

    # ---- inputs
    def load_host_inputs(self, kv=None):
        """Tensors drawn on the host by the seeded generators (bit-identical to what the
        oracle side sees).  Returns the per-sequence (k_bits, v_bits) for the caller, who
        may also pass them in (drawn already, e.g. by several threads)."""
        b = self.batch
        if kv is None:
            kv = [b.gen_kv(s) for s in range(b.n_seqs)]
        P = b.prefix_lens
        sh = b.shape
        empty = np.zeros((0, sh.n_kv_heads, sh.head_dim), dtype=np.uint16)
        cat = lambda xs: np.concatenate(xs) if xs else empty
        dec = b.chunk_lens == 1
        self.prefix_k = bf16_tensor_from_bits(cat([k[:P[s]] for s, (k, v) in enumerate(kv) if not dec[s]]), self.device)
        self.prefix_v = bf16_tensor_from_bits(cat([v[:P[s]] for s, (k, v) in enumerate(kv) if not dec[s]]), self.device)
        self.ctx_k = bf16_tensor_from_bits(cat([k[:P[s]] for s, (k, v) in enumerate(kv) if dec[s]]), self.device)
        self.ctx_v = bf16_tensor_from_bits(cat([v[:P[s]] for s, (k, v) in enumerate(kv) if dec[s]]), self.device)
        self.new_k = bf16_tensor_from_bits(cat([k[P[s]:] for s, (k, v) in enumerate(kv)]), self.device)
        self.new_v = bf16_tensor_from_bits(cat([v[P[s]:] for s, (k, v) in enumerate(kv)]), self.device)
        self.q = bf16_tensor_from_bits(b.gen_q(), self.device)
        self.out = torch.zeros_like(self.q)
        return kv

    def load_device_inputs(self, seed=0):
        """Same distribution drawn on the device (benchmarks of the full-size batches)."""
        sh = self.batch.shape
        g = torch.Generator(device=self.device)
        g.manual_seed(int(self.batch.seed) * 7919 + seed)
        mk = lambda n: (torch.randn((n, sh.n_kv_heads, sh.head_dim), generator=g, device=self.device,
                                    dtype=torch.float32) * 0.125).to(torch.bfloat16)
        self.prefix_k, self.prefix_v = mk(self.n_prefix_tokens), mk(self.n_prefix_tokens)
        self.ctx_k, self.ctx_v = mk(self.n_ctx_tokens), mk(self.n_ctx_tokens)
        self.new_k, self.new_v = mk(self.n_new_tokens), mk(self.n_new_tokens)
        self.q = (torch.randn((self.n_new_tokens, sh.n_q_heads, sh.head_dim), generator=g, device=self.device,
                              dtype=torch.float32) * 0.125).to(torch.bfloat16)
        self.out = torch.zeros_like(self.q)

    def set_fp8_scales(self, k_scale: np.ndarray, v_scale: np.ndarray):
        self.k_scale = torch.from_numpy(np.ascontiguousarray(k_scale, dtype=np.float32)).to(self.device)
        self.v_scale = torch.from_numpy(np.ascontiguousarray(v_scale, dtype=np.float32)).to(self.device)
        self._cache = None

    def amax_scales(self):
        """Per-KV-head scale = amax / 448 in fp32 over the tensors about to be cached."""
        def amax(a, b, c):
            x = torch.cat([t.abs().amax(dim=(0, 2))[None] for t in (a, b, c) if t.shape[0]]).amax(dim=0)
            return (x.to(torch.float32) / 448.0).cpu().numpy().astype(np.float32)
        return amax(self.prefix_k, self.new_k, self.ctx_k), amax(self.prefix_v, self.new_v, self.ctx_v)

    # ---- the C ABI calls
    @property
    def cache(self) -> B.cronus_kv_cache:
        if self._cache is None:
            sh = self.batch.shape
            self._cache = B.make_cache(self.k_pool, self.v_pool, self.batch.num_blocks, sh.n_q_heads, sh.n_kv_heads,
                                       sh.head_dim, B.CRONUS_KV_FP8_E4M3 if self.fp8 else B.CRONUS_KV_BF16,
                                       self.k_scale, self.v_scale)
        return self._cache

    def _stream(self):
        return torch.cuda.current_stream(self.device).cuda_stream

    def setup_decode_context(self):
        """Set-up: the KV that earlier iterations of the decode requests left in the cache."""
        b = self.batch
        return B.cronus_kv_append(self.cache, self.ctx_k, self.ctx_v, self.cu_ctx, self.zero_pos,
                                  self.block_tables, b.max_blocks, b.n_seqs, self.n_ctx_tokens, self._stream())

    def ingest_prefix(self):
        """Hot path: the transferred prefix of every continuation chunk."""
        b = self.batch
        return B.cronus_kv_append(self.cache, self.prefix_k, self.prefix_v, self.cu_prefix, self.zero_pos,
                                  self.block_tables, b.max_blocks, b.n_seqs, self.n_prefix_tokens, self._stream())

    def append_new(self):
        b = self.batch
        return B.cronus_kv_append(self.cache, self.new_k, self.new_v, self.cu_new, self.prefix_pos,
                                  self.block_tables, b.max_blocks, b.n_seqs, self.n_new_tokens, self._stream())

    def ensure_workspace(self):
        """Workspace for this batch's lengths (sized once: the lengths of a batch do not change)."""
        if self.workspace is None:
            need = B.cronus_attn_mixed_workspace_bytes(self.cache, self.batch.prefix_lens, self.batch.chunk_lens)
            if need == 0:
                raise RuntimeError("cronus_attn_mixed_workspace_bytes rejected the batch")
            self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
            self.workspace_bytes = need
        return self.workspace_bytes

    def attention(self):
        b = self.batch
        self.ensure_workspace()
        return B.cronus_attn_mixed(self.cache, self.q, self.out, b.prefix_lens, b.chunk_lens, self.block_tables,
                                   b.max_blocks, self.sm_scale, self.workspace, self.workspace_bytes, self._stream())

    def step(self):
        """One pass of the whole hot path (after setup_decode_context())."""
        self.ingest_prefix()
        self.append_new()
        self.attention()
