"""Seeded synthetic inputs for the mixed-iteration attention path.

Holds no arithmetic of the method: only random draws of lengths, block tables and
bf16 tensors shaped like the workloads of the chunked prefill instance (Cronus,
section 4.4: one iteration batches continuation chunks with decodes; section 5.1:
the Azure conversation trace, which is not available and which these draws stand in
for).  Both the tests of the CPU oracle and the GPU harness draw from here, so the
two sides see identical inputs.

All tensors are bf16 bit patterns in numpy uint16 arrays: x = bf16(N(0,1) * 0.125).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BLOCK = 16


@dataclass(frozen=True)
class HeadShape:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    kv_dtype: str = "bf16"  # "bf16" or "fp8"


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape, sigma=0.125) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    x *= np.float32(sigma)
    return f32_to_bf16_bits(x)


@dataclass
class Batch:
    name: str
    shape: HeadShape
    prefix_lens: np.ndarray  # int32 [n_seqs]
    chunk_lens: np.ndarray  # int32 [n_seqs]
    seed: int
    pool_factor: float = 1.25
    block_tables: np.ndarray = field(default=None)  # int32 [n_seqs, max_blocks], -1 padded
    num_blocks: int = 0

    def __post_init__(self):
        self.prefix_lens = np.asarray(self.prefix_lens, dtype=np.int32)
        self.chunk_lens = np.asarray(self.chunk_lens, dtype=np.int32)
        if self.block_tables is None:
            self._draw_tables()

    # ---- derived sizes
    @property
    def n_seqs(self):
        return int(self.prefix_lens.size)

    @property
    def kv_lens(self):
        return (self.prefix_lens + self.chunk_lens).astype(np.int64)

    @property
    def total_q(self):
        return int(self.chunk_lens.sum())

    @property
    def cu_q(self):
        return np.concatenate([[0], np.cumsum(self.chunk_lens)]).astype(np.int32)

    @property
    def max_blocks(self):
        return int(self.block_tables.shape[1])

    def blocks_needed(self):
        return (self.kv_lens + BLOCK - 1) // BLOCK

    def _draw_tables(self):
        """Physical block ids: one seeded permutation of a pool >= pool_factor x the
        blocks in use, dealt jointly over all sequences, so consecutive logical blocks
        of a sequence are neither adjacent nor ordered, and sequences interleave."""
        need = self.blocks_needed()
        total = int(need.sum())
        self.num_blocks = max(int(np.ceil(total * self.pool_factor)), total + 1)
        rng = np.random.default_rng([self.seed, 0xB10C])
        ids = rng.permutation(self.num_blocks)[:total].astype(np.int32)
        # deal ids round-robin-free: shuffle the (seq, logical) slots too
        slots = np.concatenate([np.stack([np.full(n, s), np.arange(n)], 1) for s, n in enumerate(need)])
        order = rng.permutation(total)
        mb = max(int(need.max()), 1)
        bt = np.full((self.n_seqs, mb), -1, dtype=np.int32)
        bt[slots[order, 0], slots[order, 1]] = ids
        self.block_tables = bt

    # ---- tensors
    def gen_q(self) -> np.ndarray:
        rng = np.random.default_rng([self.seed, 0x51])
        s = self.shape
        return normal_bf16(rng, (self.total_q, s.n_q_heads, s.head_dim))

    def gen_kv(self, s: int):
        """K, V bf16 bits [L_s, Hkv, D] of sequence s (independent stream per sequence)."""
        rng = np.random.default_rng([self.seed, 0x6B, int(s)])
        sh = self.shape
        L = int(self.kv_lens[s])
        k = normal_bf16(rng, (L, sh.n_kv_heads, sh.head_dim))
        v = normal_bf16(rng, (L, sh.n_kv_heads, sh.head_dim))
        return k, v

    # ---- algorithmic work (visible pairs only)
    def visible_pairs(self) -> int:
        p = self.prefix_lens.astype(np.int64)
        c = self.chunk_lens.astype(np.int64)
        return int((c * p + c * (c + 1) // 2).sum())

    def flops(self) -> int:
        return 4 * self.shape.head_dim * self.shape.n_q_heads * self.visible_pairs()

    def attn_bytes(self) -> int:
        """KV read once per sequence + Q read + O write + block-table entries used."""
        sh = self.shape
        esz = 2 if sh.kv_dtype == "bf16" else 1
        kv = int(self.kv_lens.sum()) * 2 * sh.n_kv_heads * sh.head_dim * esz
        qo = self.total_q * sh.n_q_heads * sh.head_dim * 2 * 2
        tables = int(self.blocks_needed().sum()) * 4 + self.n_seqs * 8
        return kv + qo + tables


SHAPE_TINY = HeadShape(8, 2, 64)
SHAPE_8B = HeadShape(32, 8, 128)
SHAPE_70B = HeadShape(64, 8, 128, "fp8")

CONFIG_NAMES = {1: "tiny", 2: "llama3_8b", 3: "prefill_heavy", 4: "decode_heavy", 5: "llama_70b_fp8"}


def config_seed(config_id: int, trial: int = 0) -> int:
    return 1000 * config_id + trial


def draw_batch(config_id: int, trial: int = 0, shuffle: bool = False, scale: float = 1.0) -> Batch:
    """One of the five benchmark batches.  Order: chunk sequences, then decodes
    (shuffle=True permutes the batch order).  `scale` < 1 shrinks every length by that
    factor (for CPU-sized variants of the same structure); 1.0 is the full size."""
    seed = config_seed(config_id, trial)
    rng = np.random.default_rng([seed, 0x1E])

    def U(lo, hi, n):
        return rng.integers(lo, hi, size=n, endpoint=True)

    def sc(x):
        return np.maximum(1, np.floor(np.asarray(x) * scale)).astype(np.int64)

    if config_id == 1:
        shape = SHAPE_TINY
        P = np.array([192] + [255] * 4)
        C = np.array([64] + [1] * 4)
    elif config_id == 2:
        shape = SHAPE_8B
        P = np.concatenate([U(512, 2048, 4), U(256, 4096, 64) - 1])
        C = np.array([512] * 4 + [1] * 64)
    elif config_id == 3:
        shape = SHAPE_8B
        N = U(4096, 8192, 8)
        f = rng.uniform(0.25, 0.75, size=8)
        Pc = np.floor(f * N).astype(np.int64)
        Cc = np.minimum(N - Pc, 2048)
        P = np.concatenate([Pc, U(512, 2048, 16) - 1])
        C = np.concatenate([Cc, [1] * 16])
    elif config_id == 4:
        shape = SHAPE_8B
        # batch order is chunks first: the single chunk, then the 256 decodes
        P = np.concatenate([[1024], U(1024, 8192, 256) - 1])
        C = np.array([256] + [1] * 256)
    elif config_id == 5:
        shape = SHAPE_70B
        P = np.concatenate([[28672] * 2, U(4096, 16384, 128) - 1])
        C = np.array([4096] * 2 + [1] * 128)
    else:
        raise ValueError("config_id must be 1..5")
    if scale != 1.0:
        dec = C == 1
        L = sc(P + C)
        C = np.where(dec, 1, np.minimum(sc(C), L))
        P = L - C
    if shuffle:
        order = rng.permutation(P.size)
        P, C = P[order], C[order]
    return Batch(CONFIG_NAMES[config_id], shape, P, C, seed)


def paper_iteration(prefill_ctx: int, decode_ctxs, budget: int = 512, seed: int = 7,
                    shape: HeadShape = SHAPE_8B) -> Batch:
    """The iteration of section 4.4 / Algorithm 1: a token budget B (512 in section
    5.1), n_d decodes, and one continuation chunk of n_p = B - n_d tokens whose
    context (keys already cached) is prefill_ctx."""
    decode_ctxs = np.asarray(decode_ctxs, dtype=np.int64)
    n_p = budget - decode_ctxs.size
    P = np.concatenate([[prefill_ctx], decode_ctxs - 1])
    C = np.concatenate([[n_p], np.ones(decode_ctxs.size, dtype=np.int64)])
    return Batch("paper_iteration", shape, P, C, seed)


def custom_batch(shape: HeadShape, prefix_lens, chunk_lens, seed: int, name="custom") -> Batch:
    return Batch(name, shape, prefix_lens, chunk_lens, seed)


def stress_qkv(kind: str, seed: int, C: int, L: int, shape: HeadShape):
    """Inputs outside the benign N(0,1)/8 regime, as bf16 bits (q [C,Hq,D], k, v [L,Hkv,D]).
    The C query rows sit at positions L-C .. L-1, so keys 0 .. L-C are visible to all of them.

    peaky         : Q x 16, sharply peaked softmax
    outlier       : one key per kv head (random position) with a huge logit against every query
    outlier_last  : that key sits three keys before the first query row's causal end: it arrives
                    late in every row's stream of keys (in the last span of a split item)
    outlier_first : that key is key 2: the peak lies in the first span only
    monotone      : logits increasing gently with key position (about 20 bits over the context)
    ramp_up       : logits rising by about 7 bits per 32 keys (the running maximum outgrows any
                    reference within two sub-tiles, all the way through the context)
    ramp_down     : the same ramp falling: the maximum comes first, later weights underflow
    equal         : all keys identical (uniform weights over the visible keys)
    """
    rng = np.random.default_rng([seed, 0x57])
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    q = rng.standard_normal((C, Hq, D), dtype=np.float32) * np.float32(0.125)
    # random K/V rows are drawn for at most 2048 keys and repeated along a longer context (cheap
    # at 100 k keys); everything is assembled as bf16 bit patterns, never as fp32 of full length
    base = min(L, 2048)
    draw = lambda: np.resize(f32_to_bf16_bits(rng.standard_normal((base, Hkv, D), dtype=np.float32) * np.float32(0.125)),
                             (L, Hkv, D))
    k, v = draw(), draw()
    per_key = lambda t: np.broadcast_to(f32_to_bf16_bits(t.astype(np.float32))[:, None, None], (L, Hkv, D)).copy()
    if kind == "peaky":
        q *= np.float32(16.0)
    elif kind in ("outlier", "outlier_last", "outlier_first"):
        q = np.abs(q) + np.float32(0.25)
        if kind == "outlier":
            j = rng.integers(0, L, size=Hkv)
        elif kind == "outlier_last":
            j = np.full(Hkv, max(L - C - 3, 0))
        else:
            j = np.full(Hkv, min(2, L - 1))
        for g in range(Hkv):
            k[j[g], g, :] = f32_to_bf16_bits(np.float32(4.0))
    elif kind == "monotone":
        q = np.abs(q) + np.float32(0.5)
        k = per_key(np.arange(L, dtype=np.float32) / np.float32(max(L - 1, 1)) * np.float32(2.0))
    elif kind in ("ramp_up", "ramp_down"):
        # q = 4 in every dim, k = t(j) in every dim: logit = sm_scale * 4 D t(j); in log2 units
        # (x log2 e, sm_scale = 1/sqrt(D)) a slope of 7/32 per key needs t' = 7 / (32 * 4 * sqrt(D) * 1.4427)
        q = np.full((C, Hq, D), 4.0, dtype=np.float32)
        step = np.float32(7.0 / (32.0 * 4.0 * np.sqrt(D) * 1.4427))
        pos = np.arange(L, dtype=np.float32)
        k = per_key((pos[::-1] if kind == "ramp_down" else pos) * step)
    elif kind == "equal":
        k = np.broadcast_to(k[:1], (L, Hkv, D)).copy()
    else:
        raise ValueError(kind)
    return f32_to_bf16_bits(q), k, v
