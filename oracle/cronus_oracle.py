"""CPU oracle for the mixed-iteration paged attention path (test infrastructure).

This module is TEST INFRASTRUCTURE.  It is a plain, slow, fp64 restatement of what
the GPU library computes, written from the paper's description of the chunked
prefill instance's iteration (Cronus, section 2 "LLM Inference", section 4.2
"Overview", section 4.4 "Chunked prefill", Algorithm 1 for the block granularity).
Only tests, the smoke check and the benchmark's cpu_baseline leg may import it; the
product path never does.  It shares no code with the HIP sources and does not
import the product package.

What is computed
----------------
* ``attn_rows`` / ``attn_mixed``: the definition of attention written out.  A
  sequence has ``prefix_len`` = P keys that were produced elsewhere (the partial
  prefill of section 4.2) and a chunk of C query tokens at absolute positions
  P .. P+C-1 (section 4.2: after the transferred prefix the request continues as
  ordinary chunked prefill; a decode is the case C = 1, section 2).  Query row i of
  head h sees keys 0 .. P+i of KV head h // G, G = Hq / Hkv:

      s_j = sm_scale * <Q[i,h,:], K[j,g,:]>      j = 0 .. P+i
      w_j = exp(s_j - max_j s_j),  Z = sum_j w_j
      out[i,h,:] = (sum_j w_j V[j,g,:]) / Z

  Everything is fp64; a matrix product from the linear-algebra library serves as
  the contraction step, nothing is tiled, no running softmax, no paging.
* ``kv_append`` / ``kv_gather``: pure index arithmetic of the paged layout (blocks
  of N_size = 16 tokens, Algorithm 1) documented in include/cronus.h.
* ``fp8_e4m3_encode`` / ``fp8_e4m3_decode``: software OCP e4m3 quantiser
  (round-to-nearest-even, saturating at +-448).  This format is not in the paper; it
  belongs to the 70B-shaped workload only.
* ``balancer_table`` / ``balancer_split``: Algorithm 1 with Eq. 1-3, as printed
  (appendix A): the per-candidate table and the split it selects.

Pins (tests/test_oracle_pins.py): split-anywhere equals unsplit prefill, rows of
softmax weights sum to one, a scalar brute force, closed forms (L = 1, constant V,
equal keys -> running mean), shift invariance, one-hot limit, decode == chunk of 1,
GQA == MHA with repeated heads, torch's scaled_dot_product_attention in fp64,
scatter/gather inverse with sentinel check, all 256 fp8 codes round trip, fp8
midpoints to even, torch.float8_e4m3fn casts; Algorithm 1: candidate tables worked by
hand (tests/golden/balancer_alg1_cases.txt), linearity of the modelled times inside an
iteration-count class, exhaustive search over the candidates.
"""
from __future__ import annotations

import math

import numpy as np

BLOCK = 16  # N_size: tokens per KV block (Algorithm 1)
CHUNK_ELEMS = 8  # elements per 16-byte (bf16) / 8-byte (fp8) layout chunk


# --------------------------------------------------------------------------- values
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> exact fp64 values."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp64 -> bf16 (nearest, ties to even) and return the bit patterns.

    Done in exact integer arithmetic on the fp64 encoding so that no double rounding
    through fp32 can occur.  Finite inputs in bf16's normal range only.
    """
    x = np.asarray(x, dtype=np.float64)
    sign = np.signbit(x)
    a = np.abs(x)
    out = np.zeros(x.shape, dtype=np.uint16)
    nz = a > 0
    m, e = np.frexp(a[nz])  # a = m * 2**e, m in [0.5, 1)
    # bf16 normal: 1.f * 2**(E-127), 7 fraction bits -> significand as integer in [128, 256)
    q = np.rint(m * 256.0)  # ties-to-even, in [128, 256]
    carry = q >= 256
    q = np.where(carry, 128, q)
    ee = e - 1 + carry.astype(np.int64)  # unbiased exponent of 1.f form
    biased = ee + 127
    if np.any(biased <= 0) or np.any(biased >= 255):
        raise ValueError("value outside bf16 normal range")
    out[nz] = (biased.astype(np.uint16) << np.uint16(7)) | (q.astype(np.uint16) - np.uint16(128))
    out |= sign.astype(np.uint16) << np.uint16(15)
    return out


# ------------------------------------------------------------------------ attention
def attn_rows(q, k, v, prefix_len, sm_scale, rows=None, return_weights=False):
    """Attention of chunk rows of ONE sequence (section 2; section 4.2 hand-off).

    q: [C, Hq, D] fp64 chunk queries (absolute positions prefix_len .. prefix_len+C-1)
    k, v: [L, Hkv, D] fp64 un-paged keys/values, L >= prefix_len + C
    rows: optional 1-D array of chunk-row indices to evaluate (each row is still the
          full definition; this only selects which rows are produced)
    returns out [len(rows), Hq, D] fp64 (and the weights [len(rows), Hq, L] if asked)
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    C, Hq, D = q.shape
    L, Hkv, Dk = k.shape
    if Dk != D or v.shape != k.shape:
        raise ValueError("shape mismatch")
    if Hq % Hkv:
        raise ValueError("Hq must be a multiple of Hkv")
    if L < prefix_len + C:
        raise ValueError("not enough keys for prefix+chunk")
    G = Hq // Hkv
    rows = np.arange(C) if rows is None else np.asarray(rows, dtype=np.int64)
    last_visible = prefix_len + rows  # key j visible to row i iff j <= P + i
    nkeys = int(last_visible.max()) + 1 if rows.size else 0
    hidden = np.arange(nkeys)[None, :] > last_visible[:, None]
    out = np.empty((rows.size, Hq, D), dtype=np.float64)
    weights = np.zeros((rows.size, Hq, L), dtype=np.float64) if return_weights else None
    for h in range(Hq):
        g = h // G
        s = sm_scale * (q[rows, h, :] @ k[:nkeys, g, :].T)
        s[hidden] = -np.inf
        w = np.exp(s - s.max(axis=1, keepdims=True))
        z = w.sum(axis=1, keepdims=True)
        out[:, h, :] = (w @ v[:nkeys, g, :]) / z
        if return_weights:
            weights[:, h, :nkeys] = w / z
    return (out, weights) if return_weights else out


def attn_mixed(q, k_seqs, v_seqs, prefix_lens, chunk_lens, sm_scale):
    """One mixed iteration (section 4.4: a batch of chunked prefill and decodes).

    q: [total_q, Hq, D] fp64, the chunk rows of all sequences back to back in batch
    order; k_seqs[s], v_seqs[s]: [L_s, Hkv, D] fp64 with L_s = prefix+chunk.
    Returns out [total_q, Hq, D] fp64.
    """
    q = np.asarray(q, dtype=np.float64)
    out = np.empty_like(q)
    off = 0
    for s, (p, c) in enumerate(zip(prefix_lens, chunk_lens)):
        p, c = int(p), int(c)
        if c == 0:
            continue
        out[off:off + c] = attn_rows(q[off:off + c], k_seqs[s][:p + c], v_seqs[s][:p + c], p, sm_scale)
        off += c
    if off != q.shape[0]:
        raise ValueError("sum(chunk_lens) != total_q")
    return out


# ---------------------------------------------------------------- paged cache layout
def k_elem_offset(block, head, slot, d, n_kv_heads, head_dim):
    """Element offset of K[token in `slot` of `block`, head, d] in the K pool.

    Layout [num_blocks][Hkv][D/8][16][8]: a 16-byte chunk holds 8 consecutive d of
    one token; the 16 tokens of a block are adjacent for a given chunk index.
    """
    return (((block * n_kv_heads + head) * (head_dim // CHUNK_ELEMS) + d // CHUNK_ELEMS) * BLOCK
            + slot) * CHUNK_ELEMS + d % CHUNK_ELEMS


def v_elem_offset(block, head, slot, d, n_kv_heads, head_dim):
    """Element offset of V[token in `slot` of `block`, head, d] in the V pool.

    Layout [num_blocks][Hkv][2][D][8]: a chunk holds 8 consecutive tokens of one d.
    """
    return (((block * n_kv_heads + head) * (BLOCK // CHUNK_ELEMS) + slot // CHUNK_ELEMS) * head_dim
            + d) * CHUNK_ELEMS + slot % CHUNK_ELEMS


def kv_append(k_pool, v_pool, k_src, v_src, cu_tokens, start_pos, block_tables, n_kv_heads, head_dim):
    """Scatter rows of k_src/v_src [n_tokens, Hkv, D] into flat pools, in place.

    Token t (0-based within sequence s's rows) goes to logical position
    start_pos[s] + t, i.e. block block_tables[s][pos // 16], slot pos % 16
    (Algorithm 1: the cache is counted in blocks of N_size tokens).  The prefix
    hand-off of section 4.2 is the call with start_pos = 0; appending an
    iteration's new tokens is the call with start_pos = tokens already cached.
    Pools are 1-D arrays of codes (uint16 bf16 bits, or uint8 fp8 codes).
    """
    Hkv, D = n_kv_heads, head_dim
    heads = np.arange(Hkv)[None, :, None]
    ds = np.arange(D)[None, None, :]
    for s in range(len(start_pos)):
        t0, t1 = int(cu_tokens[s]), int(cu_tokens[s + 1])
        if t1 == t0:
            continue
        pos = int(start_pos[s]) + np.arange(t1 - t0)  # logical positions of the rows
        blk = np.asarray(block_tables[s])[pos // BLOCK].astype(np.int64)[:, None, None]
        slot = (pos % BLOCK)[:, None, None]
        k_pool[k_elem_offset(blk, heads, slot, ds, Hkv, D)] = k_src[t0:t1]
        v_pool[v_elem_offset(blk, heads, slot, ds, Hkv, D)] = v_src[t0:t1]


def kv_gather(k_pool, v_pool, table_row, length, n_kv_heads, head_dim):
    """Inverse of kv_append for one sequence: un-paged K, V [length, Hkv, D] codes."""
    Hkv, D = n_kv_heads, head_dim
    pos = np.arange(length)
    blk = np.asarray(table_row)[pos // BLOCK].astype(np.int64)[:, None, None]
    slot = (pos % BLOCK)[:, None, None]
    heads = np.arange(Hkv)[None, :, None]
    ds = np.arange(D)[None, None, :]
    k = k_pool[k_elem_offset(blk, heads, slot, ds, Hkv, D)]
    v = v_pool[v_elem_offset(blk, heads, slot, ds, Hkv, D)]
    return k, v


# ------------------------------------------------------------------------- fp8 e4m3
FP8_MAX = 448.0


def fp8_e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """OCP e4m3 (finite-only variant: no infinities, 0x7f/0xff = NaN) -> fp64."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = c & 0x7
    normal = np.ldexp(1.0 + m / 8.0, e - 7)
    sub = np.ldexp(m / 8.0, -6)
    val = np.where(e == 0, sub, normal)
    val = np.where((e == 15) & (m == 7), np.nan, val)
    return sign * val


def fp8_e4m3_encode(x_f32: np.ndarray, scale_f32) -> np.ndarray:
    """Quantise: code = RNE_e4m3(clamp(fp32(x) / fp32(scale), -448, 448)).

    The division is a single IEEE fp32 division (the GPU side does the same), the
    rounding to the 3-bit significand is nearest-even done on exact values,
    subnormals are kept, the sign of zero is kept, |y| >= 448 saturates to 0x7e.
    """
    x = np.asarray(x_f32, dtype=np.float32)
    y = (x / np.float32(scale_f32)).astype(np.float32).astype(np.float64)
    sign = np.signbit(y).astype(np.uint8) << np.uint8(7)
    a = np.minimum(np.abs(y), FP8_MAX)
    code = np.zeros(a.shape, dtype=np.int64)
    small = a < 2.0 ** -6
    # subnormal grid: multiples of 2**-9; a result of 8 is the smallest normal (code 8)
    code[small] = np.rint(a[small] * 2.0 ** 9).astype(np.int64)
    big = ~small
    m, e = np.frexp(a[big])  # a = m * 2**e, m in [0.5, 1)  ->  1.f * 2**(e-1)
    q = np.rint(m * 16.0).astype(np.int64)  # in [8, 16]
    carry = q == 16
    q = np.where(carry, 8, q)
    ee = e - 1 + carry
    code[big] = ((ee + 7) << 3) | (q - 8)
    code = np.minimum(code, 0x7E)
    return code.astype(np.uint8) | sign


# ------------------------------------------------------------- Algorithm 1 / Eq. 1-3
def balancer_table(l_in, n_d, l_ctxd, k_p, b_p, k_ctxp, k_ctxd, b_c, batch_tokens=512, n_candidates=512):
    """The candidate table of Algorithm 1 (appendix A): one row per candidate j = 1 ..
    n_candidates, (L_p, N_iter, L_last, T_prefill, T_chunked), in the algorithm's order.

    L_p = ceil(j / n_candidates * L_in); T_prefill from Eq. 2; n_p = B - n_d prefill tokens
    per iteration; L_c = L_in - L_p tokens are left for the chunked prefill instance, which
    needs N_iter = ceil(L_c / n_p) iterations, the last of them with prefill context
    L_last = L_p + floor(L_c / n_p) * n_p; T_chunked is N_iter times the Eq. 3 iteration time
    at the mean context (L_in + L_last) / 2, as the algorithm prints it (Eq. 1 states the mean
    of the first and last iteration times; the printed form is kept).
    """
    if not 0 <= n_d < batch_tokens:
        raise ValueError("n_d must lie in [0, batch_tokens): an iteration needs at least one prefill token")
    if l_in <= 0 or n_candidates <= 0:
        raise ValueError("l_in and n_candidates must be positive")
    n_p = batch_tokens - n_d
    rows = []
    for j in range(1, n_candidates + 1):
        l_p = -(-j * l_in // n_candidates)  # ceil(j/512 * L_in) in integers
        t_prefill = k_p * l_p + b_p
        l_c = l_in - l_p
        n_iter = -(-l_c // n_p)
        l_last = l_p + (l_c // n_p) * n_p
        t_chunked = n_iter * (k_ctxp * (l_in + l_last) / 2.0 + k_ctxd * l_ctxd + b_c)
        rows.append((l_p, n_iter, l_last, t_prefill, t_chunked))
    return rows


def balancer_split(l_in, n_d, l_ctxd, n_free, k_p, b_p, k_ctxp, k_ctxd, b_c,
                   n_size=BLOCK, batch_tokens=512, n_candidates=512):
    """Partial prefill length chosen by Algorithm 1 (appendix A) with Eq. 2 and Eq. 3.

    Reading of the garbled symbols: n_d = number of decode requests on the chunked
    prefill instance, l_ctxd = sum of their context lengths, n_free = its free KV
    blocks.  The printed T_chunked uses (L_in + L_last)/2 as the mean prefill
    context, which is kept as printed.  Too few free blocks for the whole prompt:
    the prompt is prefilled entirely on the partial prefill instance (L_p = L_in).
    """
    if not 0 <= n_d < batch_tokens:
        raise ValueError("n_d must lie in [0, batch_tokens): an iteration needs at least one prefill token")
    if n_free < -(-l_in // n_size):
        return l_in
    best, best_gap = None, None
    for l_p, _, _, t_prefill, t_chunked in balancer_table(l_in, n_d, l_ctxd, k_p, b_p, k_ctxp, k_ctxd, b_c,
                                                          batch_tokens, n_candidates):
        gap = abs(t_prefill - t_chunked)
        if best_gap is None or gap < best_gap:  # argmin takes the first minimum
            best, best_gap = l_p, gap
    return best
