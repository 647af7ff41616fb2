"""Helpers of the GPU parity tests: run the HIP path through the C ABI, compute the
fp64 oracle on the same seeded inputs, and measure the error the way the tolerance is
stated (max-abs <= 2e-2 and relative L2 <= 1e-2, overall and per sequence)."""
from __future__ import annotations

import functools

import numpy as np

from oracle import cronus_oracle as orc

MAX_ABS_TOL = 2e-2
REL_L2_TOL = 1e-2


def oracle_pools(batch, kv_bits, fill=0xDEAD, k_scale=None, v_scale=None):
    """Pool images the scatter must produce (prefix ingest, then new tokens)."""
    sh = batch.shape
    n = batch.num_blocks * sh.n_kv_heads * 16 * sh.head_dim
    fp8 = sh.kv_dtype == "fp8"
    dt = np.uint8 if fp8 else np.uint16
    kp = np.full(n, fill & (0xFF if fp8 else 0xFFFF), dtype=dt)
    vp = kp.copy()
    P, C = batch.prefix_lens, batch.chunk_lens

    def codes(bits, scale):
        if not fp8:
            return bits
        x = orc.bf16_bits_to_f64(bits).astype(np.float32)
        out = np.empty(bits.shape, dtype=np.uint8)
        for g in range(sh.n_kv_heads):
            out[:, g, :] = orc.fp8_e4m3_encode(x[:, g, :], scale[g])
        return out

    empty = np.zeros((0, sh.n_kv_heads, sh.head_dim), dtype=np.uint16)
    cat = lambda xs: np.concatenate(xs) if xs else empty
    pk = codes(cat([k[:P[s]] for s, (k, v) in enumerate(kv_bits)]), k_scale)
    pv = codes(cat([v[:P[s]] for s, (k, v) in enumerate(kv_bits)]), v_scale)
    nk = codes(cat([k[P[s]:] for s, (k, v) in enumerate(kv_bits)]), k_scale)
    nv = codes(cat([v[P[s]:] for s, (k, v) in enumerate(kv_bits)]), v_scale)
    orc.kv_append(kp, vp, pk, pv, np.concatenate([[0], np.cumsum(P)]), np.zeros_like(P), batch.block_tables,
                  sh.n_kv_heads, sh.head_dim)
    orc.kv_append(kp, vp, nk, nv, np.concatenate([[0], np.cumsum(C)]), P, batch.block_tables, sh.n_kv_heads,
                  sh.head_dim)
    return kp, vp


_ALL_BF16 = np.arange(65536, dtype=np.uint32).astype(np.uint16)
_FINITE_BF16 = ((_ALL_BF16 >> 7) & 0xFF) != 0xFF


def _dequantised_table(scale):
    return _dequantised_table_cached(float(np.float32(scale)))


@functools.lru_cache(maxsize=64)
def _dequantised_table_cached(scale):
    """What the fp8 cache holds for every finite bf16 input under one scale: the oracle's
    software quantiser and its decoder applied to all 65 280 finite bf16 values (the
    quantisation is elementwise, so tabulating it over its whole domain changes nothing);
    NaN for the non-finite patterns, which no input contains."""
    tab = np.full(65536, np.nan)
    x = orc.bf16_bits_to_f64(_ALL_BF16[_FINITE_BF16]).astype(np.float32)
    tab[_FINITE_BF16] = orc.fp8_e4m3_decode(orc.fp8_e4m3_encode(x, scale)) * np.float64(np.float32(scale))
    return tab


def oracle_kv_values(batch, kv_bits, k_scale=None, v_scale=None):
    """fp64 K, V per sequence as the cache holds them (fp8: dequantised codes)."""
    sh = batch.shape
    if sh.kv_dtype != "fp8":
        return [(orc.bf16_bits_to_f64(k), orc.bf16_bits_to_f64(v)) for k, v in kv_bits]
    with np.errstate(over="ignore"):
        ktab = [_dequantised_table(k_scale[g]) for g in range(sh.n_kv_heads)]
        vtab = [_dequantised_table(v_scale[g]) for g in range(sh.n_kv_heads)]
    out = []
    for k, v in kv_bits:
        kf, vf = np.empty(k.shape), np.empty(v.shape)
        for g in range(sh.n_kv_heads):
            kf[:, g, :] = ktab[g][k[:, g, :]]
            vf[:, g, :] = vtab[g][v[:, g, :]]
        out.append((kf, vf))
    return out


def oracle_attention(batch, q_bits, kv_values, sm_scale):
    q = orc.bf16_bits_to_f64(q_bits)
    return orc.attn_mixed(q, [k for k, v in kv_values], [v for k, v in kv_values], batch.prefix_lens,
                          batch.chunk_lens, sm_scale)


def error_report(batch, got_bits, ref):
    """max-abs and relative L2: overall, chunk rows, decode rows, worst sequence."""
    got = orc.bf16_bits_to_f64(got_bits)
    diff = got - ref
    rel = lambda d, r: float(np.linalg.norm(d) / max(np.linalg.norm(r), 1e-300))
    cu = batch.cu_q
    is_dec = np.repeat(batch.chunk_lens == 1, batch.chunk_lens)
    rep = {"max_abs": float(np.abs(diff).max()) if diff.size else 0.0, "rel_l2": rel(diff, ref),
           "nan": int(np.isnan(got).sum())}
    if is_dec.any():
        rep["rel_l2_decode"] = rel(diff[is_dec], ref[is_dec])
    if (~is_dec).any():
        rep["rel_l2_chunk"] = rel(diff[~is_dec], ref[~is_dec])
    worst = 0.0
    for s in range(batch.n_seqs):
        if cu[s + 1] > cu[s]:
            worst = max(worst, rel(diff[cu[s]:cu[s + 1]], ref[cu[s]:cu[s + 1]]))
    rep["rel_l2_worst_seq"] = worst
    # per-row check as well, so that a single wrong row in a big batch cannot hide
    rn = np.linalg.norm(diff.reshape(diff.shape[0], -1), axis=1) / np.maximum(
        np.linalg.norm(ref.reshape(ref.shape[0], -1), axis=1), 1e-300)
    rep["rel_l2_worst_row"] = float(rn.max()) if rn.size else 0.0
    return rep


def assert_within_tolerance(rep, row_tol=3e-2):
    assert rep["nan"] == 0, rep
    assert rep["max_abs"] <= MAX_ABS_TOL, rep
    for key in ("rel_l2", "rel_l2_decode", "rel_l2_chunk", "rel_l2_worst_seq"):
        if key in rep:
            assert rep[key] <= REL_L2_TOL, (key, rep)
    assert rep["rel_l2_worst_row"] <= row_tol, rep


def run_hot_path(batch, q_bits, kv_bits, pool_fill=0x7FC1, scales="amax"):
    """The hot path on the GPU (prefix ingest, append, mixed attention, all through the C ABI)
    on given per-sequence K/V bit patterns and q rows.  Returns (out bits, k_scale, v_scale,
    DeviceIteration); the scales are None for a bf16 cache, amax / 448 per KV head for fp8
    unless a (k_scale, v_scale) pair is passed."""
    import torch

    from paper_2509_17357_amd.runtime import DeviceIteration, bf16_tensor_from_bits, bits_from_bf16_tensor

    fp8 = batch.shape.kv_dtype == "fp8"
    it = DeviceIteration(batch, pool_fill=0x7F if fp8 else pool_fill)
    P, C = batch.prefix_lens, batch.chunk_lens
    dec = C == 1
    sh = batch.shape
    empty = np.zeros((0, sh.n_kv_heads, sh.head_dim), dtype=np.uint16)
    cat = lambda xs: np.concatenate(xs) if xs else empty
    dev = lambda a: bf16_tensor_from_bits(a, it.device)
    it.prefix_k = dev(cat([k[:P[s]] for s, (k, v) in enumerate(kv_bits) if not dec[s]]))
    it.prefix_v = dev(cat([v[:P[s]] for s, (k, v) in enumerate(kv_bits) if not dec[s]]))
    it.ctx_k = dev(cat([k[:P[s]] for s, (k, v) in enumerate(kv_bits) if dec[s]]))
    it.ctx_v = dev(cat([v[:P[s]] for s, (k, v) in enumerate(kv_bits) if dec[s]]))
    it.new_k = dev(cat([k[P[s]:P[s] + C[s]] for s, (k, v) in enumerate(kv_bits)]))
    it.new_v = dev(cat([v[P[s]:P[s] + C[s]] for s, (k, v) in enumerate(kv_bits)]))
    it.q = dev(q_bits)
    it.out = torch.zeros_like(it.q)
    ks = vs = None
    if fp8:
        ks, vs = it.amax_scales() if isinstance(scales, str) else scales
        it.set_fp8_scales(ks, vs)
    it.setup_decode_context()
    it.step()
    torch.cuda.synchronize()
    return bits_from_bf16_tensor(it.out), ks, vs, it


def draw_all_kv(batch, workers=None):
    """Every sequence's seeded (k_bits, v_bits), drawn by a pool of threads (each sequence
    has its own random stream, so the result does not depend on the order)."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(workers or _workers()) as ex:
        return list(ex.map(batch.gen_kv, range(batch.n_seqs)))


def _workers():
    import os
    return max(1, min(16, os.cpu_count() or 1))


def check_rows_by_sequence(batch, out_bits, q_bits, kv_of, sm_scale, k_scale=None, v_scale=None, rows_of=None,
                           seqs=None, workers=None):
    """Oracle comparison sequence by sequence (bounded memory at any batch size; the sequences
    are independent and are handed to a pool of threads: the oracle itself is called as it
    is, once per sequence).  kv_of(s) returns the (k_bits, v_bits) of sequence s, rows_of(s, C)
    the chunk rows to evaluate (None: all).  Asserts the tolerances on every sequence's rows
    and returns the worst figures."""
    from concurrent.futures import ThreadPoolExecutor
    cu = batch.cu_q

    def one(s):
        P, C = int(batch.prefix_lens[s]), int(batch.chunk_lens[s])
        if C == 0:
            return None
        sub = type(batch)("one", batch.shape, [P], [C], 1, block_tables=np.zeros((1, 1), np.int32))
        (kf, vf), = oracle_kv_values(sub, [kv_of(s)], k_scale, v_scale)
        rows = np.arange(C) if rows_of is None else np.asarray(rows_of(s, C))
        q = orc.bf16_bits_to_f64(q_bits[cu[s]:cu[s + 1]])
        ref = orc.attn_rows(q, kf, vf, P, sm_scale, rows=rows)
        got = orc.bf16_bits_to_f64(out_bits[cu[s]:cu[s + 1]])[rows]
        d = got - ref
        rn = np.linalg.norm(d.reshape(len(rows), -1), axis=1) / np.maximum(
            np.linalg.norm(ref.reshape(len(rows), -1), axis=1), 1e-300)
        return (s, int(np.isnan(got).sum()), float(np.linalg.norm(d) / max(np.linalg.norm(ref), 1e-300)),
                float(np.abs(d).max()), float(rn.max()), len(rows), float((d * d).sum()), float((ref * ref).sum()))

    ids = list(range(batch.n_seqs) if seqs is None else seqs)
    with ThreadPoolExecutor(workers or _workers()) as ex:
        results = [r for r in ex.map(one, ids) if r is not None]
    worst = {"rel_l2": 0.0, "max_abs": 0.0, "rel_row": 0.0, "rows": 0, "seqs": len(results)}
    num = den = 0.0
    for s, nan, rel, mx, row, n, dd, rr in results:
        assert nan == 0, s
        assert rel <= REL_L2_TOL, (s, rel)
        assert mx <= MAX_ABS_TOL, (s, mx)
        assert row <= 3e-2, (s, row)
        worst["rel_l2"] = max(worst["rel_l2"], rel)
        worst["max_abs"] = max(worst["max_abs"], mx)
        worst["rel_row"] = max(worst["rel_row"], row)
        worst["rows"] += n
        num += dd
        den += rr
    worst["rel_l2_all"] = (num / max(den, 1e-300)) ** 0.5
    assert worst["rel_l2_all"] <= REL_L2_TOL, worst
    return worst
