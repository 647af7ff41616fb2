"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these re-types the oracle's formula with the same library calls: they are a
scalar brute force, closed forms, invariants of the method (Cronus section 4.1/4.2:
prefix computed elsewhere + remainder as chunked prefill must equal ordinary
prefill), and library special cases.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import cronus_oracle as orc

RNG = np.random.default_rng(20250917)


def rand(*shape):
    return RNG.standard_normal(shape)


def brute_force(q, k, v, P, scale):
    """Independent scalar implementation: python loops, math.exp, no matrix product."""
    C, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    out = np.zeros((C, Hq, D))
    for i in range(C):
        for h in range(Hq):
            g = h // G
            logits = []
            for j in range(P + i + 1):
                acc = 0.0
                for d in range(D):
                    acc += q[i, h, d] * k[j, g, d]
                logits.append(scale * acc)
            mx = max(logits)
            ws = [math.exp(x - mx) for x in logits]
            z = sum(ws)
            for d in range(D):
                out[i, h, d] = sum(w * v[j, g, d] for j, w in enumerate(ws)) / z
    return out


@pytest.mark.parametrize("P,C,Hq,Hkv,D", [(0, 5, 2, 1, 3), (3, 4, 4, 2, 4), (7, 1, 6, 2, 2), (2, 6, 3, 3, 4)])
def test_brute_force_tiny(P, C, Hq, Hkv, D):
    q, k, v = rand(C, Hq, D), rand(P + C, Hkv, D), rand(P + C, Hkv, D)
    ref = brute_force(q, k, v, P, 0.7)
    got = orc.attn_rows(q, k, v, P, 0.7)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_hand_computed_two_keys():
    # D=1, scale 1: logits (0, ln 2) -> weights (1/3, 2/3); first row sees only key 0.
    q = np.ones((2, 1, 1))
    k = np.array([0.0, math.log(2.0)]).reshape(2, 1, 1)
    v = np.array([3.0, 6.0]).reshape(2, 1, 1)
    out = orc.attn_rows(q, k, v, 0, 1.0)
    assert out[0, 0, 0] == 3.0
    assert abs(out[1, 0, 0] - 5.0) < 1e-14
    # same two keys as a prefix of 1 with a chunk of 1 (the continuation row)
    out2 = orc.attn_rows(q[1:], k, v, 1, 1.0)
    assert abs(out2[0, 0, 0] - 5.0) < 1e-14


@pytest.mark.parametrize("N,Hq,Hkv,D", [(37, 4, 2, 8), (64, 2, 2, 16)])
def test_split_anywhere_equals_unsplit(N, Hq, Hkv, D):
    """Section 4.1/4.2: first part elsewhere, remainder as chunked prefill."""
    q, k, v = rand(N, Hq, D), rand(N, Hkv, D), rand(N, Hkv, D)
    full = orc.attn_rows(q, k, v, 0, 0.3)
    for split in range(0, N):
        part = orc.attn_rows(q[split:], k, v, split, 0.3)
        np.testing.assert_allclose(part, full[split:], rtol=1e-13, atol=1e-15)


def test_chunk_by_chunk_equals_one_chunk():
    """Section 4.4: a prompt remainder processed n_p tokens per iteration."""
    N, P, n_p = 50, 11, 7
    q, k, v = rand(N - P, 2, 8), rand(N, 1, 8), rand(N, 1, 8)
    one = orc.attn_rows(q, k, v, P, 0.5)
    pieces = []
    done = P
    while done < N:
        c = min(n_p, N - done)
        pieces.append(orc.attn_rows(q[done - P:done - P + c], k[:done + c], v[:done + c], done, 0.5))
        done += c
    np.testing.assert_allclose(np.concatenate(pieces), one, rtol=1e-13, atol=1e-15)


def test_weights_sum_to_one_and_mask_is_exact_zero():
    P, C = 5, 9
    q, k, v = rand(C, 4, 8), rand(P + C, 2, 8), rand(P + C, 2, 8)
    _, w = orc.attn_rows(q, k, v, P, 1.3, return_weights=True)
    np.testing.assert_allclose(w.sum(axis=2), 1.0, rtol=0, atol=1e-14)
    assert (w >= 0).all()
    for i in range(C):
        assert (w[i, :, P + i + 1:] == 0.0).all()
        assert (w[i, :, :P + i + 1] > 0.0).all()


def test_closed_forms():
    D = 8
    # L = 1: output is V[0]
    q, k, v = rand(1, 2, D), rand(1, 1, D), rand(1, 1, D)
    np.testing.assert_array_equal(orc.attn_rows(q, k, v, 0, 1.0)[0, 0], v[0, 0])
    # constant V: output is that constant
    q, k = rand(6, 2, D), rand(10, 2, D)
    v = np.broadcast_to(rand(1, 2, D), (10, 2, D))
    out = orc.attn_rows(q, k, v, 4, 1.0)
    np.testing.assert_allclose(out, np.broadcast_to(v[:1], (6, 2, D)), rtol=1e-14)
    # all keys equal, or Q = 0: running mean of V over the visible keys
    P, C = 3, 7
    v = rand(P + C, 1, D)
    kk = np.broadcast_to(rand(1, 1, D), (P + C, 1, D))
    means = np.stack([v[:P + i + 1, 0].mean(axis=0) for i in range(C)])
    np.testing.assert_allclose(orc.attn_rows(rand(C, 1, D), kk, v, P, 2.0)[:, 0], means, rtol=1e-13)
    np.testing.assert_allclose(orc.attn_rows(np.zeros((C, 1, D)), rand(P + C, 1, D), v, P, 2.0)[:, 0], means,
                               rtol=1e-13)


def test_shift_invariance_and_one_hot_limit():
    P, C, D = 6, 4, 8
    q, k, v = rand(C, 2, D), rand(P + C, 2, D), rand(P + C, 2, D)
    base = orc.attn_rows(q, k, v, P, 0.9)
    u = rand(1, 1, D)
    np.testing.assert_allclose(orc.attn_rows(q, k + u, v, P, 0.9), base, rtol=1e-11, atol=1e-13)
    # one key dominates every row: k_j* = big * unit vector aligned with positive q
    q = np.abs(q)
    k2 = np.zeros_like(k)
    k2[2] = 1.0
    out = orc.attn_rows(q, k2, v, P, 400.0)
    np.testing.assert_allclose(out, np.broadcast_to(np.repeat(v[2][None], 1, 0), (C, 2, D)), rtol=1e-9, atol=1e-12)


def test_decode_is_chunk_of_one_and_gqa_is_repeated_mha():
    L, D = 33, 8
    q, k, v = rand(L, 4, D), rand(L, 2, D), rand(L, 2, D)
    full = orc.attn_rows(q, k, v, 0, 0.4)
    dec = orc.attn_rows(q[L - 1:], k, v, L - 1, 0.4)
    np.testing.assert_allclose(dec[0], full[L - 1], rtol=1e-12, atol=1e-14)
    # GQA == MHA with each kv head repeated G times (contiguous groups)
    mha = orc.attn_rows(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1), 0, 0.4)
    np.testing.assert_allclose(mha, full, rtol=1e-12, atol=1e-14)
    # heads of one group given the same queries produce the same rows; different groups do not
    q2 = q.copy()
    q2[:, 1] = q2[:, 0]
    q2[:, 2] = q2[:, 0]
    o2 = orc.attn_rows(q2, k, v, 0, 0.4)
    np.testing.assert_array_equal(o2[:, 0], o2[:, 1])
    assert not np.allclose(o2[:, 0], o2[:, 2])


@pytest.mark.parametrize("P,C", [(0, 17), (9, 8), (30, 1)])
def test_library_sdpa_fp64(P, C):
    Hq, Hkv, D = 4, 2, 16
    q, k, v = rand(C, Hq, D), rand(P + C, Hkv, D), rand(P + C, Hkv, D)
    scale = 1.0 / math.sqrt(D)
    got = orc.attn_rows(q, k, v, P, scale)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, Hq // Hkv, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, Hq // Hkv, axis=1)).permute(1, 0, 2)[None]
    mask = torch.arange(P + C)[None, :] <= (P + torch.arange(C))[:, None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    np.testing.assert_allclose(got, ref[0].permute(1, 0, 2).numpy(), rtol=1e-11, atol=1e-13)


def test_attn_mixed_batches_sequences_independently():
    Hq, Hkv, D = 4, 2, 8
    P = [5, 12, 0, 3]
    C = [3, 1, 0, 1]
    ks = [rand(p + c, Hkv, D) for p, c in zip(P, C)]
    vs = [rand(p + c, Hkv, D) for p, c in zip(P, C)]
    q = rand(sum(C), Hq, D)
    out = orc.attn_mixed(q, ks, vs, P, C, 0.35)
    np.testing.assert_array_equal(out[0:3], orc.attn_rows(q[0:3], ks[0], vs[0], 5, 0.35))
    np.testing.assert_array_equal(out[3:4], orc.attn_rows(q[3:4], ks[1], vs[1], 12, 0.35))
    np.testing.assert_array_equal(out[4:5], orc.attn_rows(q[4:5], ks[3], vs[3], 3, 0.35))
    # rows= selects rows of the same definition
    sel = orc.attn_rows(q[0:3], ks[0], vs[0], 5, 0.35, rows=[2, 0])
    np.testing.assert_array_equal(sel, out[[2, 0]])


# ----------------------------------------------------------------- bf16 helpers
def test_bf16_bits_roundtrip_and_rounding():
    bits = np.arange(0x0080, 0x7F80, dtype=np.uint16)  # all positive normals
    vals = orc.bf16_bits_to_f64(bits)
    np.testing.assert_array_equal(orc.f64_to_bf16_bits(vals), bits)
    np.testing.assert_array_equal(orc.f64_to_bf16_bits(-vals), bits | 0x8000)
    tv = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(vals, tv)
    # exact midpoints go to the even neighbour
    mids = (vals[:-1] + vals[1:]) / 2
    even = np.where(bits[:-1] & 1, bits[1:], bits[:-1])
    np.testing.assert_array_equal(orc.f64_to_bf16_bits(mids), even)
    x = RNG.standard_normal(10000)
    ref = torch.from_numpy(x).to(torch.float32).to(torch.bfloat16)  # fp64->fp32->bf16 could double round...
    got = orc.f64_to_bf16_bits(x)
    same = got == ref.view(torch.int16).numpy().view(np.uint16)
    assert same.mean() > 0.999  # ...so only near-total agreement is required here


# --------------------------------------------------------------------- scatter
@pytest.mark.parametrize("Hkv,D", [(2, 64), (3, 16)])
def test_scatter_gather_inverse_and_sentinel(Hkv, D):
    nb = 23
    lens = [37, 1, 16, 50]
    perm = RNG.permutation(nb)
    tables, used = [], 0
    for L in lens:
        n = -(-L // 16)
        tables.append(list(perm[used:used + n]) + [-1] * (5 - n))
        used += n
    tables = np.array(tables)
    pool_elems = nb * Hkv * 16 * D
    sentinel = 0xDEAD
    kp = np.full(pool_elems, sentinel, dtype=np.uint16)
    vp = np.full(pool_elems, sentinel, dtype=np.uint16)
    srcs_k = [RNG.integers(0, 0xDEAC, size=(L, Hkv, D)).astype(np.uint16) for L in lens]
    srcs_v = [RNG.integers(0, 0xDEAC, size=(L, Hkv, D)).astype(np.uint16) for L in lens]
    # first part (the transferred prefix), then the rest (appended later)
    firsts = [20, 0, 16, 49]
    cu = np.concatenate([[0], np.cumsum(firsts)])
    orc.kv_append(kp, vp, np.concatenate([k[:f] for k, f in zip(srcs_k, firsts)]),
                  np.concatenate([v[:f] for v, f in zip(srcs_v, firsts)]), cu, [0] * 4, tables, Hkv, D)
    rest = [L - f for L, f in zip(lens, firsts)]
    cu2 = np.concatenate([[0], np.cumsum(rest)])
    orc.kv_append(kp, vp, np.concatenate([k[f:] for k, f in zip(srcs_k, firsts)]),
                  np.concatenate([v[f:] for v, f in zip(srcs_v, firsts)]), cu2, firsts, tables, Hkv, D)
    for s, L in enumerate(lens):
        k, v = orc.kv_gather(kp, vp, tables[s], L, Hkv, D)
        np.testing.assert_array_equal(k, srcs_k[s])
        np.testing.assert_array_equal(v, srcs_v[s])
    written = sum(lens) * Hkv * D
    assert (kp != sentinel).sum() == written and (vp != sentinel).sum() == written
    # every written element lies in a block owned by its sequence
    blk_of_elem = np.arange(pool_elems) // (Hkv * 16 * D)
    owned = set(int(b) for row in tables for b in row if b >= 0)
    assert set(np.unique(blk_of_elem[kp != sentinel])) <= owned


def test_layout_offsets_are_bijections_with_documented_strides():
    Hkv, D, nb = 2, 32, 3
    idx = np.indices((nb, Hkv, 16, D)).reshape(4, -1)
    for fn in (orc.k_elem_offset, orc.v_elem_offset):
        off = fn(idx[0], idx[1], idx[2], idx[3], Hkv, D)
        assert sorted(off.tolist()) == list(range(nb * Hkv * 16 * D))
    # K: 8 consecutive d of a token are adjacent; next token of the block is 8 elements on
    assert orc.k_elem_offset(1, 1, 5, 9, Hkv, D) - orc.k_elem_offset(1, 1, 5, 8, Hkv, D) == 1
    assert orc.k_elem_offset(1, 1, 6, 8, Hkv, D) - orc.k_elem_offset(1, 1, 5, 8, Hkv, D) == 8
    assert orc.k_elem_offset(1, 1, 5, 16, Hkv, D) - orc.k_elem_offset(1, 1, 5, 8, Hkv, D) == 128
    # V: 8 consecutive tokens of one d are adjacent; next d is 8 elements on; tokens 8.. start D*8 on
    assert orc.v_elem_offset(2, 0, 3, 7, Hkv, D) - orc.v_elem_offset(2, 0, 2, 7, Hkv, D) == 1
    assert orc.v_elem_offset(2, 0, 2, 8, Hkv, D) - orc.v_elem_offset(2, 0, 2, 7, Hkv, D) == 8
    assert orc.v_elem_offset(2, 0, 8, 0, Hkv, D) - orc.v_elem_offset(2, 0, 0, 0, Hkv, D) == D * 8
    assert orc.k_elem_offset(1, 0, 0, 0, Hkv, D) == Hkv * 16 * D == orc.v_elem_offset(1, 0, 0, 0, Hkv, D)


# ------------------------------------------------------------------------- fp8
def test_fp8_known_code_points():
    path = os.path.join(os.path.dirname(__file__), "golden", "fp8_e4m3_known_values.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        code, val = line.split()
        assert orc.fp8_e4m3_decode(np.array([int(code, 16)], dtype=np.uint8))[0] == float(val)
        assert orc.fp8_e4m3_encode(np.array([float(val)], dtype=np.float32), 1.0)[0] == int(code, 16)


def test_fp8_all_codes_roundtrip_midpoints_saturation():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    vals = orc.fp8_e4m3_decode(codes)
    np.testing.assert_array_equal(orc.fp8_e4m3_encode(vals.astype(np.float32), 1.0), codes)
    # -0 keeps its sign
    assert orc.fp8_e4m3_encode(np.array([-0.0], dtype=np.float32), 1.0)[0] == 0x80
    pos = np.arange(0, 0x7F, dtype=np.uint8)
    pv = orc.fp8_e4m3_decode(pos)
    mids = ((pv[:-1] + pv[1:]) / 2).astype(np.float32)  # exactly representable in fp32
    even = np.where(pos[:-1] & 1, pos[1:], pos[:-1])
    np.testing.assert_array_equal(orc.fp8_e4m3_encode(mids, 1.0), even)
    np.testing.assert_array_equal(orc.fp8_e4m3_encode(np.nextafter(mids, np.float32(np.inf)), 1.0), pos[1:])
    np.testing.assert_array_equal(orc.fp8_e4m3_encode(np.nextafter(mids, np.float32(-np.inf)), 1.0), pos[:-1])
    big = np.array([448.0, 449.0, 464.0, 480.0, 1e6, -1e6, 3e38], dtype=np.float32)
    np.testing.assert_array_equal(orc.fp8_e4m3_encode(big, 1.0), [0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0x7E])
    # scale: quantise(x, s) == quantise(x/s, 1) with the division in fp32
    x = RNG.standard_normal(4096).astype(np.float32)
    s = np.float32(0.0123)
    np.testing.assert_array_equal(orc.fp8_e4m3_encode(x, s), orc.fp8_e4m3_encode((x / s).astype(np.float32), 1.0))


def test_fp8_against_torch_cast_in_range():
    x = (RNG.standard_normal(200000) * 50).astype(np.float32)
    x = x[np.abs(x) < 440]
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(orc.fp8_e4m3_encode(x, 1.0), ref)
    tiny = (RNG.standard_normal(20000) * 0.01).astype(np.float32)
    ref = torch.from_numpy(tiny).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(orc.fp8_e4m3_encode(tiny, 1.0), ref)
    codes = np.arange(256, dtype=np.uint8)
    tv = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ov = orc.fp8_e4m3_decode(codes)
    np.testing.assert_array_equal(np.isnan(ov), np.isnan(tv))
    np.testing.assert_array_equal(ov[~np.isnan(ov)], tv[~np.isnan(tv)])


# ----------------------------------------------------------------- Algorithm 1
# The arithmetic of the candidate table is pinned by hand-worked cases in
# tests/test_balancer_golden_cpu.py; here: the selection rule and structural properties,
# read off the oracle's own table (no formula of the method is restated).
COEF = dict(k_p=2.0e-4, b_p=5e-3, k_ctxp=2.0e-6, k_ctxd=1.0e-7, b_c=3e-2)


def test_balancer_capacity_fallback_and_argmin():
    # not enough free blocks: whole prompt is prefilled on the low-end GPU (Algorithm 1, first branch)
    assert orc.balancer_split(1000, 10, 5000, n_free=62, **COEF) == 1000
    assert orc.balancer_split(1000, 10, 5000, n_free=63, **COEF) < 1000
    for l_in, n_d, l_ctxd in ((37, 12, 30000), (200, 12, 30000), (512, 12, 30000), (3000, 40, 10 ** 5), (50000, 500, 10 ** 6)):
        rows = orc.balancer_table(l_in, n_d, l_ctxd, **COEF)
        assert len(rows) == 512 and rows[-1][0] == l_in and rows[-1][1] == 0 and rows[-1][4] == 0.0
        if l_in <= 512:  # every length 1 .. L_in is a candidate
            assert sorted({r[0] for r in rows}) == list(range(1, l_in + 1))
        gaps = [abs(r[3] - r[4]) for r in rows]
        got = orc.balancer_split(l_in, n_d, l_ctxd, n_free=10 ** 6, **COEF)
        assert got == rows[int(np.argmin(gaps))][0]      # numpy's argmin is the first minimum too


def test_balancer_table_structure():
    """Inside a run of candidates with the same number of iterations, one more token on the
    partial prefill instance moves the last iteration's context by exactly one token, so both
    modelled times are linear in L_p there; the iteration count never grows with L_p; and the
    tokens of all iterations add up: (N_iter - 1) n_p < L_in - L_p <= N_iter n_p."""
    l_in, n_d, l_ctxd, B_tok = 400, 112, 7000, 512   # n_p = 400: every L_p is a candidate
    rows = orc.balancer_table(l_in, n_d, l_ctxd, **COEF, batch_tokens=B_tok)
    rows = [r for i, r in enumerate(rows) if i == 0 or rows[i - 1][0] != r[0]]
    n_p = B_tok - n_d
    for (lp0, n0, last0, tp0, tc0), (lp1, n1, last1, tp1, tc1) in zip(rows, rows[1:]):
        assert lp1 == lp0 + 1 and n1 <= n0
        assert (n0 - 1) * n_p < l_in - lp0 <= n0 * n_p
        assert lp0 <= last0 <= l_in
    l_in, n_d = 3000, 12                                # n_p = 500, several iteration counts
    rows = orc.balancer_table(l_in, n_d, 0, 1.0, 0.0, 1.0, 0.0, 0.0, n_candidates=3000)
    by_n = {}
    for r in rows:
        by_n.setdefault(r[1], []).append(r)
    assert sorted(by_n) == [0, 1, 2, 3, 4, 5, 6]
    for n, rs in by_n.items():
        if n == 0 or len(rs) < 3:
            continue
        # drop the one candidate of the class whose remainder is a whole number of iterations
        # (there the printed L_last jumps to L_in), the rest is an arithmetic sequence
        inner = [r for r in rs if (l_in - r[0]) % 500]
        d = [b[4] - a[4] for a, b in zip(inner, inner[1:])]
        assert max(d) - min(d) < 1e-9 and abs(d[0] - n * 0.5) < 1e-9   # slope N_iter * k_ctxp / 2
