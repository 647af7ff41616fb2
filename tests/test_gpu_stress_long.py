"""Adversarial softmax inputs at 8192 and more keys through every kernel path, against the
fp64 oracle (same tolerance as everywhere: max-abs 2e-2, relative L2 1e-2, every row 3e-2).

The online softmax of the kernels keeps a lazily updated reference per row (rescaled only when
a row's maximum outgrew it by 8 bits), and the steady-state loop of the chunk tiles computes
numerators against the reference as it stands and redoes a sub-tile when a sum shows that it was
stale.  These inputs drive exactly that machinery for hundreds of sub-tiles: logits that keep
rising (every other sub-tile needs a rescale), logits that fall (the maximum is the first key),
a peak in the first span only, an outlier that arrives in the last tile, sharply peaked rows,
and identical keys.  Paths: an unsplit chunk tile (long steady-state run), chunk tiles cut into
key spans and merged, decodes in spans of 4096 keys (cross-wave fold, then merge), an fp8 chunk
converted on its way into LDS, an fp8 chunk that reads the launch's bf16 copy, head_dim 64."""
import numpy as np
import pytest

from paper_2509_17357_amd import binding as B
from paper_2509_17357_amd import workloads as W

import parity_util as U

pytestmark = pytest.mark.gpu

KINDS = ["peaky", "outlier_last", "outlier_first", "ramp_up", "ramp_down", "monotone", "equal"]
F = {n: i for i, n in enumerate(B.PLAN_ITEM_FIELDS)}


def plan_items(batch):
    sh = batch.shape
    c = B.make_cache(0, 0, 1 << 22, sh.n_q_heads, sh.n_kv_heads, sh.head_dim,
                     B.CRONUS_KV_FP8_E4M3 if sh.kv_dtype == "fp8" else B.CRONUS_KV_BF16)
    items = B.cronus_attn_mixed_plan_items(c, batch.prefix_lens, batch.chunk_lens)
    return items[items[:, F["wide"]] >= 0]


# path -> (shape, prefix_lens, chunk_lens, check of the plan, chunk rows to evaluate or None)
def _unsplit(items):
    wide = items[items[:, F["wide"]] >= 1]
    assert (wide[:, F["partial"]] == -1).all() and (wide[:, F["kv_begin"]] == 0).all()
    assert wide[:, F["kv_end"]].max() >= 8192 and len(wide) == 256


def _split_wide(items):
    wide = items[items[:, F["wide"]] == 1]
    assert len(wide) and (wide[:, F["partial"]] >= 0).all() and wide[:, F["kv_end"]].max() >= 8192


def _split_decode(items):
    nar = items[items[:, F["wide"]] == 0]
    span = nar[:, F["kv_end"]] - nar[:, F["kv_begin"]]
    assert (nar[:, F["partial"]] >= 0).all() and span.max() >= 4096


def _fp8_staged(items):
    wide = items[items[:, F["wide"]] >= 1]
    assert len(wide) and (wide[:, F["wide"]] == 1).all() and wide[:, F["kv_end"]].max() >= 8192


def _fp8_copy(items):
    wide = items[items[:, F["wide"]] >= 1]
    assert len(wide) and (wide[:, F["wide"]] >= 2).all() and wide[:, F["kv_end"]].max() >= 8192


def _d64(items):
    assert (items[items[:, F["wide"]] >= 1][:, F["kv_end"]].max() >= 8192) and (items[:, F["wide"]] == 0).any()


def _sample_rows(s, C):   # first and last 16 rows, every eleventh row between
    return np.unique(np.concatenate([np.arange(min(16, C)), np.arange(max(C - 16, 0), C), np.arange(0, C, 11)]))


PATHS = {
    # 4 chunks x 8 tiles x 8 KV heads = 256 tiles of 8.0-8.5 k keys each: one per CU, none is cut
    "wide_unsplit": (W.SHAPE_8B, [8000, 8000, 8000, 8000], [512, 512, 512, 512], _unsplit, _sample_rows),
    "wide_split": (W.SHAPE_8B, [12000, 9000], [256, 1], _split_wide, None),
    "decode_split": (W.SHAPE_8B, [16383, 20000, 17000, 12287, 19999, 16500, 15000, 18000], [1] * 8, _split_decode, None),
    "fp8_staged": (W.HeadShape(16, 2, 128, "fp8"), [9000, 8500], [200, 1], _fp8_staged, None),
    "fp8_copy": (W.HeadShape(16, 2, 128, "fp8"), [9000, 8500], [520, 1], _fp8_copy, None),
    "head_dim_64": (W.HeadShape(8, 2, 64), [10000, 11999], [300, 1], _d64, None),
}


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("path", sorted(PATHS))
def test_stress_inputs_at_length(path, kind):
    shape, P, C, plan_check, rows_of = PATHS[path]
    batch = W.custom_batch(shape, P, C, seed=7700 + sorted(PATHS).index(path))
    plan_check(plan_items(batch))
    kv, qs = [], []
    for s in range(batch.n_seqs):
        q, k, v = W.stress_qkv(kind, 7700 + 31 * s + KINDS.index(kind), C[s], P[s] + C[s], shape)
        kv.append((k, v))
        qs.append(q)
    q_bits = np.concatenate(qs)
    out, ks, vs, it = U.run_hot_path(batch, q_bits, kv)
    rep = U.check_rows_by_sequence(batch, out, q_bits, lambda s: kv[s], it.sm_scale, ks, vs, rows_of)
    print(path, kind, rep)
