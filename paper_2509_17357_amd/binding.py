"""ctypes binding of libcronus.so (include/cronus.h): argument marshalling only.

Every step of the path runs in the HIP library; there is no CPU or PyTorch fallback.
If the library has not been built, loading raises.  PyTorch is used by callers for
device memory and streams; this module only reads `.data_ptr()`.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CRONUS_LIB", os.path.join(HERE, "libcronus.so"))  # CRONUS_LIB: another build of the same library

CRONUS_OK = 0
CRONUS_ERR_INVALID_ARG = 1
CRONUS_ERR_UNSUPPORTED = 2
CRONUS_ERR_WORKSPACE = 3
CRONUS_ERR_HIP = 4
CRONUS_KV_BF16 = 0
CRONUS_KV_FP8_E4M3 = 1

EXPORTS = ("cronus_kv_append", "cronus_kv_gather", "cronus_attn_mixed", "cronus_attn_mixed_static",
           "cronus_attn_mixed_workspace_bytes",
           "cronus_attn_mixed_plan_stats", "cronus_attn_mixed_plan_items", "cronus_balancer_split",
           "cronus_profile_events", "cronus_probe_mfma", "cronus_probe_mfma_sink_floats", "cronus_status_string",
           "cronus_version")


class cronus_kv_cache(ctypes.Structure):
    _fields_ = [("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
                ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
                ("num_blocks", ctypes.c_int64),
                ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("kv_dtype", ctypes.c_int32)]


class cronus_balancer_model(ctypes.Structure):
    _fields_ = [("k_p", ctypes.c_double), ("b_p", ctypes.c_double),
                ("k_ctxp", ctypes.c_double), ("k_ctxd", ctypes.c_double), ("b_c", ctypes.c_double),
                ("block_size", ctypes.c_int32), ("batch_tokens", ctypes.c_int32), ("n_candidates", ctypes.c_int32)]


class CronusError(RuntimeError):
    def __init__(self, status, what):
        super().__init__(f"{what}: {status_string(status)} (status {status})")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it was never built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2509_17357_amd.build` (or __graft_entry__.build())")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i32p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)
        cp = ctypes.POINTER(cronus_kv_cache)
        L.cronus_kv_append.argtypes = [cp, vp, vp, vp, vp, vp, i32, i32, i32, vp]
        L.cronus_kv_append.restype = ctypes.c_int
        L.cronus_kv_gather.argtypes = [cp, vp, vp, vp, vp, vp, i32, i32, i32, vp]
        L.cronus_kv_gather.restype = ctypes.c_int
        i64, f64p = ctypes.c_int64, ctypes.POINTER(ctypes.c_double)
        L.cronus_balancer_split.argtypes = [ctypes.POINTER(cronus_balancer_model), i64, i64, i64, i64,
                                            ctypes.POINTER(ctypes.c_int64), f64p, f64p]
        L.cronus_balancer_split.restype = ctypes.c_int
        L.cronus_attn_mixed.argtypes = [cp, vp, vp, i32p, i32p, vp, i32, i32, ctypes.c_float, vp, ctypes.c_size_t, vp]
        L.cronus_attn_mixed.restype = ctypes.c_int
        L.cronus_attn_mixed_static.argtypes = [cp, vp, vp, i32p, i32p, vp, i32, i32, ctypes.c_float, vp]
        L.cronus_attn_mixed_static.restype = ctypes.c_int
        L.cronus_attn_mixed_workspace_bytes.argtypes = [cp, i32p, i32p, i32]
        L.cronus_attn_mixed_workspace_bytes.restype = ctypes.c_size_t
        L.cronus_attn_mixed_plan_stats.argtypes = [cp, i32p, i32p, i32, ctypes.POINTER(ctypes.c_int64)]
        L.cronus_attn_mixed_plan_stats.restype = ctypes.c_int
        L.cronus_attn_mixed_plan_items.argtypes = [cp, i32p, i32p, i32, i32p, ctypes.c_int64]
        L.cronus_attn_mixed_plan_items.restype = ctypes.c_int64
        L.cronus_profile_events.argtypes = [vp, vp, vp, vp]
        L.cronus_profile_events.restype = None
        L.cronus_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_double)]
        L.cronus_probe_mfma.restype = ctypes.c_int
        L.cronus_probe_mfma_sink_floats.argtypes = []
        L.cronus_probe_mfma_sink_floats.restype = ctypes.c_size_t
        L.cronus_status_string.argtypes = [ctypes.c_int]
        L.cronus_status_string.restype = ctypes.c_char_p
        L.cronus_version.argtypes = []
        L.cronus_version.restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().cronus_status_string(int(status)).decode()


def version() -> int:
    return lib().cronus_version()


def cronus_profile_events(main_start: int | None, main_stop: int | None, first_start: int | None = None,
                          last_stop: int | None = None) -> None:
    """Events of the main kernel's dispatch; optionally the start of the call's first kernel
    (when that is the fp8 copy) and the stop of its last kernel (when that is the merge)."""
    lib().cronus_profile_events(ctypes.c_void_p(main_start), ctypes.c_void_p(main_stop),
                                ctypes.c_void_p(first_start), ctypes.c_void_p(last_stop))


class HipEvents:
    """Plain hipEvent_t handles (timing enabled) for cronus_profile_events."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]

    def create(self) -> int:
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed ({rc})")
        return ev.value

    def elapsed_ms(self, start: int, stop: int) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventSynchronize(stop)
        rc = rc or self.hip.hipEventElapsedTime(ctypes.byref(ms), start, stop)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)

    def destroy(self, ev: int) -> None:
        self.hip.hipEventDestroy(ev)


def _ptr(t):
    """Device/host address of a torch tensor, an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _host_i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def make_cache(k_cache, v_cache, num_blocks, num_q_heads, num_kv_heads, head_dim, kv_dtype=CRONUS_KV_BF16,
               k_scale=None, v_scale=None, block_size=16) -> cronus_kv_cache:
    return cronus_kv_cache(_ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale), int(num_blocks),
                           int(num_q_heads), int(num_kv_heads), int(head_dim), int(block_size), int(kv_dtype))


def cronus_kv_append(cache: cronus_kv_cache, k_src, v_src, cu_tokens, start_pos, block_tables,
                     max_blocks_per_seq: int, n_seqs: int, n_tokens: int, stream: int = 0, check=True) -> int:
    """k_src, v_src, cu_tokens, start_pos, block_tables: device tensors (or addresses)."""
    rc = lib().cronus_kv_append(ctypes.byref(cache), _ptr(k_src), _ptr(v_src), _ptr(cu_tokens), _ptr(start_pos),
                                _ptr(block_tables), int(max_blocks_per_seq), int(n_seqs), int(n_tokens),
                                ctypes.c_void_p(stream))
    if check and rc != CRONUS_OK:
        raise CronusError(rc, "cronus_kv_append")
    return rc


def cronus_kv_gather(cache: cronus_kv_cache, k_dst, v_dst, cu_tokens, start_pos, block_tables,
                     max_blocks_per_seq: int, n_seqs: int, n_tokens: int, stream: int = 0, check=True) -> int:
    """k_dst, v_dst, cu_tokens, start_pos, block_tables: device tensors (or addresses)."""
    rc = lib().cronus_kv_gather(ctypes.byref(cache), _ptr(k_dst), _ptr(v_dst), _ptr(cu_tokens), _ptr(start_pos),
                                _ptr(block_tables), int(max_blocks_per_seq), int(n_seqs), int(n_tokens),
                                ctypes.c_void_p(stream))
    if check and rc != CRONUS_OK:
        raise CronusError(rc, "cronus_kv_gather")
    return rc


def cronus_probe_mfma(random_operands: bool, iters: int, sink, sink_floats=None, stream: int = 0, check=True):
    """Enqueues the MFMA rate probe; returns the floating-point operations of the launch.
    sink: device float32 tensor (or address + sink_floats) of at least cronus_probe_mfma_sink_floats() elements."""
    flops = ctypes.c_double(0.0)
    if sink_floats is None:
        sink_floats = sink.numel() if hasattr(sink, "numel") else 0
    rc = lib().cronus_probe_mfma(int(bool(random_operands)), int(iters), _ptr(sink), int(sink_floats),
                                 ctypes.c_void_p(stream), ctypes.byref(flops))
    if rc != CRONUS_OK:
        if check:
            raise CronusError(rc, "cronus_probe_mfma")
        return rc
    return flops.value


def cronus_probe_mfma_sink_floats() -> int:
    return int(lib().cronus_probe_mfma_sink_floats())


def cronus_balancer_split(l_in: int, n_d: int, l_ctxd: int, n_free: int, k_p: float, b_p: float, k_ctxp: float,
                          k_ctxd: float, b_c: float, n_size: int = 16, batch_tokens: int = 512,
                          n_candidates: int = 512, with_times: bool = False, check=True):
    """Partial prefill length (and, with_times, the two modelled times of that split)."""
    model = cronus_balancer_model(k_p, b_p, k_ctxp, k_ctxd, b_c, n_size, batch_tokens, n_candidates)
    l_p = ctypes.c_int64(-1)
    tp, tc = ctypes.c_double(0.0), ctypes.c_double(0.0)
    rc = lib().cronus_balancer_split(ctypes.byref(model), int(l_in), int(n_d), int(l_ctxd), int(n_free),
                                     ctypes.byref(l_p), ctypes.byref(tp), ctypes.byref(tc))
    if rc != CRONUS_OK:
        if check:
            raise CronusError(rc, "cronus_balancer_split")
        return rc
    return (l_p.value, tp.value, tc.value) if with_times else l_p.value


def cronus_attn_mixed_workspace_bytes(cache: cronus_kv_cache, prefix_lens, chunk_lens) -> int:
    p, pp = _host_i32(prefix_lens)
    c, cp = _host_i32(chunk_lens)
    return int(lib().cronus_attn_mixed_workspace_bytes(ctypes.byref(cache), pp, cp, int(p.size)))


def cronus_attn_mixed_plan_stats(cache: cronus_kv_cache, prefix_lens, chunk_lens) -> dict:
    p, pp = _host_i32(prefix_lens)
    c, cp = _host_i32(chunk_lens)
    st = (ctypes.c_int64 * 6)()
    rc = lib().cronus_attn_mixed_plan_stats(ctypes.byref(cache), pp, cp, int(p.size), st)
    if rc != CRONUS_OK:
        raise CronusError(rc, "cronus_attn_mixed_plan_stats")
    return {"items": st[0], "wide_items": st[1], "partials": st[2], "merge_rows": st[3], "merge_groups": st[4],
            "copy_blocks": st[5]}


PLAN_ITEM_FIELDS = ("seq", "kv_head", "head0", "n_heads", "q_tok0", "n_tok", "kv_begin", "kv_end", "partial", "wide",
                    "queue")


def cronus_attn_mixed_plan_items(cache: cronus_kv_cache, prefix_lens, chunk_lens) -> np.ndarray:
    """The work list as an int32 array [n_items, 11] (columns: PLAN_ITEM_FIELDS), queue by queue."""
    p, pp = _host_i32(prefix_lens)
    c, cp = _host_i32(chunk_lens)
    n = lib().cronus_attn_mixed_plan_items(ctypes.byref(cache), pp, cp, int(p.size), None, 0)
    if n < 0:
        raise CronusError(-n, "cronus_attn_mixed_plan_items")
    out = np.zeros((max(n, 1), len(PLAN_ITEM_FIELDS)), dtype=np.int32)
    lib().cronus_attn_mixed_plan_items(ctypes.byref(cache), pp, cp, int(p.size),
                                       out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), int(n))
    return out[:n]


def cronus_attn_mixed(cache: cronus_kv_cache, q, out, prefix_lens, chunk_lens, block_tables,
                      max_blocks_per_seq: int, sm_scale: float, workspace, workspace_bytes: int,
                      stream: int = 0, check=True) -> int:
    """q, out, block_tables, workspace: device tensors; prefix_lens, chunk_lens: host int arrays."""
    p, pp = _host_i32(prefix_lens)
    c, cp = _host_i32(chunk_lens)
    if p.size != c.size:
        raise ValueError("prefix_lens and chunk_lens differ in length")
    rc = lib().cronus_attn_mixed(ctypes.byref(cache), _ptr(q), _ptr(out), pp, cp, _ptr(block_tables),
                                 int(max_blocks_per_seq), int(p.size), ctypes.c_float(sm_scale), _ptr(workspace),
                                 ctypes.c_size_t(int(workspace_bytes)), ctypes.c_void_p(stream))
    if check and rc != CRONUS_OK:
        raise CronusError(rc, "cronus_attn_mixed")
    return rc


def cronus_attn_mixed_static(cache: cronus_kv_cache, q, out, prefix_lens, chunk_lens, block_tables,
                             max_blocks_per_seq: int, sm_scale: float, stream: int = 0, check=True) -> int:
    """cronus_attn_mixed without a workspace (the library's static device scratch is used)."""
    p, pp = _host_i32(prefix_lens)
    c, cp = _host_i32(chunk_lens)
    if p.size != c.size:
        raise ValueError("prefix_lens and chunk_lens differ in length")
    rc = lib().cronus_attn_mixed_static(ctypes.byref(cache), _ptr(q), _ptr(out), pp, cp, _ptr(block_tables),
                                        int(max_blocks_per_seq), int(p.size), ctypes.c_float(sm_scale),
                                        ctypes.c_void_p(stream))
    if check and rc != CRONUS_OK:
        raise CronusError(rc, "cronus_attn_mixed_static")
    return rc
