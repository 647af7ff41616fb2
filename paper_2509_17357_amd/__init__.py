"""MI355X-native mixed-iteration paged attention (Cronus chunked prefill instance hot path).

`paper_2509_17357_amd.binding` loads the C-ABI library built from csrc/ and exposes
cronus_kv_append / cronus_attn_mixed; `paper_2509_17357_amd.workloads` draws the
seeded synthetic batches.  Nothing here falls back to a CPU implementation.
"""
__all__ = ["workloads", "binding"]
