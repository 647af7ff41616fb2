"""MI355X-native mixed-iteration paged attention (Cronus chunked prefill instance hot path).

`paper_2509_17357_amd.binding` loads the C-ABI library built from csrc/ and exposes
cronus_kv_append / cronus_kv_gather / cronus_attn_mixed / cronus_balancer_split;
`paper_2509_17357_amd.workloads` draws the seeded synthetic batches; `runtime` holds the
device buffers of one iteration; `fit_eq3` and `overlap` are measurement tools.  Nothing
here falls back to a CPU implementation.
"""
__all__ = ["workloads", "binding", "runtime", "fit_eq3", "overlap", "build"]
