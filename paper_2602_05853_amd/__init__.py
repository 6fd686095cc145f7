"""RRAttention prefill path for AMD MI355X: thin ctypes binding over the HIP library librr_attn.so.

    rr_estimate(Q, K, S, B, tau)      -> BlockMask   (pattern estimation, Sec. 3.1-3.3 of the paper)
    rr_sparse_attn(Q, K, V, mask)     -> O           (causal block-sparse attention, Sec. 2.1)
    rr_dense_attn(Q, K, V, B)         -> O           (dense causal baseline)
    rr_selection_accuracy(Q, K, mask) -> [P, R, F1]  (diagnostic of the paper's appendix)

The library is loaded on first use of any of these names, so that `python -m
paper_2602_05853_amd.build` can (re)build it while an older or no library is in place; a missing
or stale library then raises at that first use -- there is no fallback path.
"""
_NAMES = ("BlockMask", "RRError", "rr_dense_attn", "rr_estimate", "rr_sparse_attn", "rr_version",
          "rr_workspace_bytes", "rr_attn_workspace_bytes", "rr_estimate_static", "rr_selection_accuracy", "rr_mask_from_dense", "rr_dense_attn_packed", "packed_seq_first",
          "RR_FLAG_PROTECT_LAST", "RR_FLAG_DIAGONAL_TOKEN", "LIB_PATH", "OFFSET_MODES")


def __getattr__(name):
    if name in _NAMES or name == "binding":
        import importlib
        binding = importlib.import_module(".binding", __name__)
        return binding if name == "binding" else getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
