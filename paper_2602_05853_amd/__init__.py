"""RRAttention prefill path for AMD MI355X: thin ctypes binding over the HIP library librr_attn.so.

    rr_estimate(Q, K, S, B, tau)      -> BlockMask   (pattern estimation, Sec. 3.1-3.3 of the paper)
    rr_sparse_attn(Q, K, V, mask)     -> O           (causal block-sparse attention, Sec. 2.1)
    rr_dense_attn(Q, K, V, B)         -> O           (dense causal baseline)
"""
from .binding import (  # noqa: F401
    BlockMask, RRError, rr_dense_attn, rr_estimate, rr_sparse_attn, rr_version, rr_workspace_bytes,
    RR_FLAG_PROTECT_LAST, LIB_PATH,
)
