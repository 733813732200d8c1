"""MI355X-native GRACE-MoE layer hot path (arxiv 2509.25041).

Thin Python binding over ``libgrace_moe.so`` (hand-written HIP kernels for
gfx950 behind a C ABI, see ``include/grace_moe.h``).  The functions here carry
the names of the C entry points and only marshal arguments: every step of the
path runs in the library's kernels.  PyTorch provides device memory and
streams, nothing else.  There is no CPU fallback: if the library cannot be
loaded, importing the binding's functions raises.
"""
from .binding import (  # noqa: F401
    GRACE_BF16,
    GRACE_F32,
    GRACE_POLICY_TAR,
    GRACE_POLICY_WRR,
    GraceError,
    GraceTable,
    grace_combine,
    grace_expert_ffn,
    grace_expert_ffn_down,
    grace_expert_ffn_down_share,
    grace_expert_ffn_up,
    grace_expert_ffn_up_share,
    grace_last_error,
    grace_mfma_sustained,
    grace_permute,
    grace_permute_rows,
    grace_route,
    grace_route_permute,
    grace_route_permute_static,
    grace_send_lists,
    grace_shared_ffn,
    grace_shared_ffn_down,
    grace_shared_ffn_up,
    grace_shared_ffn_up_scatter,
    grace_table_validate,
    grace_workspace_bytes,
    library_path,
    load_library,
)
from .layer import GraceMoELayer  # noqa: F401
