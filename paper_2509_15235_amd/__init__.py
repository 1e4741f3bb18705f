"""Python binding of libvispec_verify (tree verification for speculative decoding on MI355X).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
The functions mirror the C entry points declared in include/vispec_verify.h and take raw
device pointers (integers) or objects exposing ``data_ptr()`` (e.g. torch tensors).
There is no CPU fallback: if the shared library is missing, importing the binding's
functions raises.
"""
from .binding import (  # noqa: F401
    AttnDesc, AttnPlan, KVDesc, VSError, lib, lib_path,
    VS_BF16, VS_F32, VS_IMPL_AUTO, VS_IMPL_GENERIC, VS_IMPL_MFMA, VS_SCHED_AUTO, VS_SCHED_LOOP, VS_SCHED_PIPELINED, VS_SCHED_RESIDENT, VS_SCHED_BALANCED,
    vs_version, vs_strerror, vs_status_string, vs_tree_validate_host, vs_tree_mask_build,
    vs_attention_plan, vs_attention_workspace_bytes, vs_tree_verify_attention,
    vs_accept_workspace_bytes, vs_tree_accept, vs_tree_accept_noalloc, vs_accept_sample_workspace_bytes, vs_tree_accept_sample,
    vs_compress_attention_workspace_bytes, vs_compress_attention,
    vs_draft_expand_workspace_bytes, vs_draft_expand, vs_draft_tree_build, vs_tree_kv_commit, EXPORTED_SYMBOLS,
    PEAK_SYMBOLS, vs_peak_hbm_read, vs_peak_hbm_copy, vs_peak_mfma_bf16, vs_peak_mfma_flops,
)
