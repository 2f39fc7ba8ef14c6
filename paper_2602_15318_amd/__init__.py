"""MI355X-native hot path of one Sparrow speculative-decoding step.

Thin Python binding over the C-ABI library built from csrc/ (see include/sparrow.h):
draft_window_attn, verify_attn and accept, plus hsr_fc and draft_qkv_append (the draft's input side) and kv_commit (after acceptance).  All computation runs in the HIP kernels;
PyTorch only provides device memory and streams.
"""
__all__ = ["SparrowError", "accept", "accept_workspace_bytes", "draft_window_attn", "last_error",
           "library_path", "verify_attn", "verify_attn_workspace_bytes", "version", "AttnDesc",
           "lib", "hsr_fc", "draft_qkv_append", "kv_commit", "accept_sample",
           "accept_sample_workspace_bytes", "draft_topk", "TreePool", "stream_read",
           "verify_attn_static", "STATIC_WS_BYTES", "debug_validate_parent",
           "debug_validate_text_idx", "accept_sample_q"]


def __getattr__(name):
    # The binding (and with it libsparrow.so) is loaded on first use of any public name, so that
    # `paper_2602_15318_amd.build` stays importable on a tree that has not been built yet.  A
    # missing library raises ImportError there: there is no fallback path.
    if name in __all__:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
