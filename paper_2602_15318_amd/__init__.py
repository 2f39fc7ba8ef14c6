"""MI355X-native hot path of one Sparrow speculative-decoding step.

Thin Python binding over the C-ABI library built from csrc/ (see include/sparrow.h):
draft_window_attn, verify_attn and accept.  All computation runs in the HIP kernels;
PyTorch only provides device memory and streams.
"""
from .binding import (SparrowError, accept, accept_workspace_bytes, draft_window_attn,
                      last_error, library_path, verify_attn, verify_attn_workspace_bytes,
                      version, AttnDesc, lib)

__all__ = ["SparrowError", "accept", "accept_workspace_bytes", "draft_window_attn", "last_error",
           "library_path", "verify_attn", "verify_attn_workspace_bytes", "version", "AttnDesc",
           "lib"]
