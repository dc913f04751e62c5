"""MI355X-native DDTree draft-tree step: Python binding over the C-ABI library libddtree.so.

The binding only marshals arguments (device pointers of torch tensors, sizes, the current
stream); every step of the path runs in the HIP kernels under csrc/.  The library must have
been built (python -m paper_2604_12989_amd.build, or __graft_entry__.build()); there is no
fallback path.
"""
from .binding import (DDTreeError, accept, accept_noalloc, build, compact, error_string, library_path, load,
                      topk, verify_attn, verify_attn_spans, version, workspace_bytes, verify_attn_workspace_bytes, Workspace, DTYPE_BF16,
                      DTYPE_FP32, KERNELS, profile_enable, profile_read, profile_reset,
                      set_build_algorithm, build_giveups, selftest_host, BUILD_AUTO, BUILD_POPS, BUILD_LEVELS)

__all__ = ["DDTreeError", "accept", "accept_noalloc", "build", "compact", "error_string", "library_path", "load",
           "topk", "verify_attn", "verify_attn_spans", "version", "workspace_bytes", "verify_attn_workspace_bytes", "Workspace", "DTYPE_BF16",
           "DTYPE_FP32", "KERNELS", "profile_enable", "profile_read", "profile_reset",
           "set_build_algorithm", "build_giveups", "selftest_host", "BUILD_AUTO", "BUILD_POPS", "BUILD_LEVELS"]
