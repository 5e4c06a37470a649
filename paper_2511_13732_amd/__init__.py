"""PCG group-level verification for speculative decoding on MI355X.

Thin Python binding over ``libpcg.so`` (hand-written HIP for gfx950, C ABI in
``include/pcg.h``).  PyTorch supplies device memory and streams only; every
step of the path runs in the library's kernels.
"""
from .binding import (BF16, F32, THIN_MAX_TRIALS, AsgGroups, Diag, Groups, PcgError, PreparedInfo,
                      VerifyOutput, group_probs, group_probs_workspace_bytes,
                      asg_build, asg_build_exact, asg_normalize, groups_canonicalize_host, groups_prepare_host, groups_reverse_host,
                      groups_reverse_weights_host, groups_validate_weights_host,
                      groups_validate_host, lib, lib_path, profile_begin, profile_end, propose,
                      propose_workspace_bytes, static_scratch_bytes, strerror,
                      suggest_chunk_groups, verify, verify_thinning,
                      verify_thinning_workspace_bytes, verify_workspace_bytes, version)

__all__ = ["BF16", "F32", "THIN_MAX_TRIALS", "AsgGroups", "Diag", "Groups", "asg_build", "asg_build_exact", "asg_normalize", "PcgError", "PreparedInfo",
           "VerifyOutput", "group_probs", "group_probs_workspace_bytes",
           "groups_canonicalize_host", "groups_prepare_host", "groups_reverse_host",
           "groups_reverse_weights_host", "groups_validate_weights_host",
           "groups_validate_host", "lib", "lib_path", "profile_begin", "profile_end", "propose",
           "propose_workspace_bytes", "static_scratch_bytes", "strerror",
           "suggest_chunk_groups", "verify", "verify_thinning", "verify_thinning_workspace_bytes",
           "verify_workspace_bytes", "version"]
