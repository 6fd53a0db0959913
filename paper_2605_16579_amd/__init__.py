"""MI355X-native ARL^2 hybrid attention step: thin Python binding over the C-ABI HIP library."""
from .binding import (ARL2_BF16, ARL2_F32, ARL2_GATE_PER_ELEMENT, ARL2_GATE_PER_HEAD, ARL2_GATE_PER_TOKEN, Arl2Error, alloc_workspace, arl2_desc, arl2_hybrid_attn_fwd,
                      arl2_hybrid_attn_fwd_ex, arl2_hybrid_attn_fwd_fm, arl2_feature_map, arl2_gate_proj,
                      arl2_state_commit, arl2_state_commit_delta, arl2_state_commit_gdn, arl2_state_commit_static, arl2_state_commit_fm, arl2_static_scratch_bytes,
                      arl2_gdn_workspace_bytes, arl2_version, arl2_workspace_bytes, load_library, make_desc)

__all__ = ["ARL2_BF16", "ARL2_F32", "ARL2_GATE_PER_ELEMENT", "ARL2_GATE_PER_HEAD", "ARL2_GATE_PER_TOKEN", "Arl2Error", "alloc_workspace", "arl2_desc", "arl2_hybrid_attn_fwd", "arl2_hybrid_attn_fwd_ex", "arl2_hybrid_attn_fwd_fm", "arl2_feature_map", "arl2_gate_proj",
           "arl2_state_commit", "arl2_state_commit_delta", "arl2_state_commit_gdn", "arl2_state_commit_static", "arl2_state_commit_fm", "arl2_static_scratch_bytes", "arl2_gdn_workspace_bytes",
           "arl2_version", "arl2_workspace_bytes", "load_library", "make_desc"]
