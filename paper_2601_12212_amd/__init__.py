"""MI355X-native draft-tree speculative step (Re-SpS hot path): thin binding over libdt.so.

The functions mirror include/dt.h one to one and only marshal arguments (device tensors ->
pointers, the current torch stream -> hipStream_t).  Every step of the path runs in the HIP
kernels of the shared library; there is no CPU or PyTorch fallback: if the library is missing
the import of any entry point raises.
"""
from .binding import (DT_BF16, DT_F32, DT_ACCEPT_GREEDY, DT_ACCEPT_SAMPLED, DT_ACCEPT_STOCHASTIC, DT_D_MAX, DT_K_MAX, DT_MASK_WORDS, DT_TREE_EARLY_STOP,
                      DT_TT_MAX, DtError, dt_accept, dt_init, dt_action_table, dt_build_tree, dt_commit, dt_policy_step, dt_reward_step, dt_policy_workspace_bytes, dt_expand_level, dt_finish_tree, dt_level_state_bytes, dt_profile_enable, dt_profile_read, dt_status_string, dt_topk_rows, dt_topk_rows_static,
                      dt_tree_attention, dt_workspace_bytes, library_path, load_library)

__all__ = [n for n in dir() if n.startswith(("dt_", "DT_", "Dt"))] + ["library_path", "load_library"]
