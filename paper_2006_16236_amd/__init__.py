"""MI355X-native linear attention (arXiv 2006.16236): the hand-written gfx950
kernels behind the C ABI of include/la.h, and a thin ctypes binding.

Importing this package loads libla_hip.so; there is no fallback if it is absent.
"""
from .binding import (LA_BF16, LA_F32, LA_F32_POLY2, LaError, la_causal_bwd, la_causal_bwd_bnhd, la_causal_bwd_state, la_causal_bwd_workspace,
                      la_causal_fwd, la_causal_fwd_bnhd, la_causal_fwd_noalloc, la_causal_fwd_state, la_causal_fwd_workspace, la_global_bwd, la_global_bwd_bnhd, la_global_bwd_workspace, la_global_fwd, la_global_fwd_bnhd,
                      la_global_fwd_workspace, la_kernel_name, la_profile_begin, la_profile_end,
                      la_recurrent_step, la_recurrent_steps, la_tuning_reload, la_version, status_string)

from .autograd import causal_linear_attention, linear_attention

__all__ = ["causal_linear_attention", "linear_attention", "LA_BF16", "LA_F32", "LA_F32_POLY2", "LaError", "la_causal_bwd", "la_causal_bwd_bnhd", "la_causal_bwd_state", "la_causal_bwd_workspace",
           "la_causal_fwd", "la_causal_fwd_bnhd", "la_causal_fwd_noalloc", "la_causal_fwd_state", "la_causal_fwd_workspace", "la_global_bwd", "la_global_bwd_bnhd", "la_global_bwd_workspace", "la_global_fwd", "la_global_fwd_bnhd", "la_global_fwd_workspace",
           "la_kernel_name", "la_profile_begin", "la_profile_end", "la_recurrent_step", "la_recurrent_steps", "la_tuning_reload", "la_version",
           "status_string"]
