"""Clustered vocabulary projection for MI355X (gfx950).

The product is the C-ABI library ``libvp.so`` (``include/vp.h``); ``vp`` is its
thin ctypes binding and ``workloads`` the seeded synthetic input generators.
"""
from . import vp  # noqa: F401
from .vp import (Index, VpError, vp_build, vp_destroy, vp_get_info, vp_get_profile, vp_last_error, vp_project,  # noqa: F401
                 vp_project_debug_logits, vp_project_full, vp_project_static, vp_project_union, vp_set_option, vp_union_workspace_bytes, vp_workspace_bytes,
                 vp_active_sets, vp_active_sets_workspace_bytes, vp_kmeans, vp_kmeans_workspace_bytes, vp_round_to_half, vp_beam_step, vp_measure_ceilings)
