"""Gram-threshold representative-token selection and the cascade step for MI355X (gfx950).

``ada``        ctypes binding of the C-ABI library (include/ada.h); the library itself is csrc/.
``workloads``  seeded synthetic activations shaped like the paper's workloads.
"""
from . import workloads  # noqa: F401
from .ada import (AdaError, FLAG_ATTN_CAUSAL, FLAG_GREEDY_COVER, ada_assign_nearest, ada_attention_compressed, FLAG_CROSS_EARLIER_ONLY, FLAG_TWO_PASS, FLAG_RESIDENT_PASS, ada_workspace_init, ada_cascade_layers, ada_cascade_layers_batched, ada_cascade_step_grouped, ada_select_full_grouped, ada_pipeline_layers, ada_plan_tile_shape, ada_plan_full_units, ada_cascade_layers_adaptive, AdaTauControl, ada_cascade_layers_grouped, heads_view, AdaGroups, workspace_batched, ada_cascade_report,  # noqa: F401
                  ada_cascade_step, ada_cascade_step_static, STATIC_MAX_T, ada_profile_collect, ada_profile_copy_probe, ada_profile_enable, ada_profile_mfma_probe, ada_select_full, ada_set_overlap,
                  build_library, fetch, workspace,
                  workspace_bytes)
