"""MI355X (gfx950) implementation of the EMS prefill compression path (arXiv 2412.08521).

The product is the C-ABI library built from csrc/ (see include/ems.h); `binding` is its
ctypes front end.  Build with `python -m paper_2412_08521_amd.build`.
"""
from .binding import (EMS_BF16, EMS_F32, EMS_SIM_KEY, EMS_SIM_KEY_VALUE,  # noqa: F401
                      EMS_SIM_VALUE, EMS_STEP_FROM_STATE, DecodeState, EmsError, EmsParams, ems_attention_lse,
                      ems_decode_init, ems_decode_step, ems_decode_workspace_bytes,
                      ems_evict_merge, ems_evict_merge_static, ems_evict_merge_variant, ems_expand, ems_global_local_score,
                      ems_global_local_score_from_lse, ems_partition_sizes, ems_redundancy_rate, ems_select,
                      ems_sparsity_rate,
                      ems_version, ems_workspace_bytes)
