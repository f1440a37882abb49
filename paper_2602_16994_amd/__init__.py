"""MI355X-native batched multi-path verification of draft token trees.

The product is the C-ABI library built from csrc/ (see include/mpv.h); this
package is only the ctypes binding and the tree-shape helpers around it.
"""

from .binding import (  # noqa: F401
    MPV_DTYPE_BF16, MPV_DTYPE_F32, MPV_METHOD_SPECINFER, MPV_METHOD_TRAVERSAL, MPV_METHOD_NSS, MPV_METHOD_NAIVE, MPV_METHOD_SPECTR,
    MpvError, MpvTimeout, VerifyResult, BlockEfficiencyResult, lib_path, load_library, mpv_block_efficiency, mpv_nucleus_mask, mpv_acceptance_rates,
    mpv_fill_uniforms, mpv_last_hip_error, mpv_row_stats, mpv_strerror,
    mpv_timing_enable, mpv_timing_read, mpv_verify, mpv_version, mpv_workspace_bytes, mpv_merge_duplicates,
    MPV_KERNEL_NAMES,
    MPV_COUNTER_NEAR_TIE_ACCEPT, MPV_COUNTER_NEAR_TIE_BONUS, MPV_COUNTER_ZERO_MASS, MPV_COUNTER_BAD_TOKEN,
    MPV_COUNTER_DEPENDENCY_TIMEOUT, MPV_COUNTER_NODE_TASKS_RUN, MPV_COUNTER_NODE_TASKS_CANCELLED,
    MPV_COUNTER_NODE_TASKS_RESUMED,
)
from .trees import delayed_tree, root_tree, tree_depth  # noqa: F401
