"""MI355X-native library for AMULET's matrix-multiplication-like tasks.

The work is done by ``libamulet.so`` (hand-written HIP for gfx950, built
in-tree by ``paper_2305_08872_amd.build``); this package is the thin ctypes
binding over its C ABI (``include/amulet.h``).  PyTorch is used by callers for
device memory and streams only.
"""
from .binding import (  # noqa: F401
    AMULET_BOOST,
    AMULET_COUNT_GT,
    AMULET_DISCOUNT,
    AMULET_IDENTITY,
    AMULET_TASK_COUNT_I8,
    AMULET_THRES_COL,
    AMULET_THRES_CONST,
    AMULET_THRES_ELEM,
    AMULET_THRES_ROW,
    AmuletError,
    amulet_choose_kernel_height,
    amulet_clear_selections,
    amulet_count_i8,
    amulet_count_i8_shape,
    amulet_greedy_search,
    amulet_last_launch_error,
    amulet_mmlike_f32,
    amulet_mmlike_f32_adaptive,
    amulet_mmlike_f32_general,
    amulet_mmlike_f32_shape,
    amulet_mmlike_f32_autopack,
    amulet_mmlike_f64,
    amulet_mmlike_f64_autopack,
    amulet_autopack_workspace_bytes,
    amulet_pack,
    amulet_packed_ld,
    amulet_pitch_collides,
    amulet_probe_mfma_i8,
    amulet_probe_valu,
    amulet_register_demand,
    amulet_selected_shape,
    amulet_shape_count,
    amulet_shape_name,
    amulet_strerror,
    amulet_tile_grid,
    amulet_tile_of_workgroup,
    amulet_tune,
    amulet_version,
    library_path,
    load_library,
)
