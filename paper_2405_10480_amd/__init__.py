"""MI355X-native LeanAttention decode path: a HIP library (``csrc/``) behind the C ABI of
``include/lean_attn.h`` and a ctypes binding with the same names."""
from .binding import (  # noqa: F401
    BF16, F16, NUM_TILE_SHAPES, KV_PACKED, KV_PADDED, OUT_AS_INPUT, OUT_F32, LeanAttnError, Plan, PreparedCall, Problem, Tuning, lean_attn_attend, lean_attn_attend_prepare, lean_attn_launch,
    lean_attn_launch_block_size,
    lean_attn_decode, lean_attn_problem_schedule, lean_attn_problem_workspace_size, lean_attn_read_probe,
    lean_attn_schedule, lean_attn_strerror, lean_attn_walk, lean_attn_workspace_init,
    lean_attn_workspace_size, lean_attn_workspace_size_for_grid, lean_attn_workspace_status, library_path,
)
from .buildlib import build  # noqa: F401
