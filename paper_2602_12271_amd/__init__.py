"""MonarchRT attention (forward and backward) for AMD MI355X: HIP kernels behind a C ABI, plus a ctypes binding."""
from .binding import (  # noqa: F401
    MRT_BF16, MRT_COMPUTE_DEFAULT, MRT_COMPUTE_F32, MRT_F32, MRT_OK, MrtError, MrtProblem,
    dense_attn_check, dense_attn_fwd, last_error, load_library, make_problem, monarch_attn_check,
    monarch_attn_bwd, monarch_attn_bwd_saved, monarch_attn_fwd, monarch_attn_fwd_noalloc, monarch_attn_fwd_save,
    monarch_attn_workspace_bytes,
)
