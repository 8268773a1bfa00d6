"""Thin ctypes binding over libmonarchrt.so (the C ABI in include/monarchrt.h).

Argument marshalling only: PyTorch supplies device memory and the HIP stream, every
step of the operator runs in the library's kernels.  There is no CPU fallback: a
missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmonarchrt.so")

MRT_OK = 0
MRT_ERR_NULL, MRT_ERR_SHAPE, MRT_ERR_BLOCK, MRT_ERR_UNSUPPORTED, MRT_ERR_WORKSPACE, MRT_ERR_HIP = range(1, 7)
MRT_F32, MRT_BF16 = 0, 1
MRT_COMPUTE_DEFAULT, MRT_COMPUTE_F32 = 0, 1

EXPORTED = [
    "monarch_attn_check", "monarch_attn_workspace_min_bytes", "monarch_attn_workspace_bytes",
    "monarch_attn_fwd", "dense_attn_check", "dense_attn_fwd", "mrt_status_string", "mrt_last_error",
    "mrt_profile_enable", "mrt_profile_read", "mrt_set_head_groups",
    "monarch_attn_bwd", "monarch_attn_bwd_workspace_bytes", "monarch_attn_bwd_workspace_min_bytes",
    "monarch_attn_fwd_noalloc",
    "monarch_attn_bwd_saved_workspace_bytes", "monarch_attn_fwd_save", "monarch_attn_bwd_saved",
]
NOALLOC_SCRATCH_BYTES = 128 << 20
ASSIGNMENTS = {"fh_w": 0, "w_fh": 1, "fw_h": 2, "h_fw": 3, "f_hw": 4, "hw_f": 5}
KERNEL_STAGE_R, KERNEL_STAGE_L, KERNEL_DENSE, KERNEL_FIRST, KERNEL_LAST = 1, 2, 4, 16, 32


class MrtStrides(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_longlong), ("head", ctypes.c_longlong), ("token", ctypes.c_longlong)]


class MrtProblem(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int), ("heads", ctypes.c_int), ("head_dim", ctypes.c_int),
        ("f_q", ctypes.c_int), ("f_kv", ctypes.c_int), ("h", ctypes.c_int), ("w", ctypes.c_int),
        ("q_frame_offset", ctypes.c_int),
        ("q", MrtStrides), ("k", MrtStrides), ("v", MrtStrides), ("o", MrtStrides),
        ("dtype", ctypes.c_int), ("compute", ctypes.c_int), ("scale", ctypes.c_float),
        ("assignment", ctypes.c_int), ("tile_h", ctypes.c_int), ("head_groups", ctypes.c_int),
    ]


class MrtError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"monarchrt status {status}: {text}")
        self.status = status


_lib: Optional[ctypes.CDLL] = None


def load_library() -> ctypes.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2602_12271_amd.build). "
            "There is no fallback path.")
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(MrtProblem)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.monarch_attn_check.argtypes = [P, ci, ci, ci, ci, ci]
    lib.monarch_attn_check.restype = ci
    lib.monarch_attn_workspace_min_bytes.argtypes = [P, ci, ci, ci, ci]
    lib.monarch_attn_workspace_min_bytes.restype = sz
    lib.monarch_attn_workspace_bytes.argtypes = [P, ci, ci, ci, ci]
    lib.monarch_attn_workspace_bytes.restype = sz
    lib.monarch_attn_fwd.argtypes = [vp, vp, vp, vp, P, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.monarch_attn_fwd.restype = ci
    lib.monarch_attn_fwd_noalloc.argtypes = [vp, vp, vp, vp, P, ci, ci, ci, ci, ci, vp]
    lib.monarch_attn_fwd_noalloc.restype = ci
    fp = ctypes.c_void_p
    lib.monarch_attn_bwd_workspace_min_bytes.argtypes = [P, ci, ci, ci, ci]
    lib.monarch_attn_bwd_workspace_min_bytes.restype = sz
    lib.monarch_attn_bwd_workspace_bytes.argtypes = [P, ci, ci, ci, ci]
    lib.monarch_attn_bwd_workspace_bytes.restype = sz
    lib.monarch_attn_bwd.argtypes = [vp, vp, vp, vp, fp, fp, fp, P, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.monarch_attn_bwd.restype = ci
    lib.monarch_attn_bwd_saved_workspace_bytes.argtypes = [P, ci, ci, ci, ci]
    lib.monarch_attn_bwd_saved_workspace_bytes.restype = sz
    lib.monarch_attn_fwd_save.argtypes = [vp, vp, vp, vp, P, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.monarch_attn_fwd_save.restype = ci
    lib.monarch_attn_bwd_saved.argtypes = [vp, vp, vp, vp, fp, fp, fp, P, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.monarch_attn_bwd_saved.restype = ci
    lib.dense_attn_check.argtypes = [P, ci]
    lib.dense_attn_check.restype = ci
    lib.dense_attn_fwd.argtypes = [vp, vp, vp, vp, P, ci, vp]
    lib.dense_attn_fwd.restype = ci
    lib.mrt_status_string.argtypes = [ci]
    lib.mrt_status_string.restype = ctypes.c_char_p
    lib.mrt_last_error.argtypes = []
    lib.mrt_last_error.restype = ctypes.c_char_p
    lib.mrt_set_head_groups.argtypes = [ci]
    lib.mrt_set_head_groups.restype = None
    lib.mrt_profile_enable.argtypes = [ci]
    lib.mrt_profile_enable.restype = None
    lib.mrt_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ci), ci]
    lib.mrt_profile_read.restype = ci
    _lib = lib
    return lib


def _raise(lib, st: int):
    raise MrtError(st, f"{lib.mrt_status_string(st).decode()}: {lib.mrt_last_error().decode()}")


def make_problem(*, batch, heads, head_dim, f_q, f_kv, h, w, q_frame_offset=0, dtype=MRT_BF16,
                 compute=MRT_COMPUTE_DEFAULT, scale=1.0, q_strides=None, k_strides=None,
                 v_strides=None, o_strides=None, assign="fh_w", tile_h=0, head_groups=0) -> MrtProblem:
    """Problem descriptor; default strides are those of contiguous [batch, heads, tokens, d]."""
    nq, nkv = f_q * h * w, f_kv * h * w

    def contiguous(n):
        return (heads * n * head_dim, n * head_dim, head_dim)
    qs, ks = q_strides or contiguous(nq), k_strides or contiguous(nkv)
    vs, os_ = v_strides or contiguous(nkv), o_strides or contiguous(nq)
    return MrtProblem(batch, heads, head_dim, f_q, f_kv, h, w, q_frame_offset,
                      MrtStrides(*qs), MrtStrides(*ks), MrtStrides(*vs), MrtStrides(*os_),
                      dtype, compute, scale, assign if isinstance(assign, int) else ASSIGNMENTS[assign],
                      tile_h, head_groups)


def monarch_attn_check(prob: MrtProblem, b1, b2, tile, iters, causal_chunk=0) -> int:
    return load_library().monarch_attn_check(ctypes.byref(prob), b1, b2, tile, iters, causal_chunk)


def dense_attn_check(prob: MrtProblem, causal_chunk=0) -> int:
    return load_library().dense_attn_check(ctypes.byref(prob), causal_chunk)


def last_error() -> str:
    return load_library().mrt_last_error().decode()


def monarch_attn_workspace_bytes(prob: MrtProblem, b1, b2, tile, iters, minimum=False) -> int:
    lib = load_library()
    f = lib.monarch_attn_workspace_min_bytes if minimum else lib.monarch_attn_workspace_bytes
    return int(f(ctypes.byref(prob), b1, b2, tile, iters))


def set_head_groups(n: int) -> None:
    load_library().mrt_set_head_groups(int(n))


def profile_enable(repeats) -> None:
    """0/False: off; r >= 1: every launch is issued r times inside one event bracket."""
    load_library().mrt_profile_enable(int(repeats))


def profile_read(capacity: int = 65536):
    """[(milliseconds, kernel kind)] of the launches recorded since the last read."""
    ms = (ctypes.c_float * capacity)()
    kind = (ctypes.c_int * capacity)()
    n = load_library().mrt_profile_read(ms, kind, capacity)
    return [(ms[i], kind[i]) for i in range(n)]


# ---- torch-facing helpers ------------------------------------------------------------
def _torch_problem(Q, K, V, O, f_q, f_kv, h, w, q_frame_offset, scale, compute, assign="fh_w", tile_h=0,
                   head_groups=0):
    import torch
    assert Q.dim() == 4 and K.dim() == 4 and V.dim() == 4
    assert Q.is_cuda and K.is_cuda and V.is_cuda and O.is_cuda
    assert Q.dtype == K.dtype == V.dtype == O.dtype
    dt = {torch.float32: MRT_F32, torch.bfloat16: MRT_BF16}[Q.dtype]
    B, H, nq, d = Q.shape
    assert K.shape == (B, H, f_kv * h * w, d) and V.shape == K.shape and nq == f_q * h * w
    assert O.shape == Q.shape
    for t in (Q, K, V, O):
        assert t.stride(3) == 1, "head_dim must be contiguous"

    def st(t):
        return (t.stride(0), t.stride(1), t.stride(2))
    return make_problem(batch=B, heads=H, head_dim=d, f_q=f_q, f_kv=f_kv, h=h, w=w,
                        q_frame_offset=q_frame_offset, dtype=dt, compute=compute, scale=scale,
                        q_strides=st(Q), k_strides=st(K), v_strides=st(V), o_strides=st(O),
                        assign=assign, tile_h=tile_h, head_groups=head_groups)


def monarch_attn_fwd(Q, K, V, *, f_q, f_kv, h, w, b1, b2, tile, iters, causal_chunk=0,
                     q_frame_offset=0, scale=1.0, compute=MRT_COMPUTE_DEFAULT, out=None,
                     workspace=None, stream=None, assign="fh_w", tile_h=0, head_groups=0):
    """MonarchRT attention forward on device tensors [batch, heads, tokens, head_dim]."""
    import torch
    lib = load_library()
    O = torch.empty_like(Q) if out is None else out
    prob = _torch_problem(Q, K, V, O, f_q, f_kv, h, w, q_frame_offset, scale, compute, assign, tile_h,
                          head_groups)
    if workspace is None:
        nbytes = lib.monarch_attn_workspace_bytes(ctypes.byref(prob), b1, b2, tile, iters)
        if nbytes == 0:
            _raise(lib, lib.monarch_attn_check(ctypes.byref(prob), b1, b2, tile, iters, causal_chunk))
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=Q.device)
    s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
    st = lib.monarch_attn_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                              ctypes.byref(prob), b1, b2, tile, iters, causal_chunk,
                              workspace.data_ptr(), workspace.numel() * workspace.element_size(), s)
    if st != MRT_OK:
        _raise(lib, st)
    return O


def monarch_attn_fwd_noalloc(Q, K, V, out, *, f_q, f_kv, h, w, b1, b2, tile, iters, causal_chunk=0,
                             q_frame_offset=0, scale=1.0, compute=MRT_COMPUTE_DEFAULT, stream=None,
                             assign="fh_w", tile_h=0):
    """monarch_attn_fwd on the library's built-in scratch memory: the call allocates nothing, so the
    output tensor must be passed in."""
    import torch
    lib = load_library()
    prob = _torch_problem(Q, K, V, out, f_q, f_kv, h, w, q_frame_offset, scale, compute, assign, tile_h)
    s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
    st = lib.monarch_attn_fwd_noalloc(Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(),
                                      ctypes.byref(prob), b1, b2, tile, iters, causal_chunk, s)
    if st != MRT_OK:
        _raise(lib, st)
    return out


def monarch_attn_bwd(Q, K, V, dO, *, f_q, f_kv, h, w, b1, b2, tile, iters, causal_chunk=0,
                     q_frame_offset=0, scale=1.0, workspace=None, stream=None, assign="fh_w", tile_h=0,
                     compute=MRT_COMPUTE_DEFAULT):
    """Gradients (dQ, dK, dV), fp32, of sum(O * dO) for the forward call with the same arguments.
    compute=MRT_COMPUTE_F32 forces fp32 arithmetic everywhere (bf16 storage otherwise uses the bf16
    matrix unit where the library has such kernels)."""
    import torch
    lib = load_library()
    assert dO.shape == Q.shape and dO.dtype == Q.dtype and dO.is_cuda
    prob = _torch_problem(Q, K, V, dO, f_q, f_kv, h, w, q_frame_offset, scale, compute, assign, tile_h)
    if workspace is None:
        nbytes = lib.monarch_attn_bwd_workspace_bytes(ctypes.byref(prob), b1, b2, tile, iters)
        if nbytes == 0:
            st = lib.monarch_attn_check(ctypes.byref(prob), b1, b2, tile, iters, causal_chunk)
            _raise(lib, st if st != MRT_OK else MRT_ERR_UNSUPPORTED)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=Q.device)
    dQ = torch.empty(Q.shape, dtype=torch.float32, device=Q.device)
    dK = torch.empty(K.shape, dtype=torch.float32, device=Q.device)
    dV = torch.empty(V.shape, dtype=torch.float32, device=Q.device)
    s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
    st = lib.monarch_attn_bwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(), dQ.data_ptr(),
                              dK.data_ptr(), dV.data_ptr(), ctypes.byref(prob), b1, b2, tile, iters,
                              causal_chunk, workspace.data_ptr(),
                              workspace.numel() * workspace.element_size(), s)
    if st != MRT_OK:
        _raise(lib, st)
    return dQ, dK, dV


def monarch_attn_fwd_save(Q, K, V, *, f_q, f_kv, h, w, b1, b2, tile, iters, causal_chunk=0,
                          q_frame_offset=0, scale=1.0, workspace=None, out=None, stream=None, assign="fh_w",
                          tile_h=0, compute=MRT_COMPUTE_DEFAULT):
    """Forward call of a training step: returns (O, workspace); the workspace holds the intermediates of
    every iteration for monarch_attn_bwd_saved."""
    import torch
    lib = load_library()
    O = torch.empty_like(Q) if out is None else out
    prob = _torch_problem(Q, K, V, O, f_q, f_kv, h, w, q_frame_offset, scale, compute, assign, tile_h)
    if workspace is None:
        nbytes = lib.monarch_attn_bwd_saved_workspace_bytes(ctypes.byref(prob), b1, b2, tile, iters)
        if nbytes == 0:
            st = lib.monarch_attn_check(ctypes.byref(prob), b1, b2, tile, iters, causal_chunk)
            _raise(lib, st if st != MRT_OK else MRT_ERR_UNSUPPORTED)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=Q.device)
    s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
    st = lib.monarch_attn_fwd_save(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), ctypes.byref(prob),
                                   b1, b2, tile, iters, causal_chunk, workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), s)
    if st != MRT_OK:
        _raise(lib, st)
    return O, workspace


def monarch_attn_bwd_saved(Q, K, V, dO, workspace, *, f_q, f_kv, h, w, b1, b2, tile, iters, causal_chunk=0,
                           q_frame_offset=0, scale=1.0, stream=None, assign="fh_w", tile_h=0,
                           compute=MRT_COMPUTE_DEFAULT):
    """Gradients (dQ, dK, dV) from the intermediates monarch_attn_fwd_save left in `workspace` (same
    Q, K, V and arguments): only the reverse sweep runs."""
    import torch
    lib = load_library()
    assert dO.shape == Q.shape and dO.dtype == Q.dtype and dO.is_cuda
    prob = _torch_problem(Q, K, V, dO, f_q, f_kv, h, w, q_frame_offset, scale, compute, assign, tile_h)
    dQ = torch.empty(Q.shape, dtype=torch.float32, device=Q.device)
    dK = torch.empty(K.shape, dtype=torch.float32, device=Q.device)
    dV = torch.empty(V.shape, dtype=torch.float32, device=Q.device)
    s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
    st = lib.monarch_attn_bwd_saved(Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(), dQ.data_ptr(),
                                    dK.data_ptr(), dV.data_ptr(), ctypes.byref(prob), b1, b2, tile, iters,
                                    causal_chunk, workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), s)
    if st != MRT_OK:
        _raise(lib, st)
    return dQ, dK, dV


def dense_attn_fwd(Q, K, V, *, f_q, f_kv, h, w, causal_chunk=0, q_frame_offset=0, scale=1.0,
                   compute=MRT_COMPUTE_DEFAULT, out=None, stream=None):
    """Dense softmax attention baseline on device tensors [batch, heads, tokens, head_dim]."""
    import torch
    lib = load_library()
    O = torch.empty_like(Q) if out is None else out
    prob = _torch_problem(Q, K, V, O, f_q, f_kv, h, w, q_frame_offset, scale, compute)
    s = torch.cuda.current_stream(Q.device).cuda_stream if stream is None else stream
    st = lib.dense_attn_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                            ctypes.byref(prob), causal_chunk, s)
    if st != MRT_OK:
        _raise(lib, st)
    return O
