"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares,
and its host-side argument validation returns the documented status codes.  No kernel is
launched here."""
import ctypes
import os
import re

import pytest

import paper_2602_12271_amd as pkg
from paper_2602_12271_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "monarchrt.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{]*\)\s*;", text)
    return sorted(set(n for n in names if n.startswith(("monarch_", "dense_", "mrt_"))))


def test_library_exports_every_declared_symbol():
    lib = pkg.load_library()
    decl = declared_functions()
    assert {"monarch_attn_fwd", "dense_attn_fwd", "monarch_attn_check", "dense_attn_check",
            "monarch_attn_workspace_bytes", "monarch_attn_workspace_min_bytes",
            "mrt_status_string", "mrt_last_error", "mrt_profile_enable",
            "mrt_profile_read", "mrt_set_head_groups"} <= set(decl)
    for name in decl:
        assert hasattr(lib, name), f"{name} is declared in the header but not exported"
    assert sorted(B.EXPORTED) == decl


def test_binding_struct_matches_header_layout():
    # 8 ints, 4 x 3 long long, 2 enums, 1 float, 1 enum; natural alignment
    assert ctypes.sizeof(B.MrtStrides) == 24
    assert B.MrtProblem.q.offset == 32
    assert B.MrtProblem.dtype.offset == 32 + 4 * 24
    assert B.MrtProblem.assignment.offset == 32 + 96 + 12
    assert B.MrtProblem.tile_h.offset == 32 + 96 + 16
    assert B.MrtProblem.head_groups.offset == 32 + 96 + 20
    assert ctypes.sizeof(B.MrtProblem) == 32 + 96 + 24
    # the header lists the assignments in the binding's order
    text = open(HEADER).read()
    for name, val in B.ASSIGNMENTS.items():
        assert re.search(rf"MRT_ASSIGN_{name.upper()}\s*=\s*{val}\b", text), name


def problem(**kw):
    base = dict(batch=1, heads=12, head_dim=128, f_q=3, f_kv=3, h=30, w=52, scale=128 ** -0.5)
    base.update(kw)
    return pkg.make_problem(**base)


def test_named_configurations_are_accepted():
    assert pkg.monarch_attn_check(problem(), 90, 52, 0, 2) == B.MRT_OK                  # C1
    assert pkg.monarch_attn_check(problem(), 90, 26, 1, 2) == B.MRT_OK                  # C2
    assert pkg.monarch_attn_check(problem(f_kv=21, q_frame_offset=18), 90, 26, 1, 2, 3) == B.MRT_OK   # C3
    assert pkg.monarch_attn_check(problem(heads=40, f_kv=21, h=45, w=80, q_frame_offset=18),
                                  135, 40, 1, 3, 3) == B.MRT_OK                         # C4
    c0 = pkg.make_problem(batch=1, heads=1, head_dim=64, f_q=1, f_kv=1, h=24, w=24,
                          dtype=B.MRT_F32, scale=1.0)
    assert pkg.monarch_attn_check(c0, 24, 24, 0, 1) == B.MRT_OK                        # C0
    # regular Monarch under a chunk-causal mask (frame-causal here; 3-frame chunks hide nothing)
    assert pkg.monarch_attn_check(problem(), 90, 52, 0, 2, 1) == B.MRT_OK
    assert pkg.monarch_attn_check(problem(), 90, 52, 0, 2, 3) == B.MRT_OK
    assert pkg.monarch_attn_check(problem(assign="fw_h"), 156, 30, 0, 2, 2) == B.MRT_OK
    # other aligned assignments within the block limits, and tiles that are a row range of a frame
    assert pkg.monarch_attn_check(problem(assign="w_fh"), 52, 90, 0, 2) == B.MRT_OK
    assert pkg.monarch_attn_check(problem(assign="fw_h"), 156, 30, 0, 2) == B.MRT_OK
    assert pkg.monarch_attn_check(problem(assign="fw_h", f_kv=21, q_frame_offset=18), 52, 30, 1, 2, 3) == B.MRT_OK
    assert pkg.monarch_attn_check(problem(assign="h_fw"), 30, 52, 1, 2) == B.MRT_OK
    assert pkg.monarch_attn_check(problem(assign="hw_f"), 156, 3, 1, 1) == B.MRT_OK
    assert pkg.monarch_attn_check(problem(f_kv=21, q_frame_offset=18), 15, 26, 1, 2, 3) == B.MRT_OK
    assert pkg.monarch_attn_check(problem(), 45, 26, 1, 2) == B.MRT_OK     # 1.5 frames, no mask
    # neighbourhood tiles (n_f, n_h, n_w) = (3, 15, 26)
    assert pkg.monarch_attn_check(problem(f_kv=21, q_frame_offset=18, tile_h=15), 45, 26, 1, 2, 3) == B.MRT_OK


@pytest.mark.parametrize("kw,args,status", [
    (dict(), (90, 50, 0, 2, 0), B.MRT_ERR_BLOCK),            # b2 != w for regular
    (dict(), (45, 52, 0, 2, 0), B.MRT_ERR_BLOCK),            # b1 != f*h for regular
    (dict(f_kv=21), (90, 52, 0, 2, 0), B.MRT_ERR_UNSUPPORTED),   # rectangular needs tile=1
    (dict(assign="w_fh"), (52, 90, 0, 2, 1), B.MRT_ERR_UNSUPPORTED),   # regular + mask needs frames on the b1 side
    (dict(), (90, 52, 0, 0, 0), B.MRT_ERR_SHAPE),            # iters < 1
    (dict(), (90, 52, 2, 1, 0), B.MRT_ERR_SHAPE),            # tile flag
    (dict(), (90, 25, 1, 2, 0), B.MRT_ERR_BLOCK),            # 25 does not divide 52
    (dict(), (60, 26, 1, 2, 0), B.MRT_ERR_BLOCK),            # 60 rows do not divide 90
    (dict(f_kv=21), (45, 26, 1, 2, 1), B.MRT_ERR_BLOCK),     # 1.5-frame tiles straddle 1-frame chunks
    (dict(f_kv=21), (20, 26, 1, 2, 1), B.MRT_ERR_BLOCK),     # 20 rows divide neither frame nor grid
    (dict(assign="w_fh", f_kv=21), (52, 30, 1, 2, 0), B.MRT_ERR_UNSUPPORTED),  # frames on the b2 side, f_q != f_kv
    (dict(assign="w_fh"), (52, 30, 1, 2, 3), B.MRT_ERR_UNSUPPORTED),           # mask needs frames on the b1 side
    (dict(assign="h_fw"), (30, 52, 1, 2, 3), B.MRT_ERR_UNSUPPORTED),
    (dict(assign="fw_h"), (90, 52, 0, 2, 0), B.MRT_ERR_BLOCK),                 # regular (fw,h) is (156,30)
    (dict(assign="f_hw"), (3, 1560, 0, 2, 0), B.MRT_ERR_UNSUPPORTED),          # b2 beyond this build
    (dict(assign="hw_f"), (1560, 3, 0, 2, 0), B.MRT_ERR_UNSUPPORTED),          # b1 beyond this build
    (dict(assign=9), (90, 52, 0, 2, 0), B.MRT_ERR_SHAPE),                      # unknown assignment
    (dict(tile_h=15), (90, 52, 0, 2, 0), B.MRT_ERR_SHAPE),                     # neighbourhoods need tile = 1
    (dict(tile_h=7), (21, 26, 1, 2, 0), B.MRT_ERR_BLOCK),                      # 7 does not divide h = 30
    (dict(tile_h=15), (40, 26, 1, 2, 0), B.MRT_ERR_BLOCK),                     # b1 not a multiple of n_h
    (dict(tile_h=15), (30, 26, 1, 2, 0), B.MRT_ERR_BLOCK),                     # 2-frame neighbourhoods, 3 frames
    (dict(tile_h=15, assign="fw_h"), (45, 30, 1, 2, 0), B.MRT_ERR_UNSUPPORTED),
    (dict(tile_h=15, f_kv=21, q_frame_offset=18), (45, 26, 1, 2, 2), B.MRT_ERR_BLOCK),   # 3-frame tiles, 2-frame chunks
    (dict(tile_h=-1), (90, 52, 0, 2, 0), B.MRT_ERR_SHAPE),
    (dict(f_kv=21), (90, 26, 1, 2, 2), B.MRT_ERR_BLOCK),     # 3-frame tiles straddle 2-frame chunks
    (dict(f_kv=21, q_frame_offset=1), (90, 26, 1, 2, 3), B.MRT_ERR_BLOCK),   # offset inside a tile
    (dict(head_dim=96), (90, 52, 0, 2, 0), B.MRT_ERR_SHAPE),  # bf16 path: d in {64,128}
    (dict(scale=0.0), (90, 52, 0, 2, 0), B.MRT_ERR_SHAPE),
    (dict(heads=0), (90, 52, 0, 2, 0), B.MRT_ERR_SHAPE),
    (dict(f_q=7, f_kv=7), (210, 52, 0, 2, 0), B.MRT_ERR_UNSUPPORTED),   # b1 > 192
    (dict(w=104), (90, 104, 0, 2, 0), B.MRT_ERR_UNSUPPORTED),          # b2 > 96
])
def test_rejected_arguments(kw, args, status):
    p = problem(**kw)
    assert pkg.monarch_attn_check(p, *args) == status
    assert pkg.last_error() != ""


def test_null_problem_and_strides():
    lib = pkg.load_library()
    assert lib.monarch_attn_check(None, 90, 52, 0, 2, 0) == B.MRT_ERR_NULL
    assert lib.dense_attn_check(None, 0) == B.MRT_ERR_NULL
    bad = problem(q_strides=(1, 1, 64))          # token stride < head_dim
    assert pkg.monarch_attn_check(bad, 90, 52, 0, 2) == B.MRT_ERR_SHAPE
    odd = problem(q_strides=(12 * 4680 * 132, 4680 * 132, 132))   # not a multiple of 8 elements
    assert pkg.monarch_attn_check(odd, 90, 52, 0, 2) == B.MRT_ERR_SHAPE
    assert pkg.dense_attn_check(problem(), 3) == B.MRT_OK
    assert pkg.dense_attn_check(problem(), -1) == B.MRT_ERR_SHAPE


def test_fwd_rejects_before_touching_the_gpu():
    # every check happens on the host before the first launch: NULL tensors and a short workspace
    # are reported without a GPU in the machine
    lib = pkg.load_library()
    p = problem()
    st = lib.monarch_attn_fwd(None, None, None, None, ctypes.byref(p), 90, 52, 0, 2, 0, None, 0, None)
    assert st == B.MRT_ERR_NULL
    fake = ctypes.c_void_p(4096)
    st = lib.monarch_attn_fwd(fake, fake, fake, fake, ctypes.byref(p), 90, 52, 0, 2, 0, fake, 16, None)
    assert st == B.MRT_ERR_WORKSPACE
    st = lib.monarch_attn_fwd(fake, fake, fake, fake, ctypes.byref(p), 90, 52, 0, 2, 0,
                              ctypes.c_void_p(4096 + 8), 1 << 30, None)
    assert st == B.MRT_ERR_WORKSPACE              # misaligned workspace
    st = lib.dense_attn_fwd(None, fake, fake, fake, ctypes.byref(p), 0, None)
    assert st == B.MRT_ERR_NULL


def test_workspace_sizes():
    p = problem()
    # one (batch, head): alpha_L, Y, alpha_R of N_q*ntk*d bf16 each plus c_L of N_q*ntk fp32
    n = 4680
    slab = 3 * n * 128 * 2 + n * 4
    got = pkg.monarch_attn_workspace_bytes(p, 90, 52, 0, 2, minimum=True)
    assert slab <= got <= slab + 4 * 256
    assert pkg.monarch_attn_workspace_bytes(p, 90, 52, 0, 2) == 12 * got
    # a single iteration needs no alpha_R
    got1 = pkg.monarch_attn_workspace_bytes(p, 90, 52, 0, 1, minimum=True)
    assert got1 < got and got1 >= 2 * n * 128 * 2 + n * 4
    # tiled KV cache: ntk = 14 key tiles per query token
    p3 = problem(f_kv=21)
    got3 = pkg.monarch_attn_workspace_bytes(p3, 90, 26, 1, 2, minimum=True)
    assert got3 >= 14 * slab and got3 <= 14 * slab + 4 * 256
    assert pkg.monarch_attn_workspace_bytes(problem(), 90, 50, 0, 2) == 0      # invalid -> 0
    # fp32 compute on bf16 storage keeps fp32 intermediates
    pf = problem(compute=B.MRT_COMPUTE_F32)
    assert pkg.monarch_attn_workspace_bytes(pf, 90, 52, 0, 2, minimum=True) > 1.9 * got


def test_status_strings():
    lib = pkg.load_library()
    seen = {lib.mrt_status_string(i).decode() for i in range(7)}
    assert len(seen) == 7 and "ok" in seen


def test_backward_entry_checks_on_the_host():
    lib = pkg.load_library()
    p = problem()
    ref = ctypes.byref(p)
    # one head, fp32: alpha_L and c_L of T iterations, abar and its two column statistics of T-1, Y,
    # four gradient buffers; bf16 storage with default arithmetic adds the transposed L / dZ arrays
    # of the matrix-unit kernels (two bf16 arrays of 96 columns per (m, j, nk) row)
    n, d, T = 4680, 128, 2
    per_head = lib.monarch_attn_bwd_workspace_min_bytes(ref, 90, 52, 0, T)
    want = (2 * T + 3) * n * d * 4 + (3 * T - 1) * n * 4 + 2 * n * 96 * 2
    assert want <= per_head <= want + 16 * 256
    pf = problem(compute=B.MRT_COMPUTE_F32)
    per_head_f32 = lib.monarch_attn_bwd_workspace_min_bytes(ctypes.byref(pf), 90, 52, 0, T)
    assert want - 2 * n * 96 * 2 <= per_head_f32 <= want - 2 * n * 96 * 2 + 16 * 256
    assert lib.monarch_attn_bwd_workspace_bytes(ref, 90, 52, 0, T) == 12 * per_head
    # b1 = 135 is beyond the fp32 kernels' on-chip buffers: only the bf16 matrix-unit kernels take it
    # (ten query tiles: transposed arrays of 160 columns); fp32 arithmetic, invalid blocks give 0
    big = problem(heads=40, f_kv=21, h=45, w=80, q_frame_offset=18)
    nbig = 2 * 40 * 14 * 135                       # (m, j, nk) rows of one head
    per_head_big = lib.monarch_attn_bwd_workspace_min_bytes(ctypes.byref(big), 135, 40, 1, 3)
    # (its last stage L runs the streamed kernel, which can leave an fp32 copy of O and the rows'
    # log-sum-exp for a backward call from saved intermediates: 10800 query rows per head)
    want_big = (2 * 3 + 3) * nbig * d * 4 + (3 * 3 - 1) * nbig * 4 + 2 * nbig * 160 * 2 + 10800 * (d + 1) * 4
    assert want_big <= per_head_big <= want_big + 32 * 256
    big = problem(heads=40, f_kv=21, h=45, w=80, q_frame_offset=18, compute=B.MRT_COMPUTE_F32)
    assert lib.monarch_attn_bwd_workspace_bytes(ctypes.byref(big), 135, 40, 1, 3) == 0
    assert "backward" in pkg.last_error()
    assert lib.monarch_attn_bwd_workspace_bytes(ref, 90, 50, 0, T) == 0
    fake = ctypes.c_void_p(4096)
    args = (ref, 90, 52, 0, T, 0)
    assert lib.monarch_attn_bwd(None, fake, fake, fake, fake, fake, fake, *args, fake, 1 << 40, None) == B.MRT_ERR_NULL
    assert lib.monarch_attn_bwd(fake, fake, fake, fake, fake, fake, None, *args, fake, 1 << 40, None) == B.MRT_ERR_NULL
    assert lib.monarch_attn_bwd(fake, fake, fake, fake, fake, fake, fake, *args, fake, 1024, None) == B.MRT_ERR_WORKSPACE
    assert lib.monarch_attn_bwd(fake, fake, fake, fake, fake, fake, fake, ctypes.byref(big), 135, 40, 1, 3, 3,
                                fake, 1 << 40, None) == B.MRT_ERR_UNSUPPORTED


def test_saved_intermediates_entry_checks_on_the_host():
    """The training-step pair keeps every (batch, head) in the workspace: its size is the backward
    pass's size of one head times batch * heads, and both calls refuse anything smaller before any
    launch."""
    lib = pkg.load_library()
    p = problem()
    ref = ctypes.byref(p)
    T = 2
    per_head = lib.monarch_attn_bwd_workspace_min_bytes(ref, 90, 52, 0, T)
    total = lib.monarch_attn_bwd_saved_workspace_bytes(ref, 90, 52, 0, T)
    assert total == 12 * per_head
    assert lib.monarch_attn_bwd_saved_workspace_bytes(ref, 90, 50, 0, T) == 0      # invalid blocks
    fake = ctypes.c_void_p(4096)
    args = (ref, 90, 52, 0, T, 0)
    # room for eleven heads only
    assert lib.monarch_attn_fwd_save(fake, fake, fake, fake, *args, fake, total - 1, None) == B.MRT_ERR_WORKSPACE
    assert "every (batch,head)" in pkg.last_error()
    assert lib.monarch_attn_bwd_saved(fake, fake, fake, fake, fake, fake, fake, *args, fake, total - 1,
                                      None) == B.MRT_ERR_WORKSPACE
    assert lib.monarch_attn_fwd_save(fake, fake, fake, None, *args, fake, total, None) == B.MRT_ERR_NULL
    assert lib.monarch_attn_bwd_saved(fake, fake, fake, None, fake, fake, fake, *args, fake, total,
                                      None) == B.MRT_ERR_NULL
    assert lib.monarch_attn_fwd_save(fake, fake, fake, fake, *args, ctypes.c_void_p(4100), total,
                                     None) == B.MRT_ERR_WORKSPACE                  # misaligned workspace


def test_host_entry_points_are_thread_safe():
    """monarch_attn_check and the workspace queries keep no shared state: several host threads calling
    them at once (valid and invalid requests mixed) get the same answers as one thread, and every
    thread reads its own last-error text."""
    import threading
    lib = pkg.load_library()
    good = problem(f_kv=21, q_frame_offset=18)
    bad = problem()
    want_ws = pkg.monarch_attn_workspace_bytes(good, 90, 26, 1, 2)
    want_min = pkg.monarch_attn_workspace_bytes(good, 90, 26, 1, 2, minimum=True)
    failures = []

    def worker(k):
        for i in range(300):
            if (i + k) % 2:
                if pkg.monarch_attn_check(good, 90, 26, 1, 2, 3) != B.MRT_OK:
                    failures.append("valid request rejected")
                if pkg.monarch_attn_workspace_bytes(good, 90, 26, 1, 2) != want_ws:
                    failures.append("workspace size changed")
                if pkg.monarch_attn_workspace_bytes(good, 90, 26, 1, 2, minimum=True) != want_min:
                    failures.append("minimum workspace size changed")
            else:
                b1 = 91 + k                                     # does not divide the 90 rows
                if pkg.monarch_attn_check(bad, b1, 26, 1, 2) != B.MRT_ERR_BLOCK:
                    failures.append("invalid request accepted")
                if f"({b1},26)" not in lib.mrt_last_error().decode():
                    failures.append("another thread's error text")

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not failures, failures[:3]


def test_head_groups_field_is_checked():
    assert pkg.monarch_attn_check(problem(head_groups=2), 90, 52, 0, 2) == B.MRT_OK
    assert pkg.monarch_attn_check(problem(head_groups=9), 90, 52, 0, 2) == B.MRT_OK      # clamped to 4
    assert pkg.monarch_attn_check(problem(head_groups=-1), 90, 52, 0, 2) == B.MRT_ERR_SHAPE


def test_noalloc_entry_point_rejects_what_its_scratch_cannot_hold():
    """Host-side checks of monarch_attn_fwd_noalloc run before any GPU call: an invalid request gets
    the same status as from monarch_attn_fwd's checks, and a request whose smallest pass needs more
    than the built-in scratch (a 21-frame full sequence with 3-frame tiles of 135 x 96 at fp32:
    135 x 96 x 7 key tiles x 128 features x 4 bytes x 3 arrays per query tile row = 139 MB) is refused."""
    lib = pkg.load_library()
    p = problem()
    assert lib.monarch_attn_fwd_noalloc(None, None, None, None, ctypes.byref(p), 91, 52, 0, 2, 0, None) == B.MRT_ERR_BLOCK
    big = problem(heads=1, f_q=21, f_kv=21, h=45, w=96, dtype=B.MRT_F32)
    assert pkg.monarch_attn_workspace_bytes(big, 135, 96, 1, 2, minimum=True) > B.NOALLOC_SCRATCH_BYTES
    assert lib.monarch_attn_fwd_noalloc(None, None, None, None, ctypes.byref(big), 135, 96, 1, 2, 0, None) == B.MRT_ERR_WORKSPACE
    assert "built-in scratch" in lib.mrt_last_error().decode()
    # a request that fits but has no tensors is refused before any launch
    assert lib.monarch_attn_fwd_noalloc(None, None, None, None, ctypes.byref(p), 90, 52, 0, 2, 0, None) == B.MRT_ERR_NULL
