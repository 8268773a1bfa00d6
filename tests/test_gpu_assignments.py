"""GPU parity of the aligned block assignments (Sec. 4.1) and of tiles that are a row range of a
frame (Sec. 4.2 with n_f = 1), fp32 and bf16 paths, through the C ABI, against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2602_12271_amd as pkg
from workloads import synthetic as syn

from gpu_harness import (compare_heads, oracle_dense_head, run_dense_gpu, run_monarch_gpu, to_device)

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-2
REL_BF16 = 4e-2


def small(dtype, **kw):
    d = 64 if dtype == "f32" else 128
    base = dict(name="small", batch=1, heads=2, head_dim=d, dtype=dtype, rope=False,
                scale=1.0 if dtype == "f32" else d ** -0.5,
                sigma_qk=d ** -0.25 if dtype == "f32" else 1.0, sigma_v=1.0,
                causal_chunk=0, q_frame_offset=0, iters=2)
    base.update(kw)
    return syn.Workload(**base)


def regular(dtype, assign, f, h, w, **kw):
    size = {"f": f, "h": h, "w": w}
    ra, ca = assign.split("_")
    b1 = int(np.prod([size[c] for c in ra]))
    b2 = int(np.prod([size[c] for c in ca]))
    return small(dtype, f_q=f, f_kv=f, h=h, w=w, b1=b1, b2=b2, tile=0, assign=assign, **kw)


F32_CASES = {f"reg-{a}": regular("f32", a, 2, 5, 6) for a in ("fh_w", "w_fh", "fw_h", "h_fw", "f_hw", "hw_f")}
F32_CASES.update({
    # (frame, width) rows: tiles of one frame, of half a frame, and of 4 rows (crossing frames)
    "fw_h-frame": small("f32", f_q=2, f_kv=2, h=5, w=6, b1=6, b2=5, tile=1, assign="fw_h"),
    "fw_h-half": small("f32", f_q=2, f_kv=2, h=4, w=6, b1=3, b2=2, tile=1, assign="fw_h", iters=3),
    "fw_h-cross": small("f32", f_q=2, f_kv=2, h=4, w=6, b1=4, b2=4, tile=1, assign="fw_h"),
    # KV cache with (frame, width) rows, one hidden frame
    "fw_h-cache-mask": small("f32", f_q=1, f_kv=3, h=4, w=6, b1=3, b2=2, tile=1, assign="fw_h",
                             causal_chunk=1, q_frame_offset=1),
    # (frame, width) columns: column tiles of 4 cross the frame boundary at column 6
    "h_fw-cross": small("f32", f_q=2, f_kv=2, h=6, w=6, b1=3, b2=4, tile=1, assign="h_fw"),
    "w_fh-tiled": small("f32", f_q=2, f_kv=2, h=4, w=6, b1=3, b2=4, tile=1, assign="w_fh"),
    "f_hw-cache-mask": small("f32", f_q=2, f_kv=6, h=2, w=4, b1=2, b2=4, tile=1, assign="f_hw",
                             causal_chunk=2, q_frame_offset=2),
    "hw_f-tiled": small("f32", f_q=4, f_kv=4, h=3, w=4, b1=6, b2=2, tile=1, assign="hw_f"),
    # half-frame tiles with the stored assignment, chunk-causal with hidden chunks
    "half-frame-mask": small("f32", f_q=2, f_kv=6, h=6, w=8, b1=3, b2=4, tile=1, causal_chunk=2,
                             q_frame_offset=2, iters=3),
    # neighbourhood tiles of 2 frames x 2 rows x 4 columns; queries at frames 0..1 of a 4-frame
    # cache with 2-frame chunks: the second frame group is hidden
    "neighbourhood-mask": small("f32", f_q=2, f_kv=4, h=4, w=8, b1=4, b2=4, tile=1, causal_chunk=2,
                                q_frame_offset=0, tile_h=2, iters=3),
    "neighbourhood-3x5": small("f32", f_q=3, f_kv=3, h=10, w=6, b1=15, b2=3, tile=1, tile_h=5),
    # one and a half frames per tile, no mask
    "frame-and-a-half": small("f32", f_q=3, f_kv=3, h=4, w=6, b1=6, b2=3, tile=1),
})


@pytest.mark.parametrize("name", list(F32_CASES))
def test_assignments_f32_match_oracle(name):
    wl = F32_CASES[name]
    arrays = syn.make_inputs(wl)
    print(f"case {name}: {wl}", flush=True)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    err, omax = compare_heads(wl, arrays, O)
    print(f"  max|gpu-oracle| = {err:.3e}, max|O| = {omax:.3e}", flush=True)
    assert err <= TOL_F32


BF16_CASES = {
    # ragged 16-tiles on both sides for the three assignments within the block limits
    "reg-w_fh": regular("bf16", "w_fh", 2, 11, 21, iters=3),
    "reg-fw_h": regular("bf16", "fw_h", 2, 11, 21),
    "reg-h_fw": regular("bf16", "h_fw", 2, 21, 11),
    "reg-fw_h-d64": regular("bf16", "fw_h", 3, 9, 13, head_dim=64, scale=0.125),
    # (frame, width) rows, KV cache, hidden chunks, one-frame and half-frame tiles
    "fw_h-cache-mask": small("bf16", f_q=2, f_kv=8, h=14, w=20, b1=20, b2=7, tile=1, assign="fw_h",
                             causal_chunk=2, q_frame_offset=4),
    "fw_h-half-mask": small("bf16", f_q=2, f_kv=8, h=14, w=20, b1=10, b2=14, tile=1, assign="fw_h",
                            causal_chunk=2, q_frame_offset=4),
    # (frame, width) columns with column tiles that cross a frame boundary
    "h_fw-cross": small("bf16", f_q=2, f_kv=2, h=20, w=28, b1=10, b2=8, tile=1, assign="h_fw"),
    "w_fh-tiled": small("bf16", f_q=2, f_kv=2, h=12, w=40, b1=20, b2=8, tile=1, assign="w_fh", iters=3),
    "hw_f-tiled": small("bf16", f_q=6, f_kv=6, h=8, w=10, b1=40, b2=3, tile=1, assign="hw_f"),
    "f_hw-cache-mask": small("bf16", f_q=2, f_kv=6, h=4, w=12, b1=2, b2=24, tile=1, assign="f_hw",
                             causal_chunk=2, q_frame_offset=2),
    # neighbourhood tiles of 2 frames x 5 rows x 14 columns, hidden chunks
    "neighbourhood-mask": small("bf16", f_q=2, f_kv=8, h=10, w=28, b1=10, b2=14, tile=1, tile_h=5,
                                causal_chunk=2, q_frame_offset=4),
    "neighbourhood-ragged": small("bf16", f_q=3, f_kv=3, h=14, w=20, b1=21, b2=10, tile=1, tile_h=7, iters=3),
    # half-frame tiles, stored assignment, hidden chunks; the key range spans several chunks of 64
    "half-frame-mask": small("bf16", f_q=2, f_kv=8, h=10, w=28, b1=5, b2=14, tile=1,
                             causal_chunk=2, q_frame_offset=4),
}


def check(wl, arrays, O, heads=None, oracle=None, label=""):
    kw = {} if oracle is None else {"oracle": oracle}
    err, omax = compare_heads(wl, arrays, O, heads=heads, **kw)
    print(f"  {label}: max|gpu-oracle| = {err:.3e}, max|O| = {omax:.3e}, ratio {err / omax:.3e}",
          flush=True)
    assert err <= TOL_BF16
    assert err <= REL_BF16 * omax + 1e-3


@pytest.mark.parametrize("name", list(BF16_CASES))
def test_assignments_bf16_match_oracle(name):
    wl = BF16_CASES[name]
    arrays = syn.make_inputs(wl)
    print(f"case {name}: {wl}", flush=True)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    check(wl, arrays, O, label=name)


@pytest.mark.parametrize("name,heads", [("C1-w_fh", None), ("C1-fw_h", None), ("C3-fw_h", [0, 11]),
                                        ("C3-half", [0, 11]), ("C3-nbh", [0, 11])])
def test_assignments_bf16_named_shapes(name, heads):
    """The 4680-token chunk under the other assignments that fit the block limits, and the
    KV-cache step with (frame, width) rows and with half-frame tiles, at full size."""
    wl = syn.WORKLOADS[name]
    arrays = syn.make_inputs(wl)
    print(f"config {name}", flush=True)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    assert torch.isfinite(O.float()).all()
    check(wl, arrays, O, heads=heads, label=name)


@pytest.mark.parametrize("name", ["C1-w_fh", "C1-fw_h", "C3-fw_h"])
def test_position_only_inputs_equal_dense_under_every_assignment(name):
    """Separable positional logits are represented exactly by any aligned assignment (Sec. 4.1)."""
    wl = syn.variant(name, heads=2)
    Q = np.empty((1, wl.heads, wl.n_q, wl.head_dim), np.float32)
    K = np.empty((1, wl.heads, wl.n_kv, wl.head_dim), np.float32)
    V = np.empty_like(K)
    for hd in range(wl.heads):
        Q[0, hd], K[0, hd], V[0, hd] = syn.make_separable_head(wl, 0, hd)
    dev = to_device(wl, (Q, K, V))
    Om = run_monarch_gpu(wl, *dev)
    Od = run_dense_gpu(wl, *dev)
    diff = (Om.float() - Od.float()).abs().max().item()
    print(f"  separable {name}: max|monarch - dense| on GPU = {diff:.3e}", flush=True)
    assert diff <= TOL_BF16
    check(wl, (Q, K, V), Om, heads=[0], oracle=oracle_dense_head, label="separable vs dense oracle")
