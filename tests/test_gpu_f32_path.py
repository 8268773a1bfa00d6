"""GPU parity of the fp32 path against the fp64 oracle (tolerance 1e-4 max-abs, the
bar stated for fp32 storage), through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2602_12271_amd as pkg
from workloads import synthetic as syn

from gpu_harness import (compare_heads, oracle_dense_head, run_dense_gpu, run_monarch_gpu, to_device)

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4


def small_f32(**kw):
    base = dict(name="small", batch=1, heads=2, head_dim=64, dtype="f32", rope=False, scale=1.0,
                sigma_qk=64 ** -0.25, sigma_v=1.0)
    base.update(kw)
    return syn.Workload(**base)


CASES = {
    # the named tiny configuration
    "C0": syn.WORKLOADS["C0"],
    # same shape, logits with sigma ~ 1 (the tiny config's own logits are nearly flat), 3 iterations
    "C0-sharp": syn.variant("C0", sigma_qk=64 ** -0.25, sigma_v=1.0, iters=3),
    # regular, ragged sizes, d not a power of two, two batches
    "reg-ragged": small_f32(batch=2, heads=3, head_dim=40, f_q=2, f_kv=2, h=5, w=13, b1=10, b2=13,
                            tile=0, iters=2, causal_chunk=0, q_frame_offset=0, sigma_qk=40 ** -0.25),
    # tiled, rectangular KV cache, chunk-causal with hidden chunks, 3 iterations
    "tiled-rect-mask": small_f32(f_q=2, f_kv=6, h=5, w=14, b1=10, b2=7, tile=1, iters=3,
                                 causal_chunk=2, q_frame_offset=2),
    # tiled square, no mask, one-frame tiles
    "tiled-square": small_f32(f_q=3, f_kv=3, h=4, w=12, b1=4, b2=6, tile=1, iters=2,
                              causal_chunk=0, q_frame_offset=0),
    # degenerate: b2 = 1 (every R block is 1x1) and tiles of one row
    "tiled-b2-1": small_f32(f_q=2, f_kv=2, h=3, w=4, b1=3, b2=1, tile=1, iters=2,
                            causal_chunk=0, q_frame_offset=0),
    # largest block sizes this build accepts
    "max-blocks": small_f32(heads=1, f_q=2, f_kv=2, h=96, w=96, b1=192, b2=96, tile=0, iters=2,
                            causal_chunk=0, q_frame_offset=0, head_dim=128, sigma_qk=128 ** -0.25),
}


@pytest.mark.parametrize("name", list(CASES))
def test_monarch_f32_matches_oracle(name):
    wl = CASES[name]
    arrays = syn.make_inputs(wl)
    print(f"case {name}: {wl}", flush=True)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    err, omax = compare_heads(wl, arrays, O)
    print(f"  max|gpu-oracle| = {err:.3e}, max|O| = {omax:.3e}", flush=True)
    assert err <= TOL_F32


@pytest.mark.parametrize("name", ["C0-sharp", "tiled-rect-mask", "reg-ragged"])
def test_dense_f32_matches_oracle(name):
    wl = CASES[name]
    arrays = syn.make_inputs(wl)
    O = run_dense_gpu(wl, *to_device(wl, arrays))
    err, omax = compare_heads(wl, arrays, O, oracle=oracle_dense_head)
    print(f"  dense {name}: max|gpu-oracle| = {err:.3e}, max|O| = {omax:.3e}", flush=True)
    assert err <= TOL_F32


def test_minimum_workspace_gives_same_result():
    # one head per pass (smallest workspace) must equal all heads in one pass, bit for bit
    wl = CASES["tiled-rect-mask"]
    arrays = syn.make_inputs(wl)
    dev = to_device(wl, arrays)
    prob = pkg.make_problem(batch=wl.batch, heads=wl.heads, head_dim=wl.head_dim, f_q=wl.f_q,
                            f_kv=wl.f_kv, h=wl.h, w=wl.w, dtype=pkg.MRT_F32, scale=wl.scale)
    nmin = pkg.monarch_attn_workspace_bytes(prob, wl.b1, wl.b2, wl.tile, wl.iters, minimum=True)
    ws = torch.empty(nmin, dtype=torch.uint8, device="cuda:0")
    O1 = run_monarch_gpu(wl, *dev, workspace=ws)
    O2 = run_monarch_gpu(wl, *dev)
    assert torch.equal(O1, O2)


def test_strided_layout_tokens_major():
    # [batch, tokens, heads, d] memory viewed as [batch, heads, tokens, d]
    wl = CASES["tiled-square"]
    arrays = syn.make_inputs(wl)
    Qd, Kd, Vd = to_device(wl, arrays)
    Ocontig = run_monarch_gpu(wl, Qd, Kd, Vd)
    Qs, Ks, Vs = (x.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for x in (Qd, Kd, Vd))
    assert not Qs.is_contiguous()
    out = torch.empty_like(Qs)
    O = pkg.monarch_attn_fwd(Qs, Ks, Vs, f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1,
                             b2=wl.b2, tile=wl.tile, iters=wl.iters, scale=wl.scale, out=out)
    torch.cuda.synchronize()
    assert torch.equal(O, Ocontig)
