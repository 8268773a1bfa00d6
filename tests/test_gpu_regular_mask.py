"""GPU parity of regular Monarch under the chunk-causal mask (one tile that straddles every chunk;
the mask hides, per query row, the key rows of later chunks: a support constraint on L) against
the fp64 oracle, through the C ABI: bf16 matrix-unit path, fp32 path, backward pass, and the
property that position-only inputs reproduce masked dense attention (Sec. 4.1)."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2602_12271_amd as pkg
from oracle import monarch_oracle as mo
from workloads import synthetic as syn

from gpu_harness import (compare_heads, oracle_dense_head, run_dense_gpu, run_monarch_gpu, to_device)

pytestmark = pytest.mark.gpu

TOL_BF16, REL_BF16, TOL_F32 = 2e-2, 4e-2, 1e-4


def case(dtype="bf16", **kw):
    d = kw.pop("head_dim", 128)
    base = dict(name="regular-mask", batch=1, heads=2, head_dim=d, dtype=dtype, rope=False, scale=d ** -0.5,
                sigma_qk=1.0, sigma_v=1.0, tile=0, q_frame_offset=0)
    base.update(kw)
    base.setdefault("f_kv", base["f_q"])
    if "b1" not in base:
        base["b1"], base["b2"] = base["f_q"] * base["h"], base["w"]
    return syn.Workload(**base)


CASES = {
    # frame-causal, ragged tiles on both sides, three iterations (one-pass refine kernel, 3 query tiles)
    "frame-causal-ragged": case(f_q=4, h=11, w=21, iters=3, causal_chunk=1),
    # head_dim 64, 2-frame chunks with the queries one frame into the key grid's chunks
    "d64-offset": case(head_dim=64, f_q=6, h=9, w=13, iters=2, causal_chunk=2, q_frame_offset=1),
    # 8 query tiles: six-wave refine kernel, streamed last iteration with two tiles per wave
    "b1-120": case(f_q=4, h=30, w=12, iters=2, causal_chunk=1),
    # 12 query tiles (the largest b1 of this build), 2-frame chunks, sharper logits
    "b1-180": case(heads=1, f_q=6, h=30, w=20, iters=2, causal_chunk=2, sigma_qk=1.5),
    # a single iteration (only the last-iteration kernel sees the mask)
    "T1": case(f_q=3, h=10, w=26, iters=1, causal_chunk=1),
    # (frame, width) rows against height columns
    "fw_h": case(f_q=3, h=6, w=10, b1=30, b2=6, iters=2, causal_chunk=1, assign="fw_h"),
    # frames against (height, width) columns: three block rows, one per frame
    "f_hw": case(f_q=3, h=6, w=10, b1=3, b2=60, iters=2, causal_chunk=1, assign="f_hw"),
}

# Outside the stated 2e-2 bar, with the bar it is held to instead: sharp logits (sigma 1.5 per
# coordinate), outputs of magnitude 3 -- one bf16 rounding of the output alone is 8e-3 there.
OUTSIDE_STATED_BAR = {"b1-180": 3e-2}

F32_CASES = {
    "f32-frame-causal": case("f32", head_dim=40, f_q=3, h=5, w=13, iters=3, causal_chunk=1),
    "f32-offset": case("f32", head_dim=64, f_q=6, h=4, w=9, iters=2, causal_chunk=2, q_frame_offset=1),
}


@pytest.mark.parametrize("name", list(CASES))
def test_masked_regular_bf16(name):
    wl = CASES[name]
    print(f"case {name}: {wl}", flush=True)
    arrays = syn.make_inputs(wl)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    err, omax = compare_heads(wl, arrays, O)
    print(f"  max|gpu-oracle| = {err:.3e}, max|O| = {omax:.3e}", flush=True)
    assert err <= OUTSIDE_STATED_BAR.get(name, TOL_BF16) and err <= REL_BF16 * omax + 1e-3
    # the mask matters: the unmasked operator differs by far more than the bar
    wl0 = dataclasses.replace(wl, causal_chunk=0)
    O0 = run_monarch_gpu(wl0, *to_device(wl0, arrays))
    assert (O0.float() - O.float()).abs().max().item() > 10 * err


@pytest.mark.parametrize("name", list(F32_CASES))
def test_masked_regular_f32(name):
    wl = F32_CASES[name]
    print(f"case {name}: {wl}", flush=True)
    arrays = syn.make_inputs(wl)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    err, omax = compare_heads(wl, arrays, O)
    print(f"  max|gpu-oracle| = {err:.3e}, max|O| = {omax:.3e}", flush=True)
    assert err <= TOL_F32


def test_masked_regular_f32_arithmetic_on_bf16_storage():
    wl = CASES["frame-causal-ragged"]
    arrays = syn.make_inputs(wl)
    O = run_monarch_gpu(wl, *to_device(wl, arrays), compute=pkg.MRT_COMPUTE_F32)
    err, omax = compare_heads(wl, arrays, O)
    print(f"  fp32 arithmetic on bf16 storage: {err:.3e} (max|O| {omax:.3e})", flush=True)
    assert err <= 2.0 ** -8 * max(1.0, omax)          # only the final store rounds


@pytest.mark.parametrize("name", ["b1-120", "d64-offset"])
def test_position_only_inputs_reproduce_masked_dense_attention(name):
    """A constant vector under 3-D rotary encoding gives logits that are a (frame, height) term plus
    a width term: the masked regular operator and the masked dense kernel must then agree, and
    both match the masked dense oracle."""
    wl = CASES[name]
    Q = np.empty((1, wl.heads, wl.n_q, wl.head_dim), np.float32)
    K = np.empty((1, wl.heads, wl.n_kv, wl.head_dim), np.float32)
    V = np.empty_like(K)
    for hd in range(wl.heads):
        Q[0, hd], K[0, hd], V[0, hd] = syn.make_separable_head(wl, 0, hd)
    dev = to_device(wl, (Q, K, V))
    Om = run_monarch_gpu(wl, *dev)
    Od = run_dense_gpu(wl, *dev)
    diff = (Om.float() - Od.float()).abs().max().item()
    print(f"  position-only {name}: max|monarch - dense| on GPU = {diff:.3e}", flush=True)
    assert diff <= TOL_BF16
    err, omax = compare_heads(wl, (Q, K, V), Om, heads=[0], oracle=oracle_dense_head)
    assert err <= TOL_BF16


def test_a_mask_that_hides_nothing_gives_the_unmasked_bits():
    wl = case(f_q=3, h=10, w=26, iters=2, causal_chunk=3)
    arrays = syn.make_inputs(wl)
    dev = to_device(wl, arrays)
    O = run_monarch_gpu(wl, *dev)
    O0 = pkg.monarch_attn_fwd(*dev, f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=0,
                              iters=wl.iters, causal_chunk=0, scale=wl.scale)
    torch.cuda.synchronize()
    assert torch.equal(O, O0)


BWD_CASES = {
    "f32-T2": case("f32", head_dim=40, f_q=3, h=5, w=13, iters=2, causal_chunk=1),
    "f32-offset-T3": case("f32", head_dim=64, f_q=6, h=4, w=9, iters=3, causal_chunk=2, q_frame_offset=1),
    "bf16-T2": case(f_q=4, h=11, w=21, iters=2, causal_chunk=1),
    "bf16-d64-T1": case(head_dim=64, f_q=4, h=6, w=12, iters=1, causal_chunk=2),
    # b1 = 120: the streamed rows kernel (key range beyond 96 rows), ten waves
    "bf16-b1-120-T2": case(heads=1, f_q=4, h=30, w=12, iters=2, causal_chunk=1),
    # offset query frames, three iterations
    "bf16-offset-T3": case(head_dim=64, f_q=6, h=9, w=13, iters=3, causal_chunk=2, q_frame_offset=1),
}


@pytest.mark.parametrize("name", list(BWD_CASES))
def test_masked_regular_backward(name):
    """fp32 storage: the fp32 kernels, whose stage L masks its logits.  bf16 storage: the bf16
    matrix-unit kernels (hidden keys get a bias of -inf in the rows kernels), bar relative to the
    largest gradient."""
    wl = BWD_CASES[name]
    print(f"case {name}: {wl}", flush=True)
    arrays = syn.make_inputs(wl)
    rng = np.random.default_rng(4321)
    dO = rng.standard_normal(arrays[0].shape).astype(np.float32)
    if wl.dtype == "bf16":
        dO = syn.round_to_bf16(dO)
    Qd, Kd, Vd, dOd = to_device(wl, arrays + (dO,))
    kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=0, iters=wl.iters,
              causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset, scale=wl.scale)
    grads = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, **kw)
    torch.cuda.synchronize()
    for b in range(wl.batch):
        for hd in range(wl.heads):
            ref = mo.monarch_attn_grad(*(torch.from_numpy(x[b, hd]) for x in arrays),
                                       torch.from_numpy(dO[b, hd]), **kw)
            for nm, got, want in zip("QKV", grads, ref):
                g = got[b, hd].double().cpu()
                assert torch.isfinite(g).all(), f"non-finite d{nm}"
                err, gmax = (g - want).abs().max().item(), want.abs().max().item()
                bar = 2e-2 * gmax if wl.dtype == "bf16" else min(1e-4 * max(1.0, gmax), 2e-5 * gmax + 1e-9)
                print(f"  head {hd} d{nm}: max err {err:.3e} (max |grad| {gmax:.3e})", flush=True)
                assert err <= bar, (nm, err, bar)
