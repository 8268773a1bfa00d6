"""monarch_attn_fwd_noalloc (the forward call on the library's built-in scratch memory, for callers
that cannot allocate) against monarch_attn_fwd with a caller-provided workspace, through the C ABI:
two calls in a row on the same GPU, the second with a smaller input that leaves most of the first
call's intermediates in the scratch.  Both must give the bits of the workspace call, and match the
oracle to the bf16 bar."""
import pytest
import torch

import paper_2602_12271_amd as pkg
from workloads import synthetic as syn

from gpu_harness import compare_heads, to_device

pytestmark = pytest.mark.gpu


def run_pair(wl):
    arrays = syn.make_inputs(wl)
    dev = to_device(wl, arrays)
    kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=wl.tile, iters=wl.iters,
              causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset, scale=wl.scale)
    want = pkg.monarch_attn_fwd(*dev, **kw)
    out = torch.full_like(dev[0], float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    pkg.monarch_attn_fwd_noalloc(*dev, out, **kw)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # nothing came from torch's allocator either
    return arrays, want, out


def test_noalloc_matches_workspace_call_twice_second_smaller():
    # first call: the tiled KV-cache step at 3 heads (one head's intermediates, 50 MB, per pass of the
    # 128 MiB scratch -> two heads per pass, then one); second call: a small ragged tiled problem
    first = syn.variant("C3", heads=3, q_frame_offset=9)
    second = syn.Workload(name="small", batch=1, heads=2, head_dim=128, f_q=2, f_kv=8, h=10, w=28, b1=20,
                          b2=14, tile=1, iters=2, causal_chunk=2, q_frame_offset=4, dtype="bf16",
                          scale=128 ** -0.5, rope=False)
    for label, wl, heads in (("first", first, [0, 2]), ("second (smaller)", second, None)):
        arrays, want, out = run_pair(wl)
        assert torch.isfinite(out.float()).all()
        assert torch.equal(out, want), f"{label} call differs from the workspace call"
        err, omax = compare_heads(wl, arrays, out, heads=heads)
        print(f"  {label}: max|gpu-oracle| = {err:.3e} at max|O| = {omax:.3e}", flush=True)
        assert err <= 2e-2 and err <= 4e-2 * omax + 1e-3


def test_noalloc_fp32_path_and_regular_monarch():
    wl = syn.WORKLOADS["C0"]
    arrays, want, out = run_pair(wl)
    assert torch.equal(out, want)
    err, _ = compare_heads(wl, arrays, out)
    assert err <= 1e-4
