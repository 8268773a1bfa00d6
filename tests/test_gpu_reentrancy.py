"""Several forward calls in flight at once: two caller streams, two host threads, head groups on.

Calls with more than one head group share the device's helper streams and fork / join events; the
library hands them to one call at a time.  Each call here has its own inputs, output and workspace,
and its result must equal, bit for bit, what the same call gives when it runs alone."""
import threading

import pytest
import torch

import paper_2602_12271_amd as pkg
from workloads import synthetic as syn

from gpu_harness import to_device

pytestmark = pytest.mark.gpu


def call_kwargs(wl, **extra):
    kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=wl.tile, iters=wl.iters,
              causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset, scale=wl.scale)
    kw.update(extra)
    return kw


def workspace_for(wl):
    prob = pkg.make_problem(batch=wl.batch, heads=wl.heads, head_dim=wl.head_dim, f_q=wl.f_q, f_kv=wl.f_kv,
                            h=wl.h, w=wl.w, scale=wl.scale, q_frame_offset=wl.q_frame_offset)
    n = pkg.monarch_attn_workspace_bytes(prob, wl.b1, wl.b2, wl.tile, wl.iters)
    return torch.empty(n, dtype=torch.uint8, device="cuda:0")


def test_two_streams_with_head_groups_give_the_single_call_bits():
    wls = [syn.variant("C2", heads=6), syn.variant("C1", heads=5, seed=3)]
    devs = [to_device(wl, syn.make_inputs(wl)) for wl in wls]
    alone = []
    for wl, dev in zip(wls, devs):
        alone.append(pkg.monarch_attn_fwd(*dev, **call_kwargs(wl, head_groups=1)).clone())
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [torch.empty_like(d[0]) for d in devs]
    wss = [workspace_for(wl) for wl in wls]
    torch.cuda.synchronize()
    for rep in range(6):
        for o in outs:
            o.zero_()
        torch.cuda.synchronize()
        # interleaved enqueue from one host thread: both calls fork to the same helper streams
        for i in (0, 1):
            pkg.monarch_attn_fwd(*devs[i], out=outs[i], workspace=wss[i], stream=streams[i].cuda_stream,
                                 **call_kwargs(wls[i], head_groups=2))
        torch.cuda.synchronize()
        for i in (0, 1):
            assert torch.equal(outs[i], alone[i]), f"repeat {rep}, call {i} differs"


def test_two_host_threads_with_head_groups_give_the_single_call_bits():
    wls = [syn.variant("C2", heads=4), syn.variant("C2", heads=4, seed=9)]
    devs = [to_device(wl, syn.make_inputs(wl)) for wl in wls]
    alone = [pkg.monarch_attn_fwd(*dev, **call_kwargs(wl, head_groups=1)).clone() for wl, dev in zip(wls, devs)]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [torch.empty_like(d[0]) for d in devs]
    wss = [workspace_for(wl) for wl in wls]
    torch.cuda.synchronize()
    errors = []

    def worker(i):
        try:
            for rep in range(20):
                pkg.monarch_attn_fwd(*devs[i], out=outs[i], workspace=wss[i], stream=streams[i].cuda_stream,
                                     **call_kwargs(wls[i], head_groups=2 + (rep % 2)))
                streams[i].synchronize()
                if not torch.equal(outs[i], alone[i]):
                    errors.append(f"thread {i}, repeat {rep}: result differs")
                    return
        except Exception as exc:                      # surfaced in the main thread below
            errors.append(repr(exc))

    threads = [threading.Thread(target=worker, args=(i,)) for i in (0, 1)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_head_groups_field_overrides_the_process_default():
    wl = syn.variant("C2", heads=5)
    dev = to_device(wl, syn.make_inputs(wl))
    ref = pkg.monarch_attn_fwd(*dev, **call_kwargs(wl, head_groups=1)).clone()
    try:
        pkg.binding.set_head_groups(4)
        one = pkg.monarch_attn_fwd(*dev, **call_kwargs(wl, head_groups=1))
        three = pkg.monarch_attn_fwd(*dev, **call_kwargs(wl, head_groups=3))
        torch.cuda.synchronize()
        assert torch.equal(one, ref) and torch.equal(three, ref)
    finally:
        pkg.binding.set_head_groups(0)
