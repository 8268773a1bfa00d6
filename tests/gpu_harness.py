"""Shared helpers for the GPU parity tests: run a workload through the C ABI (via the
binding) and through the fp64 oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

import paper_2602_12271_amd as pkg
from oracle import monarch_oracle as mo
from workloads import synthetic as syn


def torch_dtype(wl):
    return torch.float32 if wl.dtype == "f32" else torch.bfloat16


def to_device(wl, arrays, dev="cuda:0"):
    return tuple(torch.from_numpy(x).to(dev).to(torch_dtype(wl)) for x in arrays)


def run_monarch_gpu(wl, Qd, Kd, Vd, compute=pkg.MRT_COMPUTE_DEFAULT, workspace=None):
    O = pkg.monarch_attn_fwd(Qd, Kd, Vd, f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1,
                             b2=wl.b2, tile=wl.tile, iters=wl.iters, causal_chunk=wl.causal_chunk,
                             q_frame_offset=wl.q_frame_offset, scale=wl.scale, compute=compute,
                             workspace=workspace, assign=wl.assign, tile_h=wl.tile_h)
    torch.cuda.synchronize()
    return O


def run_dense_gpu(wl, Qd, Kd, Vd, compute=pkg.MRT_COMPUTE_DEFAULT):
    O = pkg.dense_attn_fwd(Qd, Kd, Vd, f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w,
                           causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset,
                           scale=wl.scale, compute=compute)
    torch.cuda.synchronize()
    return O


def oracle_monarch_head(wl, Q, K, V):
    return mo.monarch_attn(torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V),
                           f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2,
                           tile=wl.tile, iters=wl.iters, causal_chunk=wl.causal_chunk,
                           q_frame_offset=wl.q_frame_offset, scale=wl.scale, assign=wl.assign, tile_h=wl.tile_h)


def oracle_dense_head(wl, Q, K, V):
    return mo.dense_attn(torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V),
                         f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, causal_chunk=wl.causal_chunk,
                         q_frame_offset=wl.q_frame_offset, scale=wl.scale)


def compare_heads(wl, arrays, O_gpu, heads=None, oracle=oracle_monarch_head):
    """max |gpu - oracle| over the chosen heads (element by element), and the oracle's max |O|."""
    Q, K, V = arrays
    Oc = O_gpu.float().cpu().double()
    err, omax = 0.0, 0.0
    for b in range(wl.batch):
        for hd in (range(wl.heads) if heads is None else heads):
            ref = oracle(wl, Q[b, hd], K[b, hd], V[b, hd])
            e = (Oc[b, hd] - ref).abs().max().item()
            assert np.isfinite(e), f"non-finite output in head {hd}"
            err = max(err, e)
            omax = max(omax, ref.abs().max().item())
    return err, omax
