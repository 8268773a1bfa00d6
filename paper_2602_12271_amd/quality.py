"""Approximation quality of MonarchRT attention against dense attention on the GPU.

The attention matrices themselves are materialised with the library's own kernels: feeding the
identity as V, head_dim columns at a time, makes the output the corresponding columns of the
matrix (O = M V).  From the two matrices this reports, per configuration, the relative Frobenius
error, the mean row-wise KL(M || A) that the refinement iterations descend on (App. A), and the
relative error of the attention output for the given V.

    python -m paper_2602_12271_amd.quality --workload C1 --iters 1 2 3

Inputs follow the paper's informal model of video attention maps (Sec. 3.1: separable positional
part + sparse semantic part + noise), synthetic and seeded; see workloads/synthetic.py."""
from __future__ import annotations

import argparse
import json
import sys


def attention_matrix(apply, n_q: int, n_kv: int, d: int, dtype, device):
    """M [n_q, n_kv] with M = apply(V) for V running over column blocks of the identity.
    apply maps V [1, 1, n_kv, d] to O [1, 1, n_q, d]."""
    import torch
    M = torch.empty(n_q, n_kv, dtype=torch.float32, device=device)
    for c0 in range(0, n_kv, d):
        cols = min(d, n_kv - c0)
        V = torch.zeros(1, 1, n_kv, d, dtype=dtype, device=device)
        idx = torch.arange(cols, device=device)
        V[0, 0, c0 + idx, idx] = 1
        M[:, c0:c0 + cols] = apply(V)[0, 0, :, :cols].float()
    return M


def compare(M, A, O_m, O_a):
    """Relative Frobenius error, mean row KL(M || A) and relative output error."""
    import torch
    fro = ((M - A).norm() / A.norm()).item()
    tiny = 1e-30
    kl = (M * (torch.log(M.clamp_min(tiny)) - torch.log(A.clamp_min(tiny)))).sum(1).mean().item()
    out = ((O_m - O_a).norm() / O_a.norm()).item()
    return dict(fro_rel=fro, kl_rows_mean=kl, out_rel=out)


def report(wl, configs, head: int = 0, inputs=None):
    """configs: iterable of dict(b1, b2, tile, iters[, assign]).  Returns one result dict each."""
    import torch
    import paper_2602_12271_amd as pkg
    from workloads import synthetic as syn

    dev = torch.device("cuda:0")
    tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
    Q, K, V = inputs if inputs is not None else syn.make_structured_head(wl, 0, head)
    Qd, Kd, Vd = (torch.from_numpy(x).to(dev).to(tdt)[None, None] for x in (Q, K, V))
    grid = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, causal_chunk=wl.causal_chunk,
                q_frame_offset=wl.q_frame_offset, scale=wl.scale)
    dense = lambda v: pkg.dense_attn_fwd(Qd, Kd, v, **grid)
    A = attention_matrix(dense, wl.n_q, wl.n_kv, wl.head_dim, tdt, dev)
    O_a = dense(Vd)[0, 0].float()
    rows = []
    for c in configs:
        kw = dict(grid, b1=c["b1"], b2=c["b2"], tile=c["tile"], iters=c["iters"],
                  assign=c.get("assign", "fh_w"))
        mon = lambda v: pkg.monarch_attn_fwd(Qd, Kd, v, **kw)
        M = attention_matrix(mon, wl.n_q, wl.n_kv, wl.head_dim, tdt, dev)
        r = dict(c)
        r.update(compare(M, A, mon(Vd)[0, 0].float(), O_a))
        r["row_sum_err"] = (M.sum(1) - 1).abs().max().item()
        rows.append(r)
    torch.cuda.synchronize()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="C1")
    ap.add_argument("--iters", type=int, nargs="+", default=[1, 2, 3])
    ap.add_argument("--head", type=int, default=0)
    args = ap.parse_args()
    from workloads import synthetic as syn
    wl = syn.WORKLOADS[args.workload]
    rq, _, cols = wl.block_grid()
    shapes = [dict(b1=wl.b1, b2=wl.b2, tile=wl.tile)]
    if wl.assign == "fh_w" and wl.f_q == wl.f_kv:
        # the regular parameterization and two refinements of it (Sec. 4.2: finer tiles are
        # strictly more expressive)
        shapes = [dict(b1=rq, b2=cols, tile=0), dict(b1=wl.h * wl.f_q, b2=cols // 2, tile=1),
                  dict(b1=wl.h, b2=cols // 2, tile=1)]
    configs = [dict(s, iters=t, assign=wl.assign) for s in shapes for t in args.iters]
    for r in report(wl, configs, head=args.head):
        print(json.dumps(r))


if __name__ == "__main__":
    sys.exit(main())
