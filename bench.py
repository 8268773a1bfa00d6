#!/usr/bin/env python3
"""Benchmark of the MonarchRT attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C1]

One "step" is one whole monarch_attn_fwd call (all 2T kernels of App. A's iteration plus the
output product) on one batch of seeded synthetic inputs that are already resident in HBM.
Prints ONE JSON line: the headline metric (ms per call at the 4680x4680, 12-head Self-Forcing
chunk shape), the roofline of the dominant kernel (duration measured with HIP events recorded
by the library around every launch), the in-library dense baseline, and the fp64 CPU oracle
timed on the host cores.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "MonarchRT attention ms/call + % MFMA/HBM roofline at 4680x4680, 12 heads"
PEAK_MFMA_BF16 = 2.5e15      # FLOP/s, dense bf16 MFMA, MI355X published
PEAK_HBM = 8.0e12            # B/s, MI355X published

PROFILES = os.path.join(ROOT, "profiles")


def recorded_traffic(workload):
    """HBM bytes per launch (fetched, written) of every kernel of a workload, as RECORDED in the
    committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary profiles/monarch_<workload>_kernels.md
    (counter values in KiB per dispatch, scaled by what the same counter reads for a device copy of
    known size; the summary names the commit it was taken at).  Not measured in this run.
    Returns ({launch name: (fetched, written)}, source text) or ({}, None) if there is no summary."""
    path = os.path.join(PROFILES, f"monarch_{workload}_kernels.md")
    if not os.path.exists(path):
        return {}, None
    out, commit, in_table = {}, "unknown", False
    for line in open(path):
        if line.lower().startswith("library sources at commit"):
            commit = line.split(":", 1)[1].strip().strip("`. ")
        if line.startswith("## "):
            in_table = "HBM traffic" in line
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if not in_table or len(cells) != 5 or not cells[0].startswith("`"):
            continue
        kernel = cells[0].strip("`")
        try:
            fetched, written = float(cells[2]) * 1e6, float(cells[4]) * 1e6
        except ValueError:
            continue
        if "stage_r<" in kernel:
            targs = [a.strip() for a in kernel[kernel.index("<") + 1:kernel.rindex(">")].split(",")]
            name = "stage_R" + ("_first" if targs[2] == "true" else "") + ("_last" if targs[3] == "true" else "")
        elif "stage_l_refine" in kernel:
            name = "stage_L_refine"
        elif "stage_l_out" in kernel:
            name = "stage_L_out"
        else:
            continue
        out[name] = (fetched, written)
    return out, f"recorded in profiles/{os.path.basename(path)} at commit {commit}, not measured in this run"


def dense_flops(wl):
    """4 d per (query, visible key) pair of the dense baseline (both products), all heads."""
    hw = wl.h * wl.w
    pairs = 0
    for fq in range(wl.f_q):
        seen = wl.f_kv if wl.causal_chunk == 0 else min(
            wl.f_kv, ((wl.q_frame_offset + fq) // wl.causal_chunk + 1) * wl.causal_chunk)
        pairs += hw * seen * hw
    return 4.0 * wl.head_dim * wl.batch * wl.heads * pairs


def visible_pairs(wl):
    """sum over query tiles of their visible key tiles (tile-level chunk-causal reading)."""
    if wl.tile == 0:
        return 1
    rows_q, rows_k, cols = wl.block_grid()
    c2 = cols // wl.b2
    c1q, c1k = rows_q // wl.b1, rows_k // wl.b1
    if wl.tile_h:
        # neighbourhood tiles: tile rows per chunk = (chunk frames / n_f) * (h / n_h)
        n_f, bands = wl.b1 // wl.tile_h, wl.h // wl.tile_h
        ct, qt0 = (wl.causal_chunk // n_f) * bands, (wl.q_frame_offset // n_f) * bands
    else:
        rpf = rows_q // wl.f_q                 # block-grid rows per frame (mask: frame axis slowest)
        ct, qt0 = wl.causal_chunk * rpf // wl.b1, wl.q_frame_offset * rpf // wl.b1
    total = 0
    for a in range(c1q):
        rows = min(c1k, ((qt0 + a) // ct + 1) * ct) if wl.causal_chunk else c1k
        total += c2 * rows * c2
    return total


def kernel_models(wl, es):
    """Algorithmic FLOPs and bytes of every launch of one call, in launch order.

    Per visible tile pair, with n_t = b1*b2 tokens per tile: the R-side products (beta_R,
    alpha_L, Y) cost n_t*b2*d MACs each, the L-side products (beta_L, alpha_R or the output) cost
    n_t*b1*d MACs each.  Bytes count every operand and result of the launch once: the alpha_L /
    Y / alpha_R intermediates (n_t*d elements per pair), c_L (4 bytes per (pair, j, k)), and the
    Q / K / V / O tensors touched."""
    H = wl.batch * wl.heads
    P = visible_pairs(wl)
    nt, d = wl.b1 * wl.b2, wl.head_dim
    inter = H * P * nt * d * es
    cl = H * P * nt * 4
    qb, ob = H * wl.n_q * d * es, H * wl.n_q * d * es
    # visible key tokens (union over query tiles) -- all query tiles of the named workloads share it
    kb = H * (P // max(1, wl.ntq)) * nt * d * es
    out = []
    for t in range(1, wl.iters + 1):
        first, last = t == 1, t == wl.iters
        fl = 2 * H * P * nt * wl.b2 * d * (3 if last else 2)
        by = (qb if first else inter) + kb + inter + cl + ((kb + inter) if last else 0)
        out.append(dict(name="stage_R" + ("_first" if first else "") + ("_last" if last else ""),
                        kind=1 | (16 if first else 0) | (32 if last else 0), flops=fl, bytes=by))
        fl = 2 * H * P * nt * wl.b1 * d * 2
        by = inter + cl + qb + ((inter + ob) if last else inter)
        out.append(dict(name="stage_L_out" if last else "stage_L_refine",
                        kind=2 | (32 if last else 0), flops=fl, bytes=by))
    return out


def backward_flops(wl):
    """2 x MACs of the products the backward pass has to form once (recomputation of logits in
    extra passes not counted): the forward intermediates (T stage R, T-1 stage L), and per
    iteration 5 products of b1 x NK x d on the L side and 5 (7 at t = T) of b2 x b2 x d on the R
    side, per visible tile pair."""
    H = wl.batch * wl.heads
    P = visible_pairs(wl)
    nt, d, T = wl.b1 * wl.b2, wl.head_dim, wl.iters
    r_prod, l_prod = nt * wl.b2 * d, nt * wl.b1 * d          # MACs of one product per tile pair
    fwd = T * 2 * r_prod + r_prod + (T - 1) * 2 * l_prod
    bwd = T * 5 * l_prod + T * 5 * r_prod + 2 * r_prod
    return 2 * H * P * (fwd + bwd)


def bench_backward(args, wl, lib, pkg, syn, torch, np, host, dev, prob, stream):
    Qh, Kh, Vh = host
    Q, K, V = dev
    rng = np.random.default_rng(1234)
    dOh = rng.standard_normal(Qh.shape).astype(np.float32)
    if wl.dtype == "bf16":
        dOh = syn.round_to_bf16(dOh)
    dO = torch.from_numpy(dOh).to(Q.device).to(Q.dtype)
    pref = ctypes.byref(prob)
    nws = lib.monarch_attn_bwd_workspace_bytes(pref, wl.b1, wl.b2, wl.tile, wl.iters)
    if nws == 0:
        raise RuntimeError(f"backward pass not available for {wl.name}: {pkg.last_error()}")
    ws = torch.empty(nws, dtype=torch.uint8, device=Q.device)
    dQ = torch.empty(Q.shape, dtype=torch.float32, device=Q.device)
    dK = torch.empty(K.shape, dtype=torch.float32, device=Q.device)
    dV = torch.empty(V.shape, dtype=torch.float32, device=Q.device)

    def step():
        st = lib.monarch_attn_bwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(), dQ.data_ptr(),
                                  dK.data_ptr(), dV.data_ptr(), pref, wl.b1, wl.b2, wl.tile, wl.iters,
                                  wl.causal_chunk, ws.data_ptr(), nws, stream)
        if st != 0:
            raise RuntimeError(f"monarch_attn_bwd failed: {pkg.last_error()}")

    steps, warmup = min(args.steps, 20), min(args.warmup, 3)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    # the same training step as two calls that hand the intermediates over (forward that saves them,
    # reverse sweep from them), when the workspace of all heads fits half of the device memory
    saved = None
    nsv = lib.monarch_attn_bwd_saved_workspace_bytes(pref, wl.b1, wl.b2, wl.tile, wl.iters)
    if 0 < nsv < torch.cuda.get_device_properties(Q.device).total_memory // 2:
        ws = None                       # release the per-pass workspace first
        wsv = torch.empty(nsv, dtype=torch.uint8, device=Q.device)
        O = torch.empty_like(Q)

        def fwd_save():
            st = lib.monarch_attn_fwd_save(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), pref, wl.b1,
                                           wl.b2, wl.tile, wl.iters, wl.causal_chunk, wsv.data_ptr(), nsv, stream)
            if st != 0:
                raise RuntimeError(f"monarch_attn_fwd_save failed: {pkg.last_error()}")

        def bwd_saved():
            st = lib.monarch_attn_bwd_saved(Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(),
                                            dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), pref, wl.b1, wl.b2,
                                            wl.tile, wl.iters, wl.causal_chunk, wsv.data_ptr(), nsv, stream)
            if st != 0:
                raise RuntimeError(f"monarch_attn_bwd_saved failed: {pkg.last_error()}")

        times = []
        for fn in (fwd_save, bwd_saved):
            for _ in range(warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) * 1e3 / steps)
        saved = {"fwd_save_ms": times[0], "bwd_saved_ms": times[1], "workspace_mb": nsv / 1e6}
    flops = backward_flops(wl)
    ach = flops / (ms / 1e3) / 1e12
    # the library's rule for running every stage on the bf16 matrix unit
    on_mfma = wl.dtype == "bf16" and wl.head_dim in (64, 128) and wl.b2 <= 96 and wl.b1 <= 144
    peak = 2500.0 if on_mfma else 157.3
    cpu = parity = None
    if not args.no_cpu_baseline:
        from oracle import monarch_oracle as mo
        kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=wl.tile,
                  iters=wl.iters, causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset,
                  scale=wl.scale, assign=wl.assign, tile_h=wl.tile_h)
        t0 = time.perf_counter()
        heads_run = 0
        while heads_run < wl.heads and time.perf_counter() - t0 < 15.0:
            ref = mo.monarch_attn_grad(*(torch.from_numpy(x[0, heads_run]) for x in (Qh, Kh, Vh)),
                                       torch.from_numpy(dOh[0, heads_run]), **kw)
            if heads_run == 0:
                parity = max((g[0, 0].double().cpu() - r).abs().max().item() for g, r in zip((dQ, dK, dV), ref))
            heads_run += 1
        dt = time.perf_counter() - t0
        cpu = dict(value=dt / heads_run * wl.batch * wl.heads * 1e3, unit="ms/call",
                   cores=torch.get_num_threads(), kind="oracle",
                   sample=f"{heads_run} of {wl.heads} heads of {wl.name} (reverse-mode gradients of the fp64 "
                          f"oracle) in {dt:.1f} s, scaled to all heads")
    print(json.dumps({
        "metric": "monarch_attn_bwd_ms", "value": ms, "unit": "ms/call", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if on_mfma else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name} backward: {wl.heads} heads x d{wl.head_dim}, N_q={wl.n_q}, "
                               f"N_kv={wl.n_kv}, blocks ({wl.b1},{wl.b2}), T={wl.iters}",
                   "workspace_mb": nws / 1e6},
        "roofline": {"bound": "mfma" if on_mfma else "alu", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                     "frac": ach / peak, "traffic": None, "algorithmic_gflop": flops / 1e9,
                     "note": ("bf16 matrix-unit kernels" if on_mfma else "fp32 kernels (fp32 matrix instructions)")
                             + ", whole call: forward recomputation + reverse sweep; blocks of this size keep "
                               "the call latency-bound, far below either roofline"},
        "cpu_baseline": cpu, "parity_max_abs_err_head0": parity,
        "saved_intermediates": saved,
    }))


def measure_forward(wl, env, steps, warmup, *, head_groups=0, settle_s=0.0, with_dense=True, with_oracle=True,
                    oracle_budget_s=0.0, calibration_copy_mb=0, copy_gbs=None):
    """One workload through monarch_attn_fwd: whole-call time (default launch configuration),
    per-launch durations (HIP events recorded by the library around every launch, one head group so
    that a launch covers all heads), roofline of the dominant launch, dense baseline, head-0 parity
    against the oracle and, with a time budget, the oracle's own time on the host cores."""
    np, torch, pkg, binding, syn, lib = env
    dev = torch.device("cuda:0")
    tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
    es = 4 if wl.dtype == "f32" else 2
    Qh, Kh, Vh = syn.make_inputs(wl)
    Q, K, V = (torch.from_numpy(x).to(dev).to(tdt) for x in (Qh, Kh, Vh))
    O = torch.empty_like(Q)
    prob = binding._torch_problem(Q, K, V, O, wl.f_q, wl.f_kv, wl.h, wl.w, wl.q_frame_offset,
                                  wl.scale, pkg.MRT_COMPUTE_DEFAULT, wl.assign, wl.tile_h, head_groups)
    nws = pkg.monarch_attn_workspace_bytes(prob, wl.b1, wl.b2, wl.tile, wl.iters)
    ws = torch.empty(nws, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    pq, pk, pv, po, pw = Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), ws.data_ptr()
    pref = ctypes.byref(prob)

    def step(p=pref):
        st = lib.monarch_attn_fwd(pq, pk, pv, po, p, wl.b1, wl.b2, wl.tile, wl.iters,
                                  wl.causal_chunk, pw, nws, stream)
        if st != 0:
            raise RuntimeError(f"monarch_attn_fwd failed: {pkg.last_error()}")

    if calibration_copy_mb:
        src = torch.empty(calibration_copy_mb * 1000 * 1000 // 4, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if settle_s > 0:
        # the other named configurations follow CPU-side work (parity check of the previous one)
        # during which the GPU idled: run untimed calls until the clocks have settled, then time
        # about settle_s seconds of calls (at least `steps`)
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < settle_s:
            step()
            n += 1
            if n % 8 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        steps = max(steps, int(n * 1.0))
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    # ---- per-launch durations.  Each launch is repeated inside its event bracket so that the
    # bracket's own cost and the dispatch latency of a short kernel do not count as kernel time;
    # one head group, so that every launch covers all heads (what the rocprofv3 summaries under
    # profiles/ record with --head-groups 1)
    prob1 = binding._torch_problem(Q, K, V, O, wl.f_q, wl.f_kv, wl.h, wl.w, wl.q_frame_offset,
                                   wl.scale, pkg.MRT_COMPUTE_DEFAULT, wl.assign, wl.tile_h, 1)
    pref1 = ctypes.byref(prob1)
    reps = max(1, min(16, round(0.5 / ms_per_step)))
    psteps = max(3, min(steps, int(200.0 / (ms_per_step * reps)) + 1))      # about 0.2 s of launches
    binding.profile_enable(reps)
    for _ in range(psteps):
        step(pref1)
    torch.cuda.synchronize()
    recs = binding.profile_read()
    binding.profile_enable(0)
    models = kernel_models(wl, es)
    per_call = len(recs) // psteps
    passes = per_call // len(models)           # passes per call (1 unless the workspace was capped)
    kernels = []
    for i, mdl in enumerate(models):
        tot = 0.0
        for s in range(psteps):
            for g in range(passes):
                ms, kind = recs[s * per_call + g * len(models) + i]
                assert kind == mdl["kind"], (kind, mdl)
                tot += ms
        dur = tot / psteps / 1e3               # seconds per call spent in this launch (all passes)
        kernels.append(dict(name=mdl["name"], launches_per_call=passes, ms_per_call=dur * 1e3,
                            gflop=mdl["flops"] / 1e9, mbytes=mdl["bytes"] / 1e6,
                            tflops=mdl["flops"] / dur / 1e12, gbps=mdl["bytes"] / dur / 1e9,
                            frac_mfma=mdl["flops"] / dur / PEAK_MFMA_BF16,
                            frac_hbm=mdl["bytes"] / dur / PEAK_HBM))
    # the dominant kernel: the longest launch; launches within 5 % of it count as tied, and of
    # those the one furthest from its roofline is reported (so the choice does not flip from run
    # to run when several launches take about the same time)
    longest = max(k["ms_per_call"] for k in kernels)
    tied = [k for k in kernels if k["ms_per_call"] >= 0.95 * longest]
    dom = min(tied, key=lambda k: max(k["frac_hbm"], k["frac_mfma"]))
    dmodel = next(m for m in models if m["name"] == dom["name"])
    hbm_bound = dmodel["bytes"] / PEAK_HBM >= dmodel["flops"] / PEAK_MFMA_BF16
    launch_s = dom["ms_per_call"] / 1e3 / dom["launches_per_call"]
    if hbm_bound:
        ach = dmodel["bytes"] / dom["launches_per_call"] / launch_s / 1e9
        roof = dict(bound="hbm", achieved=ach, peak=PEAK_HBM / 1e9, unit="GB/s", frac=ach / (PEAK_HBM / 1e9))
    else:
        ach = dmodel["flops"] / dom["launches_per_call"] / launch_s / 1e12
        roof = dict(bound="mfma", achieved=ach, peak=PEAK_MFMA_BF16 / 1e12, unit="TFLOP/s",
                    frac=ach / (PEAK_MFMA_BF16 / 1e12))
    if roof["bound"] == "hbm" and copy_gbs:
        roof.update(copy_gbs=copy_gbs, frac_of_copy=roof["achieved"] / copy_gbs)
    traffic, source = recorded_traffic(wl.name)
    tr = traffic.get(dom["name"]) if passes == 1 else None     # the summaries are per full-size launch
    roof.update(kernel=dom["name"], tied_with=[k["name"] for k in tied if k is not dom],
                launch_us=launch_s * 1e6, launch_repeats=reps,
                traffic=sum(tr) if tr else None, traffic_unit="bytes per launch (fetch + write)",
                traffic_source=source if tr else None,
                algorithmic_bytes=dmodel["bytes"] / dom["launches_per_call"])
    tot_flops = sum(m["flops"] for m in models)
    compulsory = (wl.batch * wl.heads) * (2 * wl.n_q + 2 * wl.n_kv) * wl.head_dim * es

    # ---- dense baseline in the same library, same inputs
    dense_ms = None
    if with_dense:
        Od = torch.empty_like(Q)

        def dstep():
            st = lib.dense_attn_fwd(pq, pk, pv, Od.data_ptr(), pref, wl.causal_chunk, stream)
            if st != 0:
                raise RuntimeError(f"dense_attn_fwd failed: {pkg.last_error()}")
        nd = max(3, min(steps, 20))
        for _ in range(2):
            dstep()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nd):
            dstep()
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - t0) * 1e3 / nd

    # ---- CPU oracle on the host cores (a reported baseline, not the target) + parity spot check
    cpu = parity = None
    if with_oracle:
        from oracle import monarch_oracle as mo

        def oracle_head(hd):
            return mo.monarch_attn(torch.from_numpy(Qh[0, hd]), torch.from_numpy(Kh[0, hd]),
                                   torch.from_numpy(Vh[0, hd]), f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h,
                                   w=wl.w, b1=wl.b1, b2=wl.b2, tile=wl.tile, iters=wl.iters,
                                   causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset,
                                   scale=wl.scale, assign=wl.assign, tile_h=wl.tile_h)
        step()
        torch.cuda.synchronize()
        ref0 = oracle_head(0)                       # also warms the CPU libraries up
        parity = (O[0, 0].float().cpu().double() - ref0).abs().max().item()
        if oracle_budget_s > 0:
            # a bounded sample: heads of this workload, one after the other (cycling through them
            # if they are all done early), until the budget is spent
            heads_run, t0 = 0, time.perf_counter()
            while (time.perf_counter() - t0) < oracle_budget_s:
                oracle_head(heads_run % wl.heads)
                heads_run += 1
            t_acc = time.perf_counter() - t0
            cpu = dict(value=t_acc / heads_run * wl.heads * wl.batch * 1e3, unit="ms/call",
                       cores=torch.get_num_threads(), kind="oracle",
                       sample=f"{heads_run} single-head oracle calls on the heads of {wl.name} (cycling "
                              f"through its {wl.heads} heads) in {t_acc:.1f} s, scaled to one call over all "
                              f"heads (heads are independent)")
    del Q, K, V, O, ws
    torch.cuda.empty_cache()
    return dict(
        ms=ms_per_step, roofline=roof, kernels=kernels, cpu=cpu, parity=parity, dense_ms=dense_ms,
        config={"workload": f"{wl.name}: {wl.heads} heads x d{wl.head_dim}, grid ({wl.f_q}|{wl.f_kv},"
                            f"{wl.h},{wl.w}), N_q={wl.n_q}, N_kv={wl.n_kv}, "
                            f"{'tiled' if wl.tile else 'regular'} Monarch ({wl.b1},{wl.b2}) on ({wl.assign.replace('_', ',')}), T={wl.iters}, "
                            f"causal_chunk={wl.causal_chunk}",
                "scale": wl.scale, "workspace_mb": nws / 1e6, "head_groups": head_groups or "auto",
                "passes_per_call": passes},
        whole_call={"algorithmic_gflop": tot_flops / 1e9, "tflops": tot_flops / (ms_per_step / 1e3) / 1e12,
                    "frac_mfma": tot_flops / (ms_per_step / 1e3) / PEAK_MFMA_BF16,
                    "compulsory_mbytes": compulsory / 1e6,
                    "frac_hbm_compulsory": compulsory / (ms_per_step / 1e3) / PEAK_HBM,
                    "sum_kernel_ms": sum(k["ms_per_call"] for k in kernels)},
        dense_frac_mfma=(dense_flops(wl) / (dense_ms / 1e3) / PEAK_MFMA_BF16) if dense_ms else None)


def measured_copy_rate(torch):
    """What a plain device-to-device copy of 256 MB sustains on this machine (read + write bytes per
    second): the ceiling a memory-bound kernel can actually reach, next to the published peak."""
    dev = torch.device("cuda:0")
    csrc = torch.empty(64 * 1000 * 1000, dtype=torch.float32, device=dev).normal_()
    cdst = torch.empty_like(csrc)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(2):
        cdst.copy_(csrc)
    ev0.record()
    for _ in range(5):
        cdst.copy_(csrc)
    ev1.record()
    torch.cuda.synchronize()
    return 5 * 2 * csrc.numel() * 4 / (ev0.elapsed_time(ev1) / 1e3) / 1e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C1")
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads measured after the headline one and reported under "
                         "other_workloads (default: C2,C3,C4 when the headline is C1; 'none' for none)")
    ap.add_argument("--op", default="fwd", choices=["fwd", "bwd"],
                    help="fwd: the forward operator (the headline metric); bwd: the backward pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--head-groups", type=int, default=0,
                    help="head groups run concurrently by the library in the timed calls (0 = library default)")
    ap.add_argument("--calibration-copy-mb", type=int, default=0,
                    help="also run a plain device copy of this many MB (3 times) so that a "
                         "rocprofv3 --pmc run of this command holds a dispatch of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(heads are independent and would shard over GPUs without any exchange).",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2602_12271_amd as pkg
    from paper_2602_12271_amd import binding
    from workloads import synthetic as syn

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    lib = pkg.load_library()          # raises if the HIP library is missing: no fallback
    env = (np, torch, pkg, binding, syn, lib)
    wl = syn.WORKLOADS[args.workload]

    if args.op == "bwd":
        dev = torch.device("cuda:0")
        if args.head_groups:
            binding.set_head_groups(args.head_groups)
        tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
        Qh, Kh, Vh = syn.make_inputs(wl)
        Q, K, V = (torch.from_numpy(x).to(dev).to(tdt) for x in (Qh, Kh, Vh))
        prob = binding._torch_problem(Q, K, V, torch.empty_like(Q), wl.f_q, wl.f_kv, wl.h, wl.w,
                                      wl.q_frame_offset, wl.scale, pkg.MRT_COMPUTE_DEFAULT, wl.assign, wl.tile_h)
        stream = torch.cuda.current_stream(dev).cuda_stream
        return bench_backward(args, wl, lib, pkg, syn, torch, np, (Qh, Kh, Vh), (Q, K, V), prob, stream)

    copy_gbs = measured_copy_rate(torch)
    head = measure_forward(wl, env, args.steps, args.warmup, head_groups=args.head_groups,
                           with_dense=not args.no_dense, with_oracle=not args.no_cpu_baseline,
                           oracle_budget_s=10.0, calibration_copy_mb=args.calibration_copy_mb,
                           copy_gbs=copy_gbs)
    also = args.also if args.also is not None else ("C2,C3,C4" if args.workload == "C1" else "none")
    others = []
    for name in [n for n in also.split(",") if n and n != "none"]:
        # the other named configurations: same measurement, fewer timed calls, head 0 through the
        # oracle, no oracle timing
        w2 = syn.WORKLOADS[name]
        r = measure_forward(w2, env, max(5, min(args.steps, 20)), max(2, min(args.warmup, 5)),
                            head_groups=args.head_groups, settle_s=0.1,
                            with_dense=not args.no_dense and name != "C4",
                            with_oracle=not args.no_cpu_baseline, copy_gbs=copy_gbs)
        others.append({"workload": r["config"]["workload"], "ms_per_call": r["ms"],
                       "dominant_kernel": r["roofline"]["kernel"], "bound": r["roofline"]["bound"],
                       "frac": r["roofline"]["frac"], "launch_us": r["roofline"]["launch_us"],
                       "algorithmic_bytes": r["roofline"]["algorithmic_bytes"],
                       "traffic": r["roofline"]["traffic"], "traffic_source": r["roofline"]["traffic_source"],
                       "frac_mfma_whole_call": r["whole_call"]["frac_mfma"],
                       "kernels_ms": {f"{i}:{k['name']}": round(k["ms_per_call"], 5) for i, k in enumerate(r["kernels"])},
                       "dense_baseline_ms": r["dense_ms"],
                       "parity_max_abs_err_head0": r["parity"]})

    out = {
        "metric": METRIC, "value": head["ms"], "unit": "ms/call", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": head["config"],
        "roofline": head["roofline"],
        "cpu_baseline": head["cpu"],
        "whole_call": head["whole_call"],
        "kernels": head["kernels"],
        "dense_baseline_ms": head["dense_ms"],
        "dense_frac_mfma": head["dense_frac_mfma"],
        "speedup_vs_dense": (head["dense_ms"] / head["ms"]) if head["dense_ms"] else None,
        "parity_max_abs_err_head0": head["parity"],
        "other_workloads": others,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
