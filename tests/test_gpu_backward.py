"""GPU parity of the backward pass (gradients w.r.t. Q, K, V through every refinement iteration,
Sec. 4.3) against the fp64 oracle's gradients, through the C ABI.  The kernels compute in fp32
whatever the storage type, so the bar is the fp32 one, scaled by the size of the gradients."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2602_12271_amd as pkg
from oracle import monarch_oracle as mo
from workloads import synthetic as syn

from gpu_harness import to_device

pytestmark = pytest.mark.gpu

TOL = 1e-4


def small(dtype="f32", **kw):
    d = kw.pop("head_dim", 64)
    base = dict(name="small", batch=1, heads=2, head_dim=d, dtype=dtype, rope=False, scale=d ** -0.5,
                sigma_qk=1.0, sigma_v=1.0, causal_chunk=0, q_frame_offset=0, iters=2)
    base.update(kw)
    return syn.Workload(**base)


CASES = {
    "regular-T1": small(f_q=2, f_kv=2, h=5, w=13, b1=10, b2=13, tile=0, iters=1, head_dim=40),
    "regular-T2": small(batch=2, f_q=2, f_kv=2, h=5, w=13, b1=10, b2=13, tile=0, iters=2, head_dim=40),
    "regular-T3": small(f_q=2, f_kv=2, h=6, w=12, b1=12, b2=12, tile=0, iters=3),
    "tiled-rect-mask": small(f_q=2, f_kv=6, h=5, w=14, b1=10, b2=7, tile=1, iters=2, causal_chunk=2,
                             q_frame_offset=2),
    "tiled-rect-mask-T1": small(f_q=2, f_kv=6, h=5, w=14, b1=10, b2=7, tile=1, iters=1, causal_chunk=2,
                                q_frame_offset=2),
    "tiled-half-frames-T3": small(f_q=2, f_kv=4, h=6, w=8, b1=3, b2=4, tile=1, iters=3, causal_chunk=2,
                                  q_frame_offset=2),
    "fw_h-T2": small(f_q=2, f_kv=2, h=5, w=6, b1=12, b2=5, tile=0, iters=2, assign="fw_h"),
    "h_fw-tiled": small(f_q=2, f_kv=2, h=6, w=6, b1=3, b2=4, tile=1, iters=2, assign="h_fw"),
    "neighbourhood-mask": small(f_q=2, f_kv=4, h=4, w=8, b1=4, b2=4, tile=1, iters=2, causal_chunk=2,
                                q_frame_offset=0, tile_h=2),
    "bf16-storage": small("bf16", head_dim=128, f_q=2, f_kv=4, h=8, w=24, b1=16, b2=12, tile=1, iters=2),
    "bf16-ragged-T1": small("bf16", head_dim=128, f_q=2, f_kv=2, h=11, w=21, b1=22, b2=21, tile=0, iters=1),
    "bf16-ragged-T3": small("bf16", head_dim=128, f_q=2, f_kv=2, h=11, w=21, b1=22, b2=21, tile=0, iters=3),
    "bf16-d64-mask": small("bf16", head_dim=64, f_q=2, f_kv=6, h=4, w=12, b1=8, b2=6, tile=1, iters=2,
                           causal_chunk=2, q_frame_offset=2),
    # key ranges beyond 96 rows: stage L backward streams them in segments of 64.  120 key rows of
    # which the chunk-causal mask shows 80 (a ragged second segment), ragged query tiles
    "bf16-stream-mask": small("bf16", head_dim=128, f_q=2, f_kv=6, h=10, w=14, b1=20, b2=7, tile=1, iters=2,
                              causal_chunk=2, q_frame_offset=2),
    # streamed key range (156 rows) of which the first query tile row sees 26 under the mask: the waves
    # that own the upper half of every 64-key segment never meet a visible key there
    "bf16-stream-short-visible": small("bf16", head_dim=128, f_q=4, f_kv=12, h=13, w=39, b1=26, b2=39, tile=1,
                                       iters=1, causal_chunk=2, q_frame_offset=0),
    "bf16-stream-short-visible-T2": small("bf16", head_dim=64, f_q=4, f_kv=12, h=13, w=16, b1=26, b2=8, tile=1,
                                          iters=2, causal_chunk=2, q_frame_offset=0),
    # 64 < b2 <= 96: stage R backward with five or six arithmetic waves plus loader waves; at head_dim
    # 128 and t = T the transposed scale dS array takes the V tile's place
    "bf16-b2-80": small("bf16", head_dim=128, f_q=2, f_kv=4, h=8, w=80, b1=16, b2=80, tile=1, iters=2,
                        causal_chunk=2, q_frame_offset=2),
    "bf16-b2-72-T1": small("bf16", head_dim=64, f_q=2, f_kv=2, h=9, w=72, b1=18, b2=72, tile=0, iters=1),
    "bf16-b2-96": small("bf16", head_dim=128, f_q=2, f_kv=2, h=6, w=96, b1=12, b2=96, tile=0, iters=2),
    "bf16-b2-88-d64": small("bf16", head_dim=64, f_q=2, f_kv=6, h=5, w=88, b1=10, b2=88, tile=1, iters=3,
                            causal_chunk=2, q_frame_offset=4),
    # one head of the paper's 720p tile block (3h, w) = (135, 80) as a regular Monarch problem on a
    # 3-frame 720p latent chunk (10800 tokens)
    "bf16-720p-block": small("bf16", head_dim=128, heads=1, f_q=3, f_kv=3, h=45, w=80, b1=135, b2=80, tile=0,
                             iters=1),
    # 216 key rows, three query tiles (the odd tile count leaves a zero tile), three iterations
    "bf16-stream-T3": small("bf16", head_dim=64, f_q=2, f_kv=6, h=18, w=16, b1=36, b2=8, tile=1, iters=3),
    # nine query tiles (b1 = 135, the 720p tile height): ten waves, the wider transposed arrays,
    # the cols kernel's single LDS tile; half of the key tiles hidden
    "bf16-b1-135": small("bf16", head_dim=64, f_q=3, f_kv=6, h=45, w=16, b1=135, b2=8, tile=1, iters=2,
                         causal_chunk=3, q_frame_offset=0),
    # eight query tiles: the ten-wave streamed kernel with two waves that only write zero tiles
    "bf16-b1-120": small("bf16", head_dim=128, heads=1, f_q=4, f_kv=4, h=30, w=12, b1=120, b2=12, tile=0,
                         iters=2),
}


def on_matrix_unit(wl):
    """bf16 storage: stage L backward runs on the bf16 matrix unit (bf16 operands, fp32 accumulation)
    when b1 <= 144, stage R backward when b2 <= 96; the rest stays fp32."""
    return wl.dtype == "bf16" and (wl.b1 <= 144 or wl.b2 <= 96)


def run_case(wl, heads=None, compute=None):
    arrays = syn.make_inputs(wl)
    rng = np.random.default_rng(1234)
    dO = rng.standard_normal(arrays[0].shape).astype(np.float32)
    if wl.dtype == "bf16":
        dO = syn.round_to_bf16(dO)
    Qd, Kd, Vd, dOd = to_device(wl, arrays + (dO,))
    kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=wl.tile,
              iters=wl.iters, causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset,
              scale=wl.scale, assign=wl.assign, tile_h=wl.tile_h)
    compute = pkg.MRT_COMPUTE_DEFAULT if compute is None else compute
    dQ, dK, dV = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, compute=compute, **kw)
    torch.cuda.synchronize()
    bf16_ops = on_matrix_unit(wl) and compute == pkg.MRT_COMPUTE_DEFAULT
    worst = 0.0
    for b in range(wl.batch):
        for hd in (range(wl.heads) if heads is None else heads):
            ref = mo.monarch_attn_grad(*(torch.from_numpy(x[b, hd]) for x in arrays),
                                       torch.from_numpy(dO[b, hd]), **kw)
            for name, got, want in zip("QKV", (dQ, dK, dV), ref):
                g = got[b, hd].double().cpu()
                assert torch.isfinite(g).all(), f"non-finite d{name}"
                err = (g - want).abs().max().item()
                # the stated fp32 bar, and relative to the gradients' own size so that small
                # gradients cannot hide under it (measured: <= 2e-6 of the largest gradient);
                # with bf16 operands (2^-9 relative rounding of L, dZ, alpha_L, Y, Q, dO) the bar is
                # the bf16 one of the forward path, relative to the largest gradient
                gmax = want.abs().max().item()
                bar = 2e-2 * gmax if bf16_ops else min(TOL * max(1.0, gmax), 2e-5 * gmax + 1e-9)
                print(f"  head {hd} d{name}: max err {err:.3e} (max |grad| {want.abs().max().item():.3e})",
                      flush=True)
                assert err <= bar, (name, err, bar)
                worst = max(worst, err)
    return worst


@pytest.mark.parametrize("name", list(CASES))
def test_backward_matches_oracle(name):
    print(f"case {name}: {CASES[name]}", flush=True)
    run_case(CASES[name])


@pytest.mark.parametrize("compute", ["default", "f32"])
def test_backward_on_the_4680_token_chunk(compute):
    # the headline shape (12 heads, d = 128, regular (90, 52), T = 2), two heads through the oracle;
    # default arithmetic (bf16 matrix unit for stage L backward) and fp32 throughout
    wl = syn.variant("C1")
    run_case(wl, heads=[0, 11], compute=None if compute == "default" else pkg.MRT_COMPUTE_F32)


@pytest.mark.parametrize("name", ["bf16-storage", "bf16-ragged-T1"])
def test_backward_fp32_arithmetic_on_bf16_storage(name):
    run_case(CASES[name], compute=pkg.MRT_COMPUTE_F32)


@pytest.mark.timeout(600)
def test_backward_on_the_kv_cache_step_with_hidden_chunks():
    # the 3-frame query chunk against the 21-frame cache, tiles (90, 26), T = 2, with the query
    # chunk moved back so that 3 of the 7 cached chunks are hidden; one head
    wl = syn.variant("C3", heads=1, q_frame_offset=9)
    run_case(wl)


def test_backward_minimum_workspace_gives_same_result():
    wl = CASES["tiled-rect-mask"]
    arrays = syn.make_inputs(wl)
    dO = np.ones_like(arrays[0])
    Qd, Kd, Vd, dOd = to_device(wl, arrays + (dO,))
    kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=wl.tile,
              iters=wl.iters, causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset,
              scale=wl.scale)
    prob = pkg.make_problem(batch=wl.batch, heads=wl.heads, head_dim=wl.head_dim, f_q=wl.f_q,
                            f_kv=wl.f_kv, h=wl.h, w=wl.w, dtype=pkg.MRT_F32, scale=wl.scale,
                            q_frame_offset=wl.q_frame_offset)
    lib = pkg.load_library()
    import ctypes
    nmin = lib.monarch_attn_bwd_workspace_min_bytes(ctypes.byref(prob), wl.b1, wl.b2, wl.tile, wl.iters)
    assert 0 < nmin < lib.monarch_attn_bwd_workspace_bytes(ctypes.byref(prob), wl.b1, wl.b2, wl.tile, wl.iters)
    ws = torch.empty(nmin, dtype=torch.uint8, device="cuda:0")
    g1 = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, workspace=ws, **kw)
    g2 = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, **kw)
    torch.cuda.synchronize()
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)


@pytest.mark.parametrize("name", ["bf16-storage", "bf16-ragged-T3", "bf16-stream-mask", "bf16-b2-80"])
def test_backward_rerun_is_bit_identical(name):
    """No kernel of the sweep uses atomics: every gradient entry has one owner, so two calls on the
    same inputs give the same bits (resident and streamed stage L kernels, regular and tiled)."""
    wl = CASES[name]
    arrays = syn.make_inputs(wl)
    rng = np.random.default_rng(7)
    dO = syn.round_to_bf16(rng.standard_normal(arrays[0].shape).astype(np.float32))
    Qd, Kd, Vd, dOd = to_device(wl, arrays + (dO,))
    kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=wl.tile,
              iters=wl.iters, causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset,
              scale=wl.scale)
    g1 = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, **kw)
    g2 = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, **kw)
    torch.cuda.synchronize()
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)


@pytest.mark.parametrize("name", ["bf16-stream-mask", "tiled-rect-mask", "bf16-ragged-T3"])
def test_backward_head_groups_do_not_change_the_result(name):
    """Concurrent head groups on helper streams against one group on the caller's stream: every
    group owns its heads' slices of the workspace and of the gradients, so the bits are the same."""
    wl = dataclasses.replace(CASES[name], heads=5)
    arrays = syn.make_inputs(wl)
    rng = np.random.default_rng(11)
    dO = rng.standard_normal(arrays[0].shape).astype(np.float32)
    if wl.dtype == "bf16":
        dO = syn.round_to_bf16(dO)
    Qd, Kd, Vd, dOd = to_device(wl, arrays + (dO,))
    kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=wl.tile,
              iters=wl.iters, causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset,
              scale=wl.scale)
    try:
        pkg.binding.set_head_groups(1)
        g1 = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, **kw)
        torch.cuda.synchronize()
        for n in (2, 3, 4):
            pkg.binding.set_head_groups(n)
            gn = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, **kw)
            torch.cuda.synchronize()
            for a, b in zip(g1, gn):
                assert torch.equal(a, b), f"{n} groups differ"
    finally:
        pkg.binding.set_head_groups(0)


def leaves_row_statistics(wl):
    """The saving forward call's last stage L runs the streamed kernel on a bf16 workspace (more than
    192 key rows per query tile, or more than eight query tiles of 16 rows and more than 96 key rows):
    it then also leaves every row's log-sum-exp and the unrounded output, and the backward call reads
    its key range once at t = T instead of twice."""
    if not (wl.dtype == "bf16" and wl.head_dim in (64, 128) and wl.b1 <= 144 and wl.b2 <= 96):
        return False
    rows_per_frame = wl.h if wl.assign == "fh_w" else None
    if rows_per_frame is None:
        return False
    nk = wl.f_kv * wl.h * (wl.w // wl.b2) if wl.tile else wl.b1     # key rows of one (m, j) problem
    nlt = (wl.b1 + 15) // 16
    return nk > 96 and not (nk <= 192 and nlt <= 8)


@pytest.mark.parametrize("name", ["bf16-stream-mask", "bf16-ragged-T3", "bf16-ragged-T1", "tiled-rect-mask",
                                  "bf16-b1-135", "regular-T2", "bf16-b2-80", "bf16-stream-T3",
                                  "bf16-stream-short-visible-T2", "bf16-720p-block"])
def test_forward_that_saves_and_backward_from_saved_intermediates(name):
    """The training-step pair: monarch_attn_fwd_save gives the forward output (bit for bit where the
    bf16 forward kernels run it, to the forward tolerance where the fp32 ones do) and leaves the
    intermediates in a workspace filled with NaNs beforehand; monarch_attn_bwd_saved then returns the
    very bits monarch_attn_bwd returns, twice in a row (a second dO reuses the saved intermediates),
    whatever number of head groups either call runs.  Where the forward call leaves its row
    statistics the backward call takes them instead of forming its own: the gradients then agree
    with monarch_attn_bwd's to rounding and meet the oracle's bar themselves."""
    wl = dataclasses.replace(CASES[name], heads=3) if CASES[name].heads < 3 else CASES[name]
    arrays = syn.make_inputs(wl)
    rng = np.random.default_rng(5)
    dOs = [rng.standard_normal(arrays[0].shape).astype(np.float32) for _ in range(2)]
    if wl.dtype == "bf16":
        dOs = [syn.round_to_bf16(x) for x in dOs]
    Qd, Kd, Vd, dO1, dO2 = to_device(wl, arrays + tuple(dOs))
    kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=wl.tile,
              iters=wl.iters, causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset,
              scale=wl.scale, assign=wl.assign, tile_h=wl.tile_h)
    import ctypes
    lib = pkg.load_library()
    prob = pkg.binding._torch_problem(Qd, Kd, Vd, dO1, wl.f_q, wl.f_kv, wl.h, wl.w, wl.q_frame_offset, wl.scale,
                                      pkg.MRT_COMPUTE_DEFAULT, wl.assign, wl.tile_h)
    nbytes = lib.monarch_attn_bwd_saved_workspace_bytes(ctypes.byref(prob), wl.b1, wl.b2, wl.tile, wl.iters)
    assert nbytes > 0
    ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda:0").view(torch.uint8)
    try:
        pkg.binding.set_head_groups(2)               # heads 0 | 1, 2
        O, ws = pkg.monarch_attn_fwd_save(Qd, Kd, Vd, workspace=ws, **kw)
        pkg.binding.set_head_groups(0)
        O_ref = pkg.monarch_attn_fwd(Qd, Kd, Vd, **kw)
        torch.cuda.synchronize()
        assert torch.isfinite(O.float()).all()
        every_stage_bf16 = wl.dtype == "bf16" and wl.head_dim in (64, 128) and wl.b1 <= 144 and wl.b2 <= 96
        if every_stage_bf16 or wl.dtype != "bf16":
            assert torch.equal(O, O_ref)                 # the same kernels ran
        else:
            assert (O.float() - O_ref.float()).abs().max().item() <= 2e-2
        stats = leaves_row_statistics(wl)
        for groups, dOd, dOh in ((3, dO1, dOs[0]), (1, dO2, dOs[1])):
            pkg.binding.set_head_groups(groups)      # heads 0 | 1 | 2, then all on the caller's stream
            got = pkg.monarch_attn_bwd_saved(Qd, Kd, Vd, dOd, ws, **kw)
            pkg.binding.set_head_groups(0)
            want = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, **kw)
            torch.cuda.synchronize()
            for name_g, a, b in zip("QKV", got, want):
                assert torch.isfinite(a).all(), f"non-finite d{name_g}"
                if not stats:
                    assert torch.equal(a, b), f"d{name_g} differs from monarch_attn_bwd"
                else:
                    diff = (a - b).abs().max().item()
                    print(f"  d{name_g}: max |saved - recomputed| {diff:.3e} of max |grad| {b.abs().max().item():.3e}",
                          flush=True)
                    # (both carry the bf16 rounding of the sweep's operands, which a last-bit change of a
                    # row statistic re-draws: measured up to 5.6e-3 over 270 random shapes)
                    assert diff <= 1e-2 * b.abs().max().item(), (name_g, diff)
            if stats:
                hd = wl.heads - 1
                ref = mo.monarch_attn_grad(*(torch.from_numpy(x[0, hd]) for x in arrays),
                                           torch.from_numpy(dOh[0, hd]), **kw)
                for name_g, a, r in zip("QKV", got, ref):
                    err = (a[0, hd].double().cpu() - r).abs().max().item()
                    print(f"  d{name_g} against the oracle: {err:.3e} of {r.abs().max().item():.3e}", flush=True)
                    assert err <= 2e-2 * r.abs().max().item(), (name_g, err)
    finally:
        pkg.binding.set_head_groups(0)


@pytest.mark.parametrize("name", ["bf16-b1-120", "bf16-b1-135", "bf16-stream-mask", "bf16-ragged-T3",
                                  "tiled-rect-mask", "regular-T3", "bf16-stream-short-visible-T2", "bf16-b2-80",
                                  "bf16-b2-96"])
def test_backward_reads_nothing_it_has_not_written(name):
    """A workspace full of NaN bit patterns (what a recycled allocation may hold) gives the same bits
    as a zeroed one: every workspace entry a kernel reads was written earlier in the same call,
    padding rows and tiles included."""
    wl = CASES[name]
    arrays = syn.make_inputs(wl)
    rng = np.random.default_rng(5)
    dO = rng.standard_normal(arrays[0].shape).astype(np.float32)
    if wl.dtype == "bf16":
        dO = syn.round_to_bf16(dO)
    Qd, Kd, Vd, dOd = to_device(wl, arrays + (dO,))
    kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2, tile=wl.tile,
              iters=wl.iters, causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset,
              scale=wl.scale, assign=wl.assign, tile_h=wl.tile_h)
    prob = pkg.make_problem(batch=wl.batch, heads=wl.heads, head_dim=wl.head_dim, f_q=wl.f_q, f_kv=wl.f_kv,
                            h=wl.h, w=wl.w, dtype=pkg.MRT_F32 if wl.dtype == "f32" else pkg.MRT_BF16,
                            scale=wl.scale, q_frame_offset=wl.q_frame_offset)
    import ctypes
    n = pkg.load_library().monarch_attn_bwd_workspace_bytes(ctypes.byref(prob), wl.b1, wl.b2, wl.tile, wl.iters)
    assert n > 0
    clean = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    dirty = torch.full((n,), 0xFF, dtype=torch.uint8, device="cuda:0")
    g0 = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, workspace=clean, **kw)
    g1 = pkg.monarch_attn_bwd(Qd, Kd, Vd, dOd, workspace=dirty, **kw)
    torch.cuda.synchronize()
    for nm, a, b in zip("QKV", g0, g1):
        assert torch.isfinite(b).all(), f"d{nm} picked up workspace garbage"
        assert torch.equal(a, b), f"d{nm} depends on the workspace's previous contents"
