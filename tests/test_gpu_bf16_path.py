"""GPU parity of the bf16 MFMA path against the fp64 oracle, through the C ABI.

Bar: max-abs <= 2e-2 on bf16 inputs with fp32 accumulation, asserted as such for every case.
One stress case lies outside it and says so (OUTSIDE_STATED_BAR): sharp softmaxes with outputs of
magnitude 3.5, where bf16 rounding (2^-9 relative per rounding of P, alpha_L, Y, alpha_R and O,
compounding over the iterations and amplified by the softmaxes) alone exceeds 2e-2; it is held to
the error a CPU emulation of those rounding points shows, and the fp32 arithmetic mode meets the
plain bar on it (test_f32_compute_on_bf16_storage_matches_oracle_tighter).  Because the named
workloads produce outputs of magnitude ~0.05 (their softmaxes average many N(0,1) values), the
tests also require the error to stay below a fraction of the oracle's largest output, so a wrong
result cannot hide under the absolute bar.
"""
import numpy as np
import pytest
import torch

import paper_2602_12271_amd as pkg
from workloads import synthetic as syn

from gpu_harness import (compare_heads, oracle_dense_head, run_dense_gpu, run_monarch_gpu, to_device)

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
REL_BF16 = 4e-2        # of max |O_oracle|


def small_bf16(**kw):
    base = dict(name="small", batch=1, heads=2, head_dim=128, dtype="bf16", rope=False,
                scale=128 ** -0.5, sigma_qk=1.0, sigma_v=1.0)
    base.update(kw)
    return syn.Workload(**base)


SMALL = {
    # one 16-tile per block, single chunk
    "reg-16x16": small_bf16(f_q=1, f_kv=1, h=16, w=16, b1=16, b2=16, tile=0, iters=1,
                            causal_chunk=0, q_frame_offset=0),
    # ragged tiles on both sides, three iterations
    "reg-ragged": small_bf16(batch=2, heads=3, f_q=2, f_kv=2, h=11, w=21, b1=22, b2=21, tile=0,
                             iters=3, causal_chunk=0, q_frame_offset=0),
    # head_dim 64
    "reg-d64": small_bf16(head_dim=64, scale=0.125, f_q=2, f_kv=2, h=9, w=37, b1=18, b2=37,
                          tile=0, iters=2, causal_chunk=0, q_frame_offset=0),
    # tiled, rectangular, chunk-causal with hidden chunks; nk range spans several 64-key chunks
    "tiled-rect-mask": small_bf16(f_q=2, f_kv=8, h=10, w=28, b1=20, b2=14, tile=1, iters=2,
                                  causal_chunk=2, q_frame_offset=4),
    # sharper logits (sigma ~ 3): near one-hot softmaxes, outputs of magnitude ~1
    "tiled-sharp": small_bf16(f_q=2, f_kv=4, h=8, w=24, b1=16, b2=12, tile=1, iters=3,
                              causal_chunk=0, q_frame_offset=0, sigma_qk=1.7),
    # b2 = 1 and b1 = 1 degenerate blocks
    "tiled-b2-1": small_bf16(f_q=2, f_kv=2, h=5, w=3, b1=5, b2=1, tile=1, iters=2,
                             causal_chunk=0, q_frame_offset=0),
    "tiled-b1-1": small_bf16(f_q=3, f_kv=3, h=1, w=40, b1=1, b2=20, tile=1, iters=2,
                             causal_chunk=0, q_frame_offset=0),
    # block-causal self-attention over a whole 6-frame sequence (2-frame chunks): every query tile
    # row sees a different prefix of key tiles, and stage R runs several query tiles per workgroup
    "tiled-self-causal": small_bf16(heads=3, f_q=6, f_kv=6, h=10, w=28, b1=10, b2=14, tile=1, iters=2,
                                    causal_chunk=2, q_frame_offset=0),
    # largest block sizes of this build
    "max-blocks": small_bf16(heads=1, f_q=2, f_kv=2, h=96, w=96, b1=192, b2=96, tile=0, iters=2,
                             causal_chunk=0, q_frame_offset=0),
}


# Cases outside the stated 2e-2 bar, with the bar they are held to instead (max-abs).
OUTSIDE_STATED_BAR = {"tiled-sharp": 6e-2}


def check(wl, arrays, O, heads=None, oracle=None, label="", bar=TOL_BF16):
    kw = {} if oracle is None else {"oracle": oracle}
    err, omax = compare_heads(wl, arrays, O, heads=heads, **kw)
    print(f"  {label}: max|gpu-oracle| = {err:.3e}, max|O| = {omax:.3e}, ratio {err / omax:.3e}",
          flush=True)
    assert err <= bar
    assert err <= REL_BF16 * omax + 1e-3
    return err, omax


@pytest.mark.parametrize("name", list(SMALL))
def test_monarch_bf16_small(name):
    wl = SMALL[name]
    arrays = syn.make_inputs(wl)
    print(f"case {name}", flush=True)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    check(wl, arrays, O, label=name, bar=OUTSIDE_STATED_BAR.get(name, TOL_BF16))


@pytest.mark.parametrize("name", ["reg-ragged", "tiled-rect-mask", "tiled-sharp", "reg-d64"])
def test_dense_bf16_small(name):
    wl = SMALL[name]
    arrays = syn.make_inputs(wl)
    O = run_dense_gpu(wl, *to_device(wl, arrays))
    check(wl, arrays, O, oracle=oracle_dense_head, label="dense " + name)


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_monarch_bf16_named_configs_full(name):
    """Full named configurations, every head, every output element, in the launch
    configuration the benchmark times (default workspace)."""
    wl = syn.WORKLOADS[name]
    arrays = syn.make_inputs(wl)
    print(f"config {name}", flush=True)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    check(wl, arrays, O, label=name)


def test_monarch_bf16_c3_hidden_chunks():
    # the named KV-cache configuration has every chunk visible; move the query chunk back so
    # that 3 of 7 chunks are hidden and the mask path is exercised at full size
    wl = syn.variant("C3", q_frame_offset=9)
    arrays = syn.make_inputs(wl)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    check(wl, arrays, O, heads=[0, 5, 11], label="C3 offset 9")


def c4_heads():
    """First, last and two seeded heads of the 40."""
    mid = np.random.default_rng(40).choice(np.arange(1, 39), size=2, replace=False)
    return [0, 39] + sorted(int(x) for x in mid)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("offset", [18, 9])
def test_monarch_bf16_c4_sampled_heads(offset):
    """The 720p KV-cache step: 40 heads on the GPU in the launch configuration the benchmark times,
    four of them through the oracle.  offset 18: the last query chunk, every key chunk visible (the
    timed workload).  offset 9: the query chunk moved back so that 3 of the 7 key chunks are hidden
    and the streamed stage L kernels at b1 = 135 see a visible prefix of the key tiles (block-causal
    decoding, Sec. 5)."""
    wl = syn.variant("C4", q_frame_offset=offset)
    arrays = syn.make_inputs(wl)
    heads = c4_heads()
    print(f"config C4, q_frame_offset={offset} (40 heads on the GPU, heads {heads} through the oracle)", flush=True)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    assert torch.isfinite(O.float()).all()
    check(wl, arrays, O, heads=heads, label=f"C4 offset {offset}")


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["C3", "C4"])
def test_properties_that_hold_at_any_size(name):
    """Every head of the large configurations, without the oracle: the factored matrix is
    row-stochastic and independent of V, so (i) a constant V comes back unchanged (up to the
    rounding of the probabilities) and (ii) the output is linear in V."""
    wl = syn.WORKLOADS[name]
    Qd, Kd, Vd = to_device(wl, syn.make_inputs(wl))
    const = torch.full_like(Vd, 0.75)
    Oc = run_monarch_gpu(wl, Qd, Kd, const).float()
    assert torch.isfinite(Oc).all()
    dev = (Oc - 0.75).abs().max().item()
    print(f"  {name}: constant V deviates by {dev:.3e}", flush=True)
    assert dev <= 1e-2
    # linearity in V: negating V negates O up to the rounding of the matrix unit's accumulation
    # (which is not exactly symmetric in sign), and scaling V by a power of two scales every
    # product and every rounding boundary alike, so O scales exactly
    O1 = run_monarch_gpu(wl, Qd, Kd, Vd).float()
    O2 = run_monarch_gpu(wl, Qd, Kd, -Vd).float()
    omax = O1.abs().max().item()
    sym = (O1 + O2).abs().max().item()
    print(f"  {name}: max |O(V) + O(-V)| = {sym:.3e} at max |O| = {omax:.3e}", flush=True)
    assert sym <= 2.0 ** -7 * omax
    O4 = run_monarch_gpu(wl, Qd, Kd, 4 * Vd).float()
    assert torch.equal(4 * O1, O4)


@pytest.mark.parametrize("name", ["C1", "C3"])
def test_dense_bf16_named_configs_sampled(name):
    wl = syn.WORKLOADS[name]
    arrays = syn.make_inputs(wl)
    O = run_dense_gpu(wl, *to_device(wl, arrays))
    check(wl, arrays, O, heads=[0, wl.heads - 1], oracle=oracle_dense_head, label="dense " + name)


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_separable_inputs_monarch_equals_dense(name):
    """Position-only inputs (a constant vector under 3-D rotary encoding) have logits that split
    into a (frame,height) term plus a width term, which the aligned structure represents exactly
    (Sec. 4.1): the MonarchRT kernels and the dense kernel must agree, and both match the dense
    oracle."""
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


def test_f32_compute_on_bf16_storage_matches_oracle_tighter():
    # device-side cross-check mode: fp32 arithmetic on bf16 inputs; only the final store rounds
    wl = SMALL["tiled-sharp"]
    arrays = syn.make_inputs(wl)
    O = run_monarch_gpu(wl, *to_device(wl, arrays), compute=pkg.MRT_COMPUTE_F32)
    err, omax = compare_heads(wl, arrays, O)
    print(f"  fp32 compute on bf16 storage: err {err:.3e} max|O| {omax:.3e}", flush=True)
    assert err <= omax * 2 ** -8 + 1e-5


def test_rows_far_below_their_tile_maximum_keep_their_weights():
    """The one-pass stage L kernel first sums 2^(z - reference) with one reference per 16-row query
    tile; a row whose logits all lie more than 126 (base 2) below the tile's largest logit loses
    that sum to underflow and the kernel has to redo the statistics with the row's own maximum.
    All keys equal, one query row of the opposite sign: that row's logits are 200 below the others',
    every softmax is uniform, so O must be the mean of V for every query (and the oracle agrees)."""
    wl = small_bf16(heads=1, f_q=2, f_kv=2, h=16, w=16, b1=32, b2=16, tile=0, iters=3,
                    causal_chunk=0, q_frame_offset=0)
    rng = np.random.default_rng(5)
    n, d = wl.n_q, wl.head_dim
    Q = np.full((1, 1, n, d), 2.5, np.float32)
    rows = np.arange(n) // wl.w                      # block-grid row (frame, height) of each token
    Q[0, 0, rows == 3] = -2.5
    K = np.full((1, 1, n, d), 2.5, np.float32)
    V = syn.round_to_bf16(rng.standard_normal((1, 1, n, d)).astype(np.float32))
    # logits: scale log2(e) q.k = +-102 in base 2
    assert 2 * wl.scale * 1.4427 * 2.5 * 2.5 * d > 126
    O = run_monarch_gpu(wl, *to_device(wl, (Q, K, V)))
    assert torch.isfinite(O.float()).all()
    mean = V[0, 0].astype(np.float64).mean(axis=0)
    assert np.abs(O[0, 0].float().cpu().numpy() - mean[None, :]).max() <= 2e-2
    check(wl, (Q, K, V), O, label="row 200 below its tile's maximum")


@pytest.mark.parametrize("shape", ["regular-one-pass", "tiled-streamed"])
def test_key_rows_far_below_every_query_keep_a_finite_average(shape):
    """alpha_R / c_R is an average of query rows weighted by L[l, nk]; a key row whose logits lie more
    than 126 (base 2) below every query's largest logit has all its weights underflow in fp32, and the
    kernels must then form the same ratio from log L relative to the column's maximum instead of
    dividing 0 by 0.  One key row of the opposite sign against otherwise equal keys and queries:
    its logits are 204 below the others', V is random, and the oracle (fp64 does not underflow at
    2^-204) gives the reference."""
    if shape == "regular-one-pass":
        wl = small_bf16(heads=1, f_q=2, f_kv=2, h=16, w=16, b1=32, b2=16, tile=0, iters=3,
                        causal_chunk=0, q_frame_offset=0)
    else:   # 4 key tiles of 64 rows: the streamed two-pass refine kernel
        wl = small_bf16(heads=1, f_q=1, f_kv=4, h=64, w=16, b1=64, b2=16, tile=1, iters=3,
                        causal_chunk=0, q_frame_offset=0)
    rng = np.random.default_rng(6)
    d = wl.head_dim
    Q = np.full((1, 1, wl.n_q, d), 2.5, np.float32)
    K = np.full((1, 1, wl.n_kv, d), 2.5, np.float32)
    krow = np.arange(wl.n_kv) // wl.w
    K[0, 0, krow == 5] = -2.5
    V = syn.round_to_bf16(rng.standard_normal((1, 1, wl.n_kv, d)).astype(np.float32))
    assert 2 * wl.scale * 1.4427 * 2.5 * 2.5 * d > 126
    O = run_monarch_gpu(wl, *to_device(wl, (Q, K, V)))
    assert torch.isfinite(O.float()).all()
    check(wl, (Q, K, V), O, label=f"key row 204 below the others ({shape})")


def test_rerun_is_bit_identical():
    wl = syn.variant("C2", heads=2)
    dev = to_device(wl, syn.make_inputs(wl))
    O1 = run_monarch_gpu(wl, *dev)
    O2 = run_monarch_gpu(wl, *dev)
    assert torch.equal(O1, O2)


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_tokens_major_layout_gives_the_same_bits(name):
    # [batch, tokens, heads, d] memory (what a fused QKV projection leaves behind) viewed as
    # [batch, heads, tokens, d]: only the element strides change
    wl = syn.variant(name, heads=3)
    Qd, Kd, Vd = to_device(wl, syn.make_inputs(wl))
    Oc = run_monarch_gpu(wl, Qd, Kd, Vd)
    Dc = run_dense_gpu(wl, Qd, Kd, Vd)
    Qs, Ks, Vs = (x.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for x in (Qd, Kd, Vd))
    assert not Qs.is_contiguous() and Qs.stride(2) == 3 * wl.head_dim
    out = torch.empty_like(Qs)
    O = pkg.monarch_attn_fwd(Qs, Ks, Vs, f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, b1=wl.b1, b2=wl.b2,
                             tile=wl.tile, iters=wl.iters, causal_chunk=wl.causal_chunk,
                             q_frame_offset=wl.q_frame_offset, scale=wl.scale, out=out)
    D = pkg.dense_attn_fwd(Qs, Ks, Vs, f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w,
                           causal_chunk=wl.causal_chunk, q_frame_offset=wl.q_frame_offset, scale=wl.scale,
                           out=torch.empty_like(Qs))
    torch.cuda.synchronize()
    assert O.stride() == Qs.stride()
    assert torch.equal(O, Oc) and torch.equal(D, Dc)


def test_head_groups_do_not_change_the_result():
    # concurrent head groups on helper streams vs one group on the caller's stream: bit identical
    wl = syn.variant("C2", heads=5)
    dev = to_device(wl, syn.make_inputs(wl))
    try:
        pkg.binding.set_head_groups(1)
        O1 = run_monarch_gpu(wl, *dev)
        for n in (2, 3, 4):
            pkg.binding.set_head_groups(n)
            assert torch.equal(run_monarch_gpu(wl, *dev), O1), f"{n} groups differ"
    finally:
        pkg.binding.set_head_groups(0)


def test_hip_graph_replays_match_eager():
    # the whole call (fork to helper streams, 2T kernels per head group, join) captured once and
    # replayed several times with eager work in between
    wl = syn.variant("C1", heads=6)
    arrays = syn.make_inputs(wl)
    Qd, Kd, Vd = to_device(wl, arrays)
    eager = run_monarch_gpu(wl, Qd, Kd, Vd).clone()
    prob_ws = pkg.monarch_attn_workspace_bytes(
        pkg.make_problem(batch=1, heads=wl.heads, head_dim=wl.head_dim, f_q=wl.f_q, f_kv=wl.f_kv,
                         h=wl.h, w=wl.w, scale=wl.scale), wl.b1, wl.b2, wl.tile, wl.iters)
    ws = torch.empty(prob_ws, dtype=torch.uint8, device="cuda:0")
    out = torch.empty_like(Qd)
    run = lambda: pkg.monarch_attn_fwd(Qd, Kd, Vd, f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w,
                                       b1=wl.b1, b2=wl.b2, tile=wl.tile, iters=wl.iters,
                                       scale=wl.scale, out=out, workspace=ws)
    pkg.binding.set_head_groups(3)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                   # warm-up outside capture (creates helper streams)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(4):
        out.zero_()
        ws.random_(0, 255)                      # eager work between replays; the workspace is scratch
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager result"
    pkg.binding.set_head_groups(0)


def test_mini_sequence_passes_match_single_pass_and_oracle():
    # full bidirectional sequence (f_q = f_kv = 6) with 2-frame tiles: three query tile rows.  With
    # the minimum workspace the library finishes one query tile row at a time (Sec. 4.3,
    # mini-sequence); the result must equal the single-pass result bit for bit.
    wl = small_bf16(heads=2, f_q=6, f_kv=6, h=8, w=28, b1=16, b2=14, tile=1, iters=2,
                    causal_chunk=0, q_frame_offset=0)
    arrays = syn.make_inputs(wl)
    dev = to_device(wl, arrays)
    prob = pkg.make_problem(batch=1, heads=wl.heads, head_dim=wl.head_dim, f_q=wl.f_q, f_kv=wl.f_kv,
                            h=wl.h, w=wl.w, scale=wl.scale)
    nmin = pkg.monarch_attn_workspace_bytes(prob, wl.b1, wl.b2, wl.tile, wl.iters, minimum=True)
    nall = pkg.monarch_attn_workspace_bytes(prob, wl.b1, wl.b2, wl.tile, wl.iters)
    assert nall == nmin * 3 * wl.heads
    O_full = run_monarch_gpu(wl, *dev)
    for units in (1, 2, 3, 4):                  # 1-2 rows per pass, one head, one head + change
        ws = torch.empty(nmin * units, dtype=torch.uint8, device="cuda:0")
        assert torch.equal(run_monarch_gpu(wl, *dev, workspace=ws), O_full), f"{units} slabs"
    check(wl, arrays, O_full, label="bidirectional 6 frames")


def test_bidirectional_480p_one_frame_tiles():
    # the paper's s = 0.95 point for the 81-frame video: every frame its own tile row, tile blocks
    # (h, w) = (30, 52), full 32760 x 32760 attention; one head through the oracle
    wl = syn.variant("C3", heads=2, f_q=21, f_kv=21, b1=30, b2=52, iters=1, causal_chunk=0,
                     q_frame_offset=0)
    arrays = syn.make_inputs(wl)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    check(wl, arrays, O, heads=[1], label="480p bidirectional (30,52) T=1")


@pytest.mark.parametrize("name", ["reg-ragged", "reg-d64", "tiled-rect-mask", "tiled-b2-1", "tiled-self-causal",
                                  "max-blocks"])
def test_forward_reads_nothing_it_has_not_written(name):
    """A workspace full of NaN bit patterns (what a recycled allocation may hold) gives the same bits
    as a zeroed one: every intermediate a kernel reads was written earlier in the same call."""
    wl = SMALL[name]
    dev = to_device(wl, syn.make_inputs(wl))
    prob = pkg.make_problem(batch=wl.batch, heads=wl.heads, head_dim=wl.head_dim, f_q=wl.f_q, f_kv=wl.f_kv,
                            h=wl.h, w=wl.w, scale=wl.scale, q_frame_offset=wl.q_frame_offset)
    n = pkg.monarch_attn_workspace_bytes(prob, wl.b1, wl.b2, wl.tile, wl.iters)
    clean = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    dirty = torch.full((n,), 0xFF, dtype=torch.uint8, device="cuda:0")
    O0 = run_monarch_gpu(wl, *dev, workspace=clean)
    O1 = run_monarch_gpu(wl, *dev, workspace=dirty)
    assert torch.isfinite(O1.float()).all()
    assert torch.equal(O0, O1)
