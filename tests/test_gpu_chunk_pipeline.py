"""GPU parity cases aimed at the streamed kernels' chunk pipeline (ring of four 32-key LDS slots, two or
four register sets in flight, chunks consumed in pairs) and at its online softmax, which takes the
exponentials against a lazily raised reference instead of the running maximum.

* The in-library dense baseline runs the same pipeline on logits we control directly
  (softmax(scale Q K^T) V, Sec. 2.2): key logits that rise steadily (the reference is raised many times),
  fall steadily (raised once), zig-zag, or hold one spike far above everything else.  Key counts are
  chosen so that the number of 32-key chunks is odd and even, below and above the ring's four slots.
* MonarchRT shapes whose stage L key range sits just above the one-pass kernels' limit (192 rows), with
  a single query tile (three of the four waves own no tile), with 9 to 12 query tiles (eight-wave
  workgroups, four register sets, head_dim 64: fewer 16-byte pieces per chunk than threads), and with
  an odd and an even number of chunk pairs.  T = 2, so the streamed refine kernel (pass 2 one pair of
  query tiles at a time) and the streamed last-iteration kernel both run.

Everything is compared element by element with the fp64 oracle on the same bf16-rounded inputs.
"""
import numpy as np
import pytest
import torch

from workloads import synthetic as syn

from gpu_harness import compare_heads, oracle_dense_head, run_dense_gpu, run_monarch_gpu, to_device

pytestmark = pytest.mark.gpu

TOL_BF16, REL_BF16 = 2e-2, 4e-2


def workload(**kw):
    d = kw["head_dim"]
    base = dict(name="pipe", batch=1, heads=2, dtype="bf16", rope=False, scale=d ** -0.5,
                sigma_qk=1.0, sigma_v=1.0, causal_chunk=0, q_frame_offset=0, tile=0, iters=1, b1=1, b2=1)
    base.update(kw)
    return syn.Workload(**base)


def crafted_dense_inputs(wl, profile, seed):
    """Q and K that give logit(i, k) = amp_i * shape_k plus a little noise, with shape_k in [-1, 1] over the
    keys and amp_i between 30 and 55 natural units (a base-2 range of 90 to 160 per query, so that a rising
    profile raises the reference ten to twenty times); V random.  bf16-rounded, as the GPU sees them."""
    rng = np.random.default_rng(seed)
    d, nq, nk = wl.head_dim, wl.n_q, wl.n_kv
    x = np.linspace(-1.0, 1.0, nk)
    shape = dict(rising=x, falling=-x, zigzag=np.where(np.arange(nk) % 64 < 32, x, -x),
                 spike=np.where(np.arange(nk) == (2 * nk) // 3, 1.0, -1.0 + 0.05 * rng.standard_normal(nk)))[profile]
    Q = np.zeros((1, wl.heads, nq, d), np.float32)
    K = np.zeros((1, wl.heads, nk, d), np.float32)
    amp = rng.uniform(0.5, 1.0, size=(wl.heads, nq))
    # logit = scale * (Q[i, 0] K[k, 0] + Q[i, 1] K[k, 1]) + noise = (576 amp_i + 64) / sqrt(d) * shape_k + noise
    Q[0, :, :, 0] = 24.0 * amp
    K[0, :, :, 0] = 24.0 * shape[None, :]
    Q[0, :, :, 1] = 8.0
    K[0, :, :, 1] = 8.0 * shape[None, :]
    Q[0, :, :, 2:] = 0.1 * rng.standard_normal((wl.heads, nq, d - 2))
    K[0, :, :, 2:] = 0.1 * rng.standard_normal((wl.heads, nk, d - 2))
    V = rng.standard_normal((1, wl.heads, nk, d)).astype(np.float32)
    return tuple(syn.round_to_bf16(a) for a in (Q, K, V))


DENSE_GRIDS = {
    # (f_q, f_kv, h, w): N_q = 77 (five query tiles: waves with two, one and no tile), keys in 32-key chunks
    "3-chunks": (1, 1, 7, 11),      # 77 keys: fewer chunks than ring slots, odd
    "13-chunks": (1, 5, 7, 11),     # 385 keys: odd number of chunks, the last one ragged
    "16-chunks": (2, 8, 4, 16),     # 512 keys: even, no ragged tail; 128 queries
    "25-chunks": (1, 10, 7, 11),    # 770 keys
}


@pytest.mark.parametrize("profile", ["rising", "falling", "zigzag", "spike"])
@pytest.mark.parametrize("grid", list(DENSE_GRIDS))
def test_dense_baseline_with_moving_maxima(grid, profile):
    f_q, f_kv, h, w = DENSE_GRIDS[grid]
    wl = workload(head_dim=128, f_q=f_q, f_kv=f_kv, h=h, w=w, q_frame_offset=f_kv - f_q)
    arrays = crafted_dense_inputs(wl, profile, seed=len(grid) * 7 + len(profile))
    O = run_dense_gpu(wl, *to_device(wl, arrays))
    assert torch.isfinite(O.float()).all()
    err, omax = compare_heads(wl, arrays, O, oracle=oracle_dense_head)
    print(f"  dense {grid} {profile}: max|gpu-oracle| = {err:.3e}, max|O| = {omax:.3e}", flush=True)
    assert err <= TOL_BF16 and err <= REL_BF16 * omax + 1e-3


def test_dense_baseline_chunk_causal_rows_see_different_prefixes():
    # chunk-causal mask: queries of the first chunk see 2 of 6 frames; the per-key chunk comparison hides
    # the rest inside the pipeline (fully hidden chunks leave a query's reference at -inf for a while)
    wl = workload(head_dim=64, f_q=6, f_kv=6, h=5, w=9, causal_chunk=2)
    arrays = syn.make_inputs(wl)
    O = run_dense_gpu(wl, *to_device(wl, arrays))
    err, omax = compare_heads(wl, arrays, O, oracle=oracle_dense_head)
    print(f"  dense chunk-causal: max|gpu-oracle| = {err:.3e}, max|O| = {omax:.3e}", flush=True)
    assert err <= TOL_BF16 and err <= REL_BF16 * omax + 1e-3


STREAMED = {
    # key range NK = c1k * b1 just above the one-pass limit; 8 chunks (even), four waves of one tile
    "nk-240": workload(head_dim=128, f_q=1, f_kv=5, h=48, w=20, b1=48, b2=20, tile=1, iters=2),
    # 11 chunks: odd, the sixth pair ends with an empty chunk; hidden last tile row for the first query rows
    "nk-336-odd": workload(head_dim=128, f_q=2, f_kv=7, h=48, w=17, b1=48, b2=17, tile=1, iters=2,
                           causal_chunk=1, q_frame_offset=5),
    # one query tile: three of the four waves own none and only move data
    "one-tile": workload(head_dim=64, f_q=1, f_kv=13, h=16, w=33, b1=16, b2=33, tile=1, iters=2),
    # 9 query tiles, head_dim 64: eight-wave last-iteration workgroups with more threads than pieces per chunk
    "b1-144-d64": workload(head_dim=64, f_q=1, f_kv=2, h=144, w=16, b1=144, b2=16, tile=1, iters=2),
    # 12 query tiles: 12 chunks = 6 pairs (even) and 18 chunks = 9 pairs (odd: the four-set loop's empty pair)
    "b1-192-even": workload(head_dim=128, f_q=1, f_kv=2, h=192, w=16, b1=192, b2=16, tile=1, iters=2),
    "b1-192-odd": workload(head_dim=128, f_q=1, f_kv=3, h=192, w=15, b1=192, b2=15, tile=1, iters=3),
    # 10 query tiles with a ragged last one, two column tiles
    "b1-150": workload(head_dim=128, f_q=1, f_kv=2, h=150, w=34, b1=150, b2=17, tile=1, iters=2),
}


@pytest.mark.parametrize("name", list(STREAMED))
def test_streamed_stage_l_shapes(name):
    wl = STREAMED[name]
    arrays = syn.make_inputs(wl)
    print(f"case {name}: up to {wl.ntk * wl.b1} key rows per stage L column", flush=True)
    O = run_monarch_gpu(wl, *to_device(wl, arrays))
    assert torch.isfinite(O.float()).all()
    err, omax = compare_heads(wl, arrays, O)
    print(f"  {name}: max|gpu-oracle| = {err:.3e}, max|O| = {omax:.3e}", flush=True)
    assert err <= TOL_BF16 and err <= REL_BF16 * omax + 1e-3
