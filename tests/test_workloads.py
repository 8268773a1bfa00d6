"""CPU checks of the seeded input generators and of the workload table."""
import numpy as np
import torch

from oracle import monarch_oracle as mo
from workloads import synthetic as syn


def test_named_workload_shapes():
    w = syn.WORKLOADS
    assert (w["C0"].n_q, w["C0"].head_dim, w["C0"].dtype, w["C0"].iters) == (576, 64, "f32", 1)
    assert (w["C1"].n_q, w["C1"].n_kv, w["C1"].heads, w["C1"].ntq, w["C1"].ntk) == (4680, 4680, 12, 1, 1)
    assert (w["C2"].ntq, w["C2"].ntk, w["C2"].b1, w["C2"].b2) == (2, 2, 90, 26)
    assert (w["C3"].n_q, w["C3"].n_kv, w["C3"].ntq, w["C3"].ntk) == (4680, 32760, 2, 14)
    assert (w["C4"].n_q, w["C4"].n_kv, w["C4"].heads, w["C4"].iters) == (10800, 75600, 40, 3)
    assert w["C3"].causal_chunk == 3 and w["C3"].q_frame_offset == 18


def test_bf16_rounding_is_nearest_even_and_matches_torch():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(100000).astype(np.float32) * 3
    x[:4] = [1.0, 1.00390625, 1.01171875, -1.00390625]     # exact ties between bf16 neighbours
    got = syn.round_to_bf16(x)
    want = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    assert np.array_equal(got, want)
    assert got[1] == 1.0 and got[2] == np.float32(1.015625) and got[3] == -1.0
    bits = syn.bf16_bits(got)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(back, got)


def test_heads_are_independent_and_reproducible():
    wl = syn.variant("C2", heads=3, f_q=1, f_kv=1, h=6, w=26, b1=6, b2=13)
    Q, K, V = syn.make_inputs(wl)
    q1, k1, v1 = syn.make_head(wl, 0, 1)
    assert np.array_equal(Q[0, 1], q1) and np.array_equal(K[0, 1], k1) and np.array_equal(V[0, 1], v1)
    assert not np.array_equal(Q[0, 0], Q[0, 1])
    assert abs(float(V.std()) - 1.0) < 0.05
    # stored values are exactly representable in bf16
    assert np.array_equal(syn.round_to_bf16(Q), Q)


def test_rope_is_a_rotation_and_depends_on_relative_position_only():
    d, h, w = 128, 4, 5
    ang = syn.rope_angles(np.arange(3), h, w, d)
    assert ang.shape == (3 * h * w, d // 2)
    assert syn.rope_pairs_split(d) == (22, 21, 21)
    rng = np.random.default_rng(1)
    x = rng.standard_normal(d).astype(np.float32)
    y = rng.standard_normal(d).astype(np.float32)
    X = syn.apply_rope(np.broadcast_to(x, (3 * h * w, d)).copy(), ang).astype(np.float64)
    Y = syn.apply_rope(np.broadcast_to(y, (3 * h * w, d)).copy(), ang).astype(np.float64)
    assert np.allclose(np.linalg.norm(X, axis=1), np.linalg.norm(x), rtol=1e-5)
    S = X @ Y.T
    tok = lambda f, a, b: (f * h + a) * w + b
    # same displacement (1 frame, 2 rows, 3 columns) from two different origins
    assert np.isclose(S[tok(0, 0, 0), tok(1, 2, 3)], S[tok(1, 1, 1), tok(2, 3, 4)], atol=1e-3)
    # separability: the (frame,height) part and the width part add up
    # S[(r,c),(r',c')] = A[r,r'] + G[c,c']: changing the query column shifts the logit by the
    # same amount whatever the query row, and the same on the key side
    a, b, c, e = tok(0, 1, 0), tok(0, 1, 4), tok(2, 3, 0), tok(2, 3, 4)
    k0, k1 = tok(1, 0, 2), tok(1, 0, 3)
    assert np.isclose(S[a, k0] - S[b, k0], S[c, k0] - S[e, k0], atol=1e-3)
    assert np.isclose(S[a, k0] - S[a, k1], S[c, k0] - S[c, k1], atol=1e-3)


def test_position_only_inputs_make_monarch_equal_dense_in_the_oracle():
    # full-precision version of the GPU test: a small (f,h,w) grid with rotary position-only
    # queries and keys; aligned blocks represent separable logits exactly (Sec. 4.1)
    wl = syn.variant("C3", heads=1, f_q=1, f_kv=3, h=4, w=12, b1=4, b2=6, causal_chunk=1,
                     q_frame_offset=1, dtype="f32")
    Q, K, V = (torch.from_numpy(x).double() for x in syn.make_separable_head(wl, 0, 0))
    kw = dict(f_q=wl.f_q, f_kv=wl.f_kv, h=wl.h, w=wl.w, causal_chunk=wl.causal_chunk,
              q_frame_offset=wl.q_frame_offset, scale=wl.scale)
    for T in (1, 2):
        O = mo.monarch_attn(Q, K, V, b1=wl.b1, b2=wl.b2, tile=1, iters=T, **kw)
        D = mo.dense_attn(Q, K, V, **kw)
        assert torch.allclose(O, D, atol=1e-6)     # inputs were built in fp32
    # ... and ordinary random inputs do not
    Q, K, V = (torch.from_numpy(x).double() for x in syn.make_head(wl, 0, 0))
    O = mo.monarch_attn(Q, K, V, b1=wl.b1, b2=wl.b2, tile=1, iters=2, **kw)
    assert (O - mo.dense_attn(Q, K, V, **kw)).abs().max() > 1e-3
