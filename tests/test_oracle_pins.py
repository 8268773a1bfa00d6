"""Pins for the fp64 oracle: each test checks it against something fixed by the
paper or by mathematics, not against itself.

  P1  degenerate block sizes are dense softmax attention (Sec. 4.1 take-away box;
      Sec. 4.2 example, neighbourhood (1,1,1))
  P2  materialised M from the final factors: M @ V == factored output; M is
      row-stochastic and non-negative (Sec. 4.2 entry formula; row-stochasticity
      stated in Sec. 4.2 "Algorithm")
  P3  separable logits a[l,k] + g[j,i] are represented exactly: output == dense
      attention for every T >= 1 (Sec. 4.1 "An aligned construction"), also
      tiled, rectangular and tile-masked
  P4  tiled with c1 = c2 = 1 is the regular algorithm (Thm 4.1 containment)
  P5  parameter tying reproduces the regular matrix (App. B.2 containment)
  P5' two single-entry tiles give a rank-2 slice (App. B.2 strictness)
  P6  an index-loop transcription of the update equations (App. A.1 / A.2, the
      7-index form) agrees with the einsum form of the pseudocode
  P7  KL(M^(t) || softmax(QK^T)) never increases with t and is >= 0
      (Sec. 2.1 variational objective: the updates are block-coordinate ascent)
  P8  V constant along tokens => O equals it
  plus mutation checks: oracles with a planted mistake FAIL the pins.
"""
import itertools
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import monarch_oracle as mo

F64 = torch.float64


def rnd(shape, seed, sigma=1.0):
    g = torch.Generator().manual_seed(seed)
    return sigma * torch.randn(*shape, generator=g, dtype=F64)


def textbook_dense(Q, K, V, mask=None):
    """softmax(QK^T)V with numpy/scipy only (not the oracle's dense routine)."""
    S = Q.numpy() @ K.numpy().T
    if mask is not None:
        S = np.where(mask.numpy(), S, -np.inf)
    return torch.from_numpy(scipy.special.softmax(S, axis=1) @ V.numpy())


# ------------------------------------------------------------------ P1
@pytest.mark.parametrize("T", [1, 2, 3])
@pytest.mark.parametrize("blocks", ["1xN", "Nx1"])
def test_p1_degenerate_regular_is_dense(T, blocks):
    N, d = 30, 8
    Q, K, V = rnd((N, d), 1), rnd((N, d), 2), rnd((N, d), 3)
    b1, b2 = (1, N) if blocks == "1xN" else (N, 1)
    O = mo.monarch_attention_regular(Q, K, V, T, b1, b2)
    assert torch.allclose(O, textbook_dense(Q, K, V), atol=1e-12, rtol=0)


@pytest.mark.parametrize("T", [1, 2])
def test_p1_tiled_unit_tiles_is_dense(T):
    # tiles of block size (1,1): every token its own tile (Sec. 4.2, (n_f,n_h,n_w)=(1,1,1))
    rows_q, rows_k, w, d = 3, 5, 4, 6
    Q, K, V = rnd((rows_q * w, d), 4), rnd((rows_k * w, d), 5), rnd((rows_k * w, d), 6)
    g = mo.TileGeometry(1, 1, rows_q, rows_k, w)
    O = mo.monarch_attention_tiled(Q, K, V, T, g)
    assert torch.allclose(O, textbook_dense(Q, K, V), atol=1e-12, rtol=0)


def test_dense_routine_matches_textbook_and_mask():
    Q, K, V = rnd((24, 5), 7), rnd((36, 5), 8), rnd((36, 7), 9)
    assert torch.allclose(mo.dense_attention(Q, K, V), textbook_dense(Q, K, V), atol=1e-13)
    mask = mo.token_chunk_causal_mask(f_q=2, f_kv=3, h=3, w=4, causal_chunk=1, q_frame_offset=1)
    # query frames are absolute 1,2; keys 0,1,2
    assert mask.shape == (24, 36)
    assert mask[0].tolist() == [True] * 24 + [False] * 12
    assert mask[12].tolist() == [True] * 36
    assert torch.allclose(mo.dense_attention(Q, K, V, 1.0, mask), textbook_dense(Q, K, V, mask),
                          atol=1e-13)
    # scale is the logits multiplier
    assert torch.allclose(mo.dense_attention(Q, K, V, 0.37), textbook_dense(0.37 * Q, K, V),
                          atol=1e-13)


# ------------------------------------------------------------------ P2
@pytest.mark.parametrize("b1,b2,T", [(3, 4, 1), (6, 4, 2), (12, 12, 3), (24, 24, 1)])
def test_p2_materialised_regular(b1, b2, T):
    N, d = b1 * b2, 8
    Q, K, V = rnd((N, d), 10, 0.8), rnd((N, d), 11, 0.8), rnd((N, d), 12)
    O, L, R = mo.monarch_attention_regular(Q, K, V, T, b1, b2, return_factors=True)
    M = mo.materialise_regular(L, R)
    assert (M >= 0).all()
    assert torch.allclose(M.sum(1), torch.ones(N, dtype=F64), atol=1e-12)
    assert torch.allclose(R.sum(2), torch.ones(b1, b2, dtype=F64), atol=1e-12)
    assert torch.allclose(L.sum(1), torch.ones(b2, b1, dtype=F64), atol=1e-12)
    assert torch.allclose(M @ V, O, atol=1e-12)
    # the entry formula itself, spelt out element by element on a few entries
    for (l, j, k, i) in [(0, 0, 0, 0), (b1 - 1, 1, 1, b2 - 1), (1, b2 - 1, b1 - 1, 2)]:
        assert M[l * b2 + j, k * b2 + i].item() == pytest.approx(
            (L[j, k, l] * R[k, j, i]).item(), abs=1e-15)


@pytest.mark.parametrize("T", [1, 2])
def test_p2_materialised_tiled_rect_masked(T):
    h, w, b1, b2 = 2, 6, 4, 3          # 2 frames per tile row
    f_q, f_kv = 2, 6
    g = mo.geometry_from_grid(f_q, f_kv, h, w, b1, b2, tile=1)
    assert (g.c1q, g.c1k, g.c2) == (1, 3, 2)
    vis = mo.chunk_causal_visibility(g, h, causal_chunk=2, q_frame_offset=2)
    # query chunk 1 sees key chunks 0,1 -> key tile rows 0,1 -> tiles 0..3
    assert vis.tolist() == [[True] * 4 + [False] * 2] * 2
    d = 5
    Q = rnd((f_q * h * w, d), 13)
    K = rnd((f_kv * h * w, d), 14)
    V = rnd((f_kv * h * w, d), 15)
    O, ids, Ls, Rs = mo.monarch_attention_tiled(Q, K, V, T, g, 1.0, vis, return_factors=True)
    M = mo.materialise_tiled(g, ids, Ls, Rs)
    assert (M >= 0).all()
    assert torch.allclose(M.sum(1), torch.ones(M.shape[0], dtype=F64), atol=1e-12)
    assert torch.allclose(M @ V, O, atol=1e-12)
    # hidden keys (frames 4,5) get exactly zero weight
    assert (M[:, 4 * h * w:] == 0).all()
    for m in range(g.ntq):
        assert torch.allclose(Rs[m].sum(3), torch.ones_like(Rs[m].sum(3)), atol=1e-12)
        # joint over (n,k)
        assert torch.allclose(Ls[m].sum((0, 2)), torch.ones(b2, b1, dtype=F64), atol=1e-12)


# ------------------------------------------------------------------ P3
def separable_qk(rows_q, rows_k, w, da, db, seed, sigma=1.0):
    """Q[(r,c)] = [qa_r | qb_c], K[(r,c)] = [ka_r | kb_c]  =>  QK^T = a[r,r'] + g[c,c']."""
    qa, ka = rnd((rows_q, da), seed, sigma), rnd((rows_k, da), seed + 1, sigma)
    qb, kb = rnd((w, db), seed + 2, sigma), rnd((w, db), seed + 3, sigma)
    Q = torch.cat([qa[:, None, :].expand(rows_q, w, da), qb[None].expand(rows_q, w, db)], 2)
    K = torch.cat([ka[:, None, :].expand(rows_k, w, da), kb[None].expand(rows_k, w, db)], 2)
    return Q.reshape(rows_q * w, da + db).contiguous(), K.reshape(rows_k * w, da + db).contiguous()


@pytest.mark.parametrize("T", [1, 2, 4])
def test_p3_separable_regular_exact(T):
    b1, b2 = 6, 5
    Q, K = separable_qk(b1, b1, b2, 3, 4, 20, 1.3)
    V = rnd((b1 * b2, 7), 24)
    O = mo.monarch_attention_regular(Q, K, V, T, b1, b2)
    assert torch.allclose(O, textbook_dense(Q, K, V), atol=1e-12)


@pytest.mark.parametrize("T", [1, 2, 3])
@pytest.mark.parametrize("offset", [0, 2, 4])
def test_p3_separable_tiled_rect_masked_exact(T, offset):
    h, w, b1, b2 = 2, 6, 4, 3
    f_q, f_kv = 2, 6
    g = mo.geometry_from_grid(f_q, f_kv, h, w, b1, b2, tile=1)
    Q, K = separable_qk(f_q * h, f_kv * h, w, 3, 3, 30, 1.1)
    V = rnd((f_kv * h * w, 4), 34)
    O = mo.monarch_attn(Q, K, V, f_q=f_q, f_kv=f_kv, h=h, w=w, b1=b1, b2=b2, tile=1, iters=T,
                        causal_chunk=2, q_frame_offset=offset)
    mask = mo.token_chunk_causal_mask(f_q, f_kv, h, w, 2, offset)
    assert torch.allclose(O, textbook_dense(Q, K, V, mask), atol=1e-12)
    # and unmasked
    O = mo.monarch_attention_tiled(Q, K, V, T, g)
    assert torch.allclose(O, textbook_dense(Q, K, V), atol=1e-12)


def general_separable_qk(ntq, ntk, b1, b2, seed, sigma=1.0):
    """Vectors whose logits are a[m,n,j,l,k] + g[m,n,k,j,i] (the widest family the
    rank-1-per-slice structure represents exactly): one-hot coordinates carry the
    index that lives on the other side.  Tokens are produced in tile order
    [tile, row, col]; the caller un-tiles them."""
    a = rnd((ntq, ntk, b2, b1, b1), seed, sigma)          # m n j l k
    g = rnd((ntq, ntk, b1, b2, b2), seed + 1, sigma)      # m n k j i
    da, db = ntk * b1, ntq * b2
    Q = torch.zeros(ntq, b1, b2, da + db, dtype=F64)      # m l j
    K = torch.zeros(ntk, b1, b2, da + db, dtype=F64)      # n k i
    for m, l, j in itertools.product(range(ntq), range(b1), range(b2)):
        Q[m, l, j, :da] = a[m, :, j, l, :].reshape(-1)
        Q[m, l, j, da + m * b2 + j] = 1.0
    for n, k, i in itertools.product(range(ntk), range(b1), range(b2)):
        K[n, k, i, n * b1 + k] = 1.0
        K[n, k, i, da:] = g[:, n, k, :, i].reshape(-1)
    return Q, K


@pytest.mark.parametrize("T", [1, 2, 3])
def test_p3_general_separable_regular_exact(T):
    b1, b2 = 5, 4
    Qt, Kt = general_separable_qk(1, 1, b1, b2, 35, 1.2)
    Q, K = Qt.reshape(b1 * b2, -1), Kt.reshape(b1 * b2, -1)
    V = rnd((b1 * b2, 6), 37)
    O = mo.monarch_attention_regular(Q, K, V, T, b1, b2)
    assert torch.allclose(O, textbook_dense(Q, K, V), atol=1e-12)


@pytest.mark.parametrize("T", [1, 2, 3])
def test_p3_general_separable_tiled_exact(T):
    g = mo.TileGeometry(3, 2, 1, 2, 2)                    # rectangular: 2 query tiles, 4 key tiles
    Qt, Kt = general_separable_qk(g.ntq, g.ntk, g.b1, g.b2, 38, 1.2)
    Q = mo.from_tiles(Qt, g.c1q, g.b1, g.c2, g.b2)
    K = mo.from_tiles(Kt, g.c1k, g.b1, g.c2, g.b2)
    V = rnd((K.shape[0], 5), 39)
    O = mo.monarch_attention_tiled(Q, K, V, T, g)
    assert torch.allclose(O, textbook_dense(Q, K, V), atol=1e-12)
    # with a tile mask: key tile row 1 hidden == dense attention with those keys masked
    vis = torch.tensor([[True, True, False, False]] * 2)
    O = mo.monarch_attention_tiled(Q, K, V, T, g, 1.0, vis)
    mask = torch.zeros(Q.shape[0], K.shape[0], dtype=torch.bool)
    mask[:, : 2 * g.b1 * g.b2] = True
    assert torch.allclose(O, textbook_dense(Q, K, V, mask), atol=1e-12)


def test_p3_nonseparable_is_not_dense():
    # the approximation is not trivially dense: generic inputs differ from dense
    b1, b2 = 6, 5
    Q, K, V = rnd((30, 8), 40), rnd((30, 8), 41), rnd((30, 8), 42)
    O = mo.monarch_attention_regular(Q, K, V, 2, b1, b2)
    assert (O - textbook_dense(Q, K, V)).abs().max() > 1e-2


# ------------------------------------------------------------------ P4
@pytest.mark.parametrize("T", [1, 3])
def test_p4_single_tile_equals_regular(T):
    b1, b2, d = 5, 4, 6
    Q, K, V = rnd((20, d), 50), rnd((20, d), 51), rnd((20, d), 52)
    g = mo.TileGeometry(b1, b2, 1, 1, 1)
    O_t = mo.monarch_attention_tiled(Q, K, V, T, g, 0.7)
    O_r = mo.monarch_attention_regular(Q, K, V, T, b1, b2, 0.7)
    assert torch.allclose(O_t, O_r, atol=1e-13)


# ------------------------------------------------------------------ P5
def test_p5_parameter_tying_reproduces_regular_matrix():
    bb1, bb2, c1, c2 = 4, 6, 2, 3
    tb1, tb2 = bb1 // c1, bb2 // c2
    L = torch.rand(bb2, bb1, bb1, dtype=F64, generator=torch.Generator().manual_seed(60))  # j k l
    R = torch.rand(bb1, bb2, bb2, dtype=F64, generator=torch.Generator().manual_seed(61))  # k j i
    M_reg = mo.materialise_regular(L, R)
    g = mo.TileGeometry(tb1, tb2, c1, c1, c2)
    ids, Ls, Rs = [], [], []
    for m in range(g.ntq):
        l1, j1 = m // c2, m % c2
        Lm = torch.zeros(g.ntk, tb2, tb1, tb1, dtype=F64)
        Rm = torch.zeros(g.ntk, tb1, tb2, tb2, dtype=F64)
        for n in range(g.ntk):
            k1, i1 = n // c2, n % c2
            for j2, k2, l2 in itertools.product(range(tb2), range(tb1), range(tb1)):
                Lm[n, j2, k2, l2] = L[j1 * tb2 + j2, k1 * tb1 + k2, l1 * tb1 + l2]   # ignores i1
            for k2, j2, i2 in itertools.product(range(tb1), range(tb2), range(tb2)):
                Rm[n, k2, j2, i2] = R[k1 * tb1 + k2, j1 * tb2 + j2, i1 * tb2 + i2]   # ignores l1
        ids.append(torch.arange(g.ntk)); Ls.append(Lm); Rs.append(Rm)
    assert torch.equal(mo.materialise_tiled(g, ids, Ls, Rs), M_reg)


def test_p5_strictness_two_single_entry_tiles_rank2():
    bb1, bb2, c1, c2 = 4, 4, 2, 2
    tb1, tb2 = 2, 2
    g = mo.TileGeometry(tb1, tb2, c1, c1, c2)
    ids = [torch.arange(g.ntk) for _ in range(g.ntq)]
    Ls = [torch.zeros(g.ntk, tb2, tb1, tb1, dtype=F64) for _ in range(g.ntq)]
    Rs = [torch.zeros(g.ntk, tb1, tb2, tb2, dtype=F64) for _ in range(g.ntq)]
    # slice B^(j=0,k=0) of the 4-D view [l, j, k, i]: rows l, cols i.  Put a one at
    # (l,i)=(0,0) [query tile (0,0), key tile (0,0)] and at (2,2) [query tile (1,0), key tile (0,1)].
    Ls[0][0][0, 0, 0] = 1; Rs[0][0][0, 0, 0] = 1
    Ls[2][1][0, 0, 0] = 1; Rs[2][1][0, 0, 0] = 1
    M = mo.materialise_tiled(g, ids, Ls, Rs).reshape(bb1, bb2, bb1, bb2)
    B00 = M[:, 0, 0, :]
    assert B00[0, 0] == 1 and B00[2, 2] == 1 and B00.sum() == 2
    assert torch.linalg.matrix_rank(B00) == 2


# ------------------------------------------------------------------ P6
def loops_regular(Q, K, V, T, b1, b2, scale):
    """App. A.1 equations, one index at a time (numpy, python loops)."""
    d = Q.shape[1]
    Qv, Kv, Vv = (x.numpy().reshape(b1, b2, -1) for x in (Q, K, V))
    L = np.zeros((b2, b1, b1))                 # text storage: L[j, l, k]
    for j in range(b2):
        L[j] = np.eye(b1)
    R = np.zeros((b1, b2, b2))                 # R[k, j, i]
    for _ in range(T):
        for k in range(b1):
            for j in range(b2):
                a = sum(L[j, l, k] * Qv[l, j] for l in range(b1))
                c = sum(L[j, l, k] for l in range(b1))
                z = np.array([scale * np.dot(a, Kv[k, i]) / c for i in range(b2)])
                e = np.exp(z - z.max())
                R[k, j] = e / e.sum()
        Z = np.zeros((b2, b1, b1))             # Z[j, l, k]
        for j in range(b2):
            for k in range(b1):
                aL = sum(R[k, j, i] * Kv[k, i] for i in range(b2))
                cL = sum(R[k, j, i] * math.log(R[k, j, i]) for i in range(b2))
                for l in range(b1):
                    Z[j, l, k] = scale * np.dot(aL, Qv[l, j]) - cL
        for j in range(b2):
            for l in range(b1):
                e = np.exp(Z[j, l] - Z[j, l].max())
                L[j, l] = e / e.sum()
    O = np.zeros((b1, b2, Vv.shape[2]))
    for l in range(b1):
        for j in range(b2):
            for k in range(b1):
                Y = sum(R[k, j, i] * Vv[k, i] for i in range(b2))
                O[l, j] += L[j, l, k] * Y
    return torch.from_numpy(O.reshape(b1 * b2, -1))


def loops_tiled(Q, K, V, T, bb1, bb2, c1, c2, scale):
    """App. A.2 equations in their 7-index form (square case), python loops."""
    t1, t2 = bb1 // c1, bb2 // c2
    Q5 = Q.numpy().reshape(c1, t1, c2, t2, -1)      # l1 l2 j1 j2 v
    K5 = K.numpy().reshape(c1, t1, c2, t2, -1)      # k1 k2 i1 i2 v
    V5 = V.numpy().reshape(c1, t1, c2, t2, -1)
    # L[l1,j1,k1,i1,j2,l2,k2], R[l1,j1,k1,i1,k2,j2,i2]
    L = np.zeros((c1, c2, c1, c2, t2, t1, t1))
    L[..., :, :] = np.eye(t1)
    R = np.zeros((c1, c2, c1, c2, t1, t2, t2))
    tiles = list(itertools.product(range(c1), range(c2)))
    for _ in range(T):
        for (l1, j1), (k1, i1) in itertools.product(tiles, tiles):
            for k2, j2 in itertools.product(range(t1), range(t2)):
                a = sum(L[l1, j1, k1, i1, j2, l2, k2] * Q5[l1, l2, j1, j2] for l2 in range(t1))
                c = sum(L[l1, j1, k1, i1, j2, l2, k2] for l2 in range(t1))
                z = np.array([scale * np.dot(a, K5[k1, k2, i1, i2]) / c for i2 in range(t2)])
                e = np.exp(z - z.max())
                R[l1, j1, k1, i1, k2, j2] = e / e.sum()
        Z = np.zeros_like(L)
        for (l1, j1), (k1, i1) in itertools.product(tiles, tiles):
            for j2, k2 in itertools.product(range(t2), range(t1)):
                r = R[l1, j1, k1, i1, k2, j2]
                aL = sum(r[i2] * K5[k1, k2, i1, i2] for i2 in range(t2))
                cL = sum(r[i2] * math.log(r[i2]) for i2 in range(t2))
                for l2 in range(t1):
                    Z[l1, j1, k1, i1, j2, l2, k2] = scale * np.dot(aL, Q5[l1, l2, j1, j2]) - cL
        for (l1, j1) in tiles:
            for j2, l2 in itertools.product(range(t2), range(t1)):
                z = Z[l1, j1, :, :, j2, l2, :]              # over (k1, i1, k2)
                e = np.exp(z - z.max())
                L[l1, j1, :, :, j2, l2, :] = e / e.sum()
    O = np.zeros((c1, t1, c2, t2, V5.shape[-1]))
    for (l1, j1), (k1, i1) in itertools.product(tiles, tiles):
        for j2, k2 in itertools.product(range(t2), range(t1)):
            Y = sum(R[l1, j1, k1, i1, k2, j2, i2] * V5[k1, k2, i1, i2] for i2 in range(t2))
            for l2 in range(t1):
                O[l1, l2, j1, j2] += L[l1, j1, k1, i1, j2, l2, k2] * Y
    return torch.from_numpy(O.reshape(bb1 * bb2, -1))


@pytest.mark.parametrize("T", [1, 2, 3])
def test_p6_loops_vs_einsum_regular(T):
    b1, b2, d = 4, 3, 5
    Q, K, V = rnd((12, d), 70), rnd((12, d), 71), rnd((12, d), 72)
    O = mo.monarch_attention_regular(Q, K, V, T, b1, b2, 0.9)
    assert torch.allclose(O, loops_regular(Q, K, V, T, b1, b2, 0.9), atol=1e-13)


@pytest.mark.parametrize("T", [1, 2, 3])
def test_p6_loops_vs_einsum_tiled(T):
    bb1, bb2, c1, c2, d = 4, 6, 2, 2, 4
    N = bb1 * bb2
    Q, K, V = rnd((N, d), 73), rnd((N, d), 74), rnd((N, d), 75)
    g = mo.TileGeometry(bb1 // c1, bb2 // c2, c1, c1, c2)
    O = mo.monarch_attention_tiled(Q, K, V, T, g, 1.1)
    assert torch.allclose(O, loops_tiled(Q, K, V, T, bb1, bb2, c1, c2, 1.1), atol=1e-13)


def test_p6_illustration_sizes_12_and_18():
    # the 12x12 illustrations (regular (3,4); tiled with tiles (3,2)) and the 18-token
    # (f,h,w)=(2,3,3) example with (6,3): brute force vs einsum at the paper's own sizes
    Q, K, V = rnd((12, 4), 76), rnd((12, 4), 77), rnd((12, 4), 78)
    assert torch.allclose(mo.monarch_attention_regular(Q, K, V, 2, 3, 4),
                          loops_regular(Q, K, V, 2, 3, 4, 1.0), atol=1e-13)
    g = mo.TileGeometry(3, 2, 1, 1, 2)
    assert torch.allclose(mo.monarch_attention_tiled(Q, K, V, 2, g),
                          loops_tiled(Q, K, V, 2, 3, 4, 1, 2, 1.0), atol=1e-13)
    Q, K, V = rnd((18, 4), 79), rnd((18, 4), 80), rnd((18, 4), 81)
    O = mo.monarch_attn(Q, K, V, f_q=2, f_kv=2, h=3, w=3, b1=6, b2=3, tile=0, iters=2)
    assert torch.allclose(O, loops_regular(Q, K, V, 2, 6, 3, 1.0), atol=1e-13)


# ------------------------------------------------------------------ P7
def kl_rows(M, A):
    t = torch.where(M > 0, M * (torch.log(torch.where(M > 0, M, torch.ones_like(M))) - torch.log(A)),
                    torch.zeros_like(M))
    return t.sum().item()


def test_p7_kl_monotone_regular():
    b1, b2, d = 6, 4, 8
    Q, K, V = rnd((24, d), 90), rnd((24, d), 91), rnd((24, d), 92)
    A = torch.softmax(Q @ K.T, 1)
    kls = []
    for T in range(1, 7):
        _, L, R = mo.monarch_attention_regular(Q, K, V, T, b1, b2, return_factors=True)
        kls.append(kl_rows(mo.materialise_regular(L, R), A))
    assert all(k >= -1e-12 for k in kls)
    assert all(kls[t + 1] <= kls[t] + 1e-12 for t in range(len(kls) - 1))
    assert kls[-1] < kls[0]                       # it actually improves


def test_p7_kl_monotone_tiled():
    g = mo.TileGeometry(3, 2, 2, 2, 2)
    N, d = 24, 6
    Q, K, V = rnd((N, d), 93), rnd((N, d), 94), rnd((N, d), 95)
    A = torch.softmax(Q @ K.T, 1)
    kls = []
    for T in range(1, 7):
        _, ids, Ls, Rs = mo.monarch_attention_tiled(Q, K, V, T, g, return_factors=True)
        kls.append(kl_rows(mo.materialise_tiled(g, ids, Ls, Rs), A))
    assert all(k >= -1e-12 for k in kls)
    assert all(kls[t + 1] <= kls[t] + 1e-12 for t in range(len(kls) - 1))
    assert kls[-1] < kls[0]


# ------------------------------------------------------------------ P8
def test_p8_constant_v():
    g = mo.TileGeometry(3, 2, 1, 3, 2)
    Q, K = rnd((12, 5), 100), rnd((36, 5), 101)
    row = rnd((1, 7), 102)
    O = mo.monarch_attention_tiled(Q, K, row.expand(36, 7), 2, g)
    assert torch.allclose(O, row.expand(12, 7), atol=1e-13)


def test_scale_equals_prescaled_q():
    b1, b2 = 5, 4
    Q, K, V = rnd((20, 6), 110), rnd((20, 6), 111), rnd((20, 6), 112)
    assert torch.allclose(mo.monarch_attention_regular(Q, K, V, 2, b1, b2, 0.3),
                          mo.monarch_attention_regular(0.3 * Q, K, V, 2, b1, b2, 1.0), atol=1e-13)
    g = mo.TileGeometry(5, 2, 1, 1, 2)
    assert torch.allclose(mo.monarch_attention_tiled(Q, K, V, 2, g, 0.3),
                          mo.monarch_attention_tiled(0.3 * Q, K, V, 2, g, 1.0), atol=1e-13)


def test_to_tiles_token_order():
    # token = ((a*b1 + l)*c2 + b)*b2 + j  (Alg. 2 pseudocode rearrange; row-major grid, App. B.1)
    c1, b1, c2, b2 = 2, 3, 2, 4
    X = torch.arange(c1 * b1 * c2 * b2, dtype=F64)[:, None]
    Tt = mo.to_tiles(X, c1, b1, c2, b2)
    for a, b, l, j in itertools.product(range(c1), range(c2), range(b1), range(b2)):
        assert Tt[a * c2 + b, l, j, 0].item() == ((a * b1 + l) * c2 + b) * b2 + j
    assert torch.equal(mo.from_tiles(Tt, c1, b1, c2, b2), X)


def test_visibility_tables_for_the_kv_cache_configs():
    # 21-frame cache, 3-frame chunks, tiles of 3 frames x half width (30 rows per frame)
    g = mo.geometry_from_grid(3, 21, 30, 52, 90, 26, tile=1)
    assert (g.ntq, g.ntk) == (2, 14)
    assert mo.chunk_causal_visibility(g, 30, 3, 18).all()
    v = mo.chunk_causal_visibility(g, 30, 3, 9)
    assert v.sum(1).tolist() == [8, 8] and v[:, :8].all()
    assert mo.chunk_causal_visibility(g, 30, 0, 0).all()


# ------------------------------------------------------------------ mutation checks
def _p3_holds():
    b1, b2 = 5, 4
    Qt, Kt = general_separable_qk(1, 1, b1, b2, 35, 1.2)
    Q, K = Qt.reshape(b1 * b2, -1), Kt.reshape(b1 * b2, -1)
    V = rnd((b1 * b2, 6), 37)
    ok = True
    for T in (1, 2):
        O = mo.monarch_attention_regular(Q, K, V, T, b1, b2)
        ok &= bool(torch.allclose(O, textbook_dense(Q, K, V), atol=1e-9))
        g = mo.TileGeometry(b1, b2, 1, 1, 1)
        O = mo.monarch_attention_tiled(Q, K, V, T, g)
        ok &= bool(torch.allclose(O, textbook_dense(Q, K, V), atol=1e-9))
    return ok


def test_mutants_fail_the_pins(monkeypatch):
    assert _p3_holds()
    # dropped entropy term c_L
    with monkeypatch.context() as mp:
        mp.setattr(mo, "_xlogx_sum", lambda R, dim: torch.zeros_like(R.sum(dim)))
        assert not _p3_holds()
    # wrong sign of c_L
    orig = mo._xlogx_sum
    with monkeypatch.context() as mp:
        mp.setattr(mo, "_xlogx_sum", lambda R, dim: -orig(R, dim))
        assert not _p3_holds()
    # dropped division by c_R (visible from the second iteration on)
    with monkeypatch.context() as mp:
        mp.setattr(mo, "_safe_rows_div", lambda bR, cR: bR)
        assert not _p3_holds()
    assert _p3_holds()
