"""Pins for the oracle's chunk-causal mask on REGULAR Monarch (one tile that straddles every
chunk): the mask depends on the block-row pair (l, k) alone, so it is a support constraint on L.
Each test checks the oracle against something fixed by the mathematics, not against itself.

  M1  degenerate blocks (N, 1): the masked operator IS masked dense softmax attention
      (Sec. 4.1: block size (N,1) is dense attention), for every T
  M2  separable logits a[l,k] + g[j,i] are represented exactly under the mask: output == masked
      dense attention for every T >= 1 (Sec. 4.1, aligned construction); not so for general logits
  M3  the materialised matrix M = L R (Sec. 4.2 entry formula) is zero exactly on the hidden
      token pairs, row-stochastic, and M @ V is the factored output
  M4  KL(M^(t) || masked softmax(QK^T)) never increases with t and is >= 0 (Sec. 2.1: the updates
      stay exact alternating maximisation when L's support is restricted)
  M5  a mask that hides nothing (chunk >= frames) is the unmasked algorithm; a frame offset that
      puts every query into the last chunk likewise
  M6  other assignments: (fw,h) with the mask equals the same algorithm on re-ordered tokens
      against masked dense attention for position-only (separable) logits
  plus mutation checks: a transposed mask, a dropped mask and shifted chunk boundaries fail the pins.
"""
import numpy as np
import pytest
import scipy.special
import torch

from oracle import monarch_oracle as mo

F64 = torch.float64


def rnd(shape, seed, sigma=1.0):
    g = torch.Generator().manual_seed(seed)
    return sigma * torch.randn(*shape, generator=g, dtype=F64)


def textbook_masked_dense(Q, K, V, f, h, w, cc, off=0):
    """softmax(QK^T + mask)V with numpy/scipy only; the mask written out token by token."""
    N = f * h * w
    S = Q.numpy() @ K.numpy().T
    frame = np.arange(N) // (h * w)
    vis = (frame[None, :] // cc) <= ((frame[:, None] + off) // cc)
    S = np.where(vis, S, -np.inf)
    return torch.from_numpy(scipy.special.softmax(S, axis=1) @ V.numpy()), torch.from_numpy(vis)


def separable_qk(rows, w, da, db, seed, sigma=1.0):
    qa, ka = rnd((rows, da), seed, sigma), rnd((rows, da), seed + 1, sigma)
    qb, kb = rnd((w, db), seed + 2, sigma), rnd((w, db), seed + 3, sigma)
    Q = torch.cat([qa[:, None, :].expand(rows, w, da), qb[None].expand(rows, w, db)], 2)
    K = torch.cat([ka[:, None, :].expand(rows, w, da), kb[None].expand(rows, w, db)], 2)
    return Q.reshape(rows * w, da + db).contiguous(), K.reshape(rows * w, da + db).contiguous()


def run(Q, K, V, f, h, w, T, cc, off=0, assign="fh_w", b1=None, b2=None):
    b1 = f * h if b1 is None else b1
    b2 = w if b2 is None else b2
    return mo.monarch_attn(Q, K, V, f_q=f, f_kv=f, h=h, w=w, b1=b1, b2=b2, tile=0, iters=T,
                           causal_chunk=cc, q_frame_offset=off, assign=assign)


# ------------------------------------------------------------------ M1
@pytest.mark.parametrize("T", [1, 2, 3])
@pytest.mark.parametrize("cc,off", [(1, 0), (2, 0), (2, 1)])
def test_m1_column_blocks_are_masked_dense(T, cc, off):
    f, h, w, d = 5, 3, 1, 6
    N = f * h * w
    Q, K, V = rnd((N, d), 1), rnd((N, d), 2), rnd((N, 4), 3)
    want, _ = textbook_masked_dense(Q, K, V, f, h, w, cc, off)
    assert torch.allclose(run(Q, K, V, f, h, w, T, cc, off), want, atol=1e-12)


# ------------------------------------------------------------------ M2
@pytest.mark.parametrize("T", [1, 2, 4])
@pytest.mark.parametrize("cc,off", [(1, 0), (2, 0), (3, 2)])
def test_m2_separable_logits_exact_under_the_mask(T, cc, off):
    f, h, w = 6, 2, 5
    Q, K = separable_qk(f * h, w, 3, 4, 20, 1.3)
    V = rnd((f * h * w, 7), 24)
    want, vis = textbook_masked_dense(Q, K, V, f, h, w, cc, off)
    assert not vis.all()
    got = run(Q, K, V, f, h, w, T, cc, off)
    assert torch.allclose(got, want, atol=1e-12)
    # the mask matters on these inputs
    assert not torch.allclose(got, run(Q, K, V, f, h, w, T, 0), atol=1e-3)


def test_m2_general_logits_are_only_approximated():
    f, h, w, d = 4, 2, 5, 8
    N = f * h * w
    Q, K, V = rnd((N, d), 5), rnd((N, d), 6), rnd((N, d), 7)
    want, _ = textbook_masked_dense(Q, K, V, f, h, w, 2)
    assert (run(Q, K, V, f, h, w, 2, 2) - want).abs().max() > 1e-3


# ------------------------------------------------------------------ M3
@pytest.mark.parametrize("T", [1, 3])
def test_m3_materialised_matrix_has_the_masks_support(T):
    f, h, w, d, cc = 4, 3, 4, 8, 2
    b1, b2, N = f * h, w, f * h * w
    Q, K, V = rnd((N, d), 11), rnd((N, d), 12), rnd((N, 5), 13)
    frame_of_row = torch.arange(b1) // h
    vis_rows = (frame_of_row[None, :] // cc) <= (frame_of_row[:, None] // cc)
    O, L, R = mo.monarch_attention_regular(Q, K, V, T, b1, b2, return_factors=True, row_visible=vis_rows)
    M = mo.materialise_regular(L, R)
    _, vis_tok = textbook_masked_dense(Q, K, V, f, h, w, cc)
    assert (M[~vis_tok] == 0).all() and (M[vis_tok] > 0).all()
    assert torch.allclose(M.sum(1), torch.ones(N, dtype=F64), atol=1e-13)
    assert torch.allclose(M @ V, O, atol=1e-13)
    assert torch.allclose(O, run(Q, K, V, f, h, w, T, cc), atol=0)


# ------------------------------------------------------------------ M4
def test_m4_kl_to_masked_attention_never_increases():
    f, h, w, d, cc = 4, 2, 4, 8, 2
    b1, b2, N = f * h, w, f * h * w
    Q, K, V = rnd((N, d), 90), rnd((N, d), 91), rnd((N, d), 92)
    frame = torch.arange(N) // (h * w)
    vis_tok = (frame[None, :] // cc) <= (frame[:, None] // cc)
    A = torch.softmax((Q @ K.T).masked_fill(~vis_tok, -float("inf")), 1)
    frame_of_row = torch.arange(b1) // h
    vis_rows = (frame_of_row[None, :] // cc) <= (frame_of_row[:, None] // cc)
    kls = []
    for T in range(1, 7):
        _, L, R = mo.monarch_attention_regular(Q, K, V, T, b1, b2, return_factors=True, row_visible=vis_rows)
        M = mo.materialise_regular(L, R)
        pos = M > 0
        kls.append((M[pos] * (torch.log(M[pos]) - torch.log(A[pos]))).sum().item())
    assert all(k >= -1e-12 for k in kls)
    assert all(kls[t + 1] <= kls[t] + 1e-12 for t in range(len(kls) - 1))
    assert kls[-1] < kls[0]


# ------------------------------------------------------------------ M5
@pytest.mark.parametrize("cc,off", [(4, 0), (9, 0), (2, 3)])
def test_m5_a_mask_that_hides_nothing_changes_nothing(cc, off):
    f, h, w, d = 4, 3, 5, 8
    N = f * h * w
    Q, K, V = rnd((N, d), 31), rnd((N, d), 32), rnd((N, d), 33)
    # (2, 3): queries sit at frames 3..6 of a 4-frame key grid, every key chunk is at or before chunk 1
    assert torch.equal(run(Q, K, V, f, h, w, 2, cc, off), run(Q, K, V, f, h, w, 2, 0))


# ------------------------------------------------------------------ M6
@pytest.mark.parametrize("assign,b1,b2", [("fw_h", 4 * 5, 3), ("f_hw", 4, 15)])
def test_m6_other_assignments_with_position_only_logits(assign, b1, b2):
    """Logits that are a sum of one term per video axis are separable for every assignment, so each
    masked regular Monarch reproduces masked dense attention (Sec. 4.1)."""
    f, h, w, cc = 4, 3, 5, 2
    parts_q = [rnd((n, 3), 40 + i, 1.2) for i, n in enumerate((f, h, w))]
    parts_k = [rnd((n, 3), 50 + i, 1.2) for i, n in enumerate((f, h, w))]

    def tokens(parts):
        a, b, c = parts
        return torch.cat([a[:, None, None, :].expand(f, h, w, 3), b[None, :, None, :].expand(f, h, w, 3),
                          c[None, None, :, :].expand(f, h, w, 3)], 3).reshape(f * h * w, 9).contiguous()

    Q, K = tokens(parts_q), tokens(parts_k)
    V = rnd((f * h * w, 6), 60)
    want, _ = textbook_masked_dense(Q, K, V, f, h, w, cc)
    for T in (1, 2):
        assert torch.allclose(run(Q, K, V, f, h, w, T, cc, 0, assign, b1, b2), want, atol=1e-12)


# ------------------------------------------------------------------ mutation checks
def _pins_hold():
    f, h, w = 5, 2, 4
    Q, K = separable_qk(f * h, w, 3, 4, 70, 1.3)
    V = rnd((f * h * w, 5), 74)
    want, _ = textbook_masked_dense(Q, K, V, f, h, w, 2)
    return all(bool(torch.allclose(run(Q, K, V, f, h, w, T, 2), want, atol=1e-9)) for T in (1, 2))


def test_mutants_fail_the_mask_pins(monkeypatch):
    assert _pins_hold()
    orig = mo.monarch_attention_regular
    # mask transposed (keys see later queries instead)
    with monkeypatch.context() as mp:
        mp.setattr(mo, "monarch_attention_regular",
                   lambda *a, row_visible=None, **k: orig(*a, row_visible=None if row_visible is None
                                                          else row_visible.T.contiguous(), **k))
        assert not _pins_hold()
    # mask dropped
    with monkeypatch.context() as mp:
        mp.setattr(mo, "monarch_attention_regular", lambda *a, row_visible=None, **k: orig(*a, **k))
        assert not _pins_hold()
    # chunk boundaries shifted by one frame
    with monkeypatch.context() as mp:
        def shifted(*a, row_visible=None, **k):
            rv = torch.roll(row_visible, 1, 1) | torch.eye(row_visible.shape[0], dtype=torch.bool)
            return orig(*a, row_visible=rv, **k)
        mp.setattr(mo, "monarch_attention_regular", shifted)
        assert not _pins_hold()
    assert _pins_hold()
