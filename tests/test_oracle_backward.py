"""CPU pins for the oracle's gradients (the backward pass of Sec. 4.3's Monarch finetuning).
None of the references below uses reverse-mode differentiation."""
import numpy as np
import pytest
import torch

from oracle import monarch_oracle as mo

F64 = torch.float64


def rnd(shape, seed, sigma=1.0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=F64) * sigma


CASES = {
    "regular-T1": dict(f_q=2, f_kv=2, h=3, w=4, b1=6, b2=4, tile=0, iters=1),
    "regular-T3": dict(f_q=2, f_kv=2, h=3, w=4, b1=6, b2=4, tile=0, iters=3),
    "tiled-rect-mask-T2": dict(f_q=1, f_kv=3, h=4, w=4, b1=2, b2=2, tile=1, iters=2, causal_chunk=1,
                               q_frame_offset=1),
    "tiled-T1": dict(f_q=2, f_kv=2, h=2, w=6, b1=2, b2=3, tile=1, iters=1),
    "fw_h-T2": dict(f_q=2, f_kv=2, h=3, w=4, b1=8, b2=3, tile=0, iters=2, assign="fw_h"),
    "regular-mask-T2": dict(f_q=3, f_kv=3, h=2, w=4, b1=6, b2=4, tile=0, iters=2, causal_chunk=1),
    "regular-mask-offset-T3": dict(f_q=4, f_kv=4, h=2, w=3, b1=8, b2=3, tile=0, iters=3, causal_chunk=2,
                                   q_frame_offset=1),
}


def inputs(kw, d=5, seed=0):
    nq, nk = kw["f_q"] * kw["h"] * kw["w"], kw["f_kv"] * kw["h"] * kw["w"]
    return rnd((nq, d), seed), rnd((nk, d), seed + 1), rnd((nk, d), seed + 2), rnd((nq, d), seed + 3)


@pytest.mark.parametrize("name", list(CASES))
def test_gradients_match_central_differences(name):
    kw = dict(CASES[name], scale=0.6)
    Q, K, V, dO = inputs(kw)
    gQ, gK, gV = mo.monarch_attn_grad(Q, K, V, dO, **kw)

    def f(q, k, v):
        return float((mo.monarch_attn(q, k, v, **kw) * dO).sum())

    eps = 1e-6
    for trial in range(4):
        U, W, X = rnd(Q.shape, 50 + trial), rnd(K.shape, 60 + trial), rnd(V.shape, 70 + trial)
        for which, (G, D) in enumerate(((gQ, U), (gK, W), (gV, X))):
            z = [torch.zeros_like(Q), torch.zeros_like(K), torch.zeros_like(V)]
            z[which] = D
            num = (f(Q + eps * z[0], K + eps * z[1], V + eps * z[2]) -
                   f(Q - eps * z[0], K - eps * z[1], V - eps * z[2])) / (2 * eps)
            ana = float((G * D).sum())
            assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana)), (name, which, num, ana)


@pytest.mark.parametrize("name", ["regular-T3", "tiled-rect-mask-T2"])
def test_value_gradient_is_the_transposed_matrix_times_dO(name):
    # O = M V with M independent of V, so dV = M^T dO; M is materialised by feeding the identity
    kw = dict(CASES[name], scale=0.6)
    Q, K, V, dO = inputs(kw)
    M = mo.monarch_attn(Q, K, torch.eye(K.shape[0], dtype=F64), **kw)
    _, _, gV = mo.monarch_attn_grad(Q, K, V, dO, **kw)
    assert torch.allclose(gV, M.T @ dO, atol=1e-12)
    # rows of M sum to one: the value gradients of all keys add up to the output gradients
    assert torch.allclose(gV.sum(0), dO.sum(0), atol=1e-12)


def dense_backward(Q, K, V, dO, scale):
    """Textbook gradient of softmax(scale Q K^T) V."""
    Qn, Kn, Vn, G = (x.numpy() for x in (Q, K, V, dO))
    S = scale * Qn @ Kn.T
    P = np.exp(S - S.max(1, keepdims=True))
    P /= P.sum(1, keepdims=True)
    dV = P.T @ G
    dP = G @ Vn.T
    dS = P * (dP - (dP * P).sum(1, keepdims=True))
    return scale * dS @ Kn, scale * dS.T @ Qn, dV


@pytest.mark.parametrize("blocks,T", [((12, 1), 1), ((1, 12), 2), ((12, 1), 3)])
def test_degenerate_blocks_have_the_dense_attention_gradient(blocks, T):
    # b1 = 1 or b2 = 1 makes MonarchAttention equal to dense attention for every input, so the
    # gradients agree as well
    b1, b2 = blocks
    kw = dict(f_q=1, f_kv=1, h=b1, w=b2, b1=b1, b2=b2, tile=0, iters=T, scale=0.8)
    Q, K, V, dO = inputs(kw, d=4, seed=9)
    gQ, gK, gV = mo.monarch_attn_grad(Q, K, V, dO, **kw)
    rQ, rK, rV = dense_backward(Q, K, V, dO, 0.8)
    assert np.allclose(gQ.numpy(), rQ, atol=1e-10)
    assert np.allclose(gK.numpy(), rK, atol=1e-10)
    assert np.allclose(gV.numpy(), rV, atol=1e-10)


def test_gradients_are_linear_in_dO_and_leave_inputs_untouched():
    kw = dict(CASES["tiled-T1"], scale=1.0)
    Q, K, V, dO = inputs(kw)
    Q0 = Q.clone()
    g1 = mo.monarch_attn_grad(Q, K, V, dO, **kw)
    g2 = mo.monarch_attn_grad(Q, K, V, -2.5 * dO, **kw)
    for a, b in zip(g1, g2):
        assert torch.allclose(-2.5 * a, b, atol=1e-12)
    assert torch.equal(Q, Q0) and not Q.requires_grad
