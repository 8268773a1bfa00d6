"""The oracle's factors have the shapes and parameter counts the paper states (Sec. 4.2 tiled
shape formula; Sec. 4.1 parameter count N (b1 + b2) of regular Monarch; tiling multiplies L's
parameters by c2 and R's by c1).  The expected numbers are a text fixture written out from those
statements, not produced by any code."""
import os

import pytest
import torch

from oracle import monarch_oracle as mo

ROWS = []
with open(os.path.join(os.path.dirname(__file__), "golden", "factor_shapes.txt")) as fh:
    for line in fh:
        line = line.split("#")[0].split()
        if line:
            ROWS.append(tuple(int(x) for x in line))


def rnd(shape, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=torch.float64)


def test_fixture_is_consistent_with_the_stated_formulas():
    assert len(ROWS) == 6
    for N, b1, b2, c1, c2, nL, nR in ROWS:
        assert b1 * b2 == N and b1 % c1 == 0 and b2 % c2 == 0
        # shape products of Sec. 4.2
        assert nL == c1 * c2 * c1 * c2 * (b2 // c2) * (b1 // c1) ** 2
        assert nR == c1 * c2 * c1 * c2 * (b1 // c1) * (b2 // c2) ** 2
        # regular count N (b1 + b2), times c2 for L and c1 for R
        assert nL == c2 * N * b1 and nR == c1 * N * b2


@pytest.mark.parametrize("row", ROWS)
def test_oracle_factors_have_the_stated_shapes(row):
    N, b1, b2, c1, c2, nL, nR = row
    Q, K, V = rnd((N, 4), 1), rnd((N, 4), 2), rnd((N, 3), 3)
    if c1 == c2 == 1:
        _, L, R = mo.monarch_attention_regular(Q, K, V, 2, b1, b2, return_factors=True)
        assert tuple(L.shape) == (b2, b1, b1) and tuple(R.shape) == (b1, b2, b2)
        assert L.numel() == nL and R.numel() == nR
    t1, t2 = b1 // c1, b2 // c2
    g = mo.TileGeometry(t1, t2, c1, c1, c2)
    _, ids, Ls, Rs = mo.monarch_attention_tiled(Q, K, V, 2, g, return_factors=True)
    assert len(Ls) == c1 * c2 and all(len(i) == c1 * c2 for i in ids)
    for Lm, Rm in zip(Ls, Rs):
        assert tuple(Lm.shape) == (c1 * c2, t2, t1, t1)       # n, j, k, l
        assert tuple(Rm.shape) == (c1 * c2, t1, t2, t2)       # n, k, j, i
    assert sum(x.numel() for x in Ls) == nL and sum(x.numel() for x in Rs) == nR
