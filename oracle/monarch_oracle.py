"""fp64 CPU oracle for MonarchRT attention.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain statement of what the operator computes.  It is
imported by tests, by the smoke check and by the benchmark's cpu_baseline leg,
and by nothing on the product path.  It shares no code with the HIP kernels and
never imports them.

Every function works on ONE head: Q is [N_q, d], K and V are [N_kv, d], tokens
in row-major (frame, height, width) order (App. B.1, the ordering called phi).
All arithmetic is float64 (torch CPU tensors); inputs of any float dtype are
widened first.

Notation follows App. A (the update equations of Alg. 1 / Alg. 2):
  l  query row inside a tile      j  column inside a tile (queries and keys)
  k  key row inside a tile        i  key column inside a tile
  m  query tile                   n  key tile              v  feature
  L[m,n,j,k,l], R[m,n,k,j,i]      (regular Monarch: one tile, m = n = 0)

Readings taken where the paper is silent or garbled (each is listed in the
design document as well):
  * an explicit `scale` multiplies both logit contractions (beta_R, beta_L);
    scale = 1 is the paper's softmax(Q K^T).
  * c_L sums R log R over i (the text's summation index is a typo; the
    pseudocode's einsum is over i), with 0 log 0 = 0.
  * the tiled pseudocode's second rearrange assigns K.
  * rectangular N_q != N_kv: query tiles m and key tiles n are counted
    separately, the initial L is the identity in (k,l) for every pair (m,n).
  * chunk-causal mask: applied per tile pair.  A key tile is visible to a query
    tile iff the chunk of the key tile's frames is not later than the chunk of
    the query tile's frames; hidden pairs take no part at all (no R, not in the
    joint softmax of L).  A tile never straddles a chunk boundary.
  * chunk-causal mask on regular Monarch (one tile, which straddles every chunk):
    with the frame as the slowest axis of the block row index the mask depends on
    the row pair (l, k) alone, so the hidden entries of the attention matrix are
    the hidden entries of L[j, k, l]: L's softmax over k runs over the key rows
    whose frame's chunk is not later than the query row's.  R, c_L, alpha_R / c_R
    are unchanged in form (they see L's zeros).  The updates are then still the
    exact alternating maximisation of the variational objective of Sec. 3 over
    Monarch matrices with that support.  The diagonal (k = l) is always visible,
    so the identity initialisation respects the mask.
  * tiles are the contiguous row / column ranges of Alg. 2's rearrange, so any
    b1 dividing the row count is a tiling (also a fraction of a frame: the
    neighbourhood tiles of Sec. 4.2 with n_f = 1).
  * Sec. 4.2's neighbourhood tiles (n_f frames x n_h rows x n_w columns) with
    n_f > 1 and n_h < h are not a contiguous row range of the stored order; they
    are the same algorithm on tokens re-ordered so that each neighbourhood's rows
    are consecutive (neighbourhood_order), the mask taken per frame group.
  * the six aligned block assignments of Sec. 4.1 are the same algorithm on
    tokens re-ordered so that the axes given to b1 become the row index and the
    axes given to b2 the column index (block_assignment_order).
  * beta_R / c_R with c_R == 0 exactly: that row of Z_R is set to 0 (uniform R).

Parity status: every function here is pinned by tests/test_oracle_pins.py
(degenerate block sizes == dense softmax attention; separable logits == dense
for every T; materialised M @ V == factored product; row-stochasticity;
parameter tying; an independent index-loop transcription of the update
equations; monotone KL along the iterations; constant V) and, for the block
assignments and fractional-frame tiles, by tests/test_oracle_assignments.py
(rank-one block structure of the materialised matrix under an index map
written out in the test; position-only logits == dense for all six
assignments; assignments that coincide on degenerate grids).  monarch_attn_grad is
pinned by tests/test_oracle_backward.py (central differences of the forward oracle,
dV = M^T dO with the materialised matrix, the closed-form gradient of dense attention
for degenerate block sizes).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

F64 = torch.float64


# --------------------------------------------------------------------------
# geometry (index arithmetic only)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class TileGeometry:
    """Tile-local block sizes (b1, b2) laid over row-major (f*h, w) token grids.

    Rows of the grid are (frame, height) pairs, columns are width (Sec. 4.1,
    the aligned choice (fh, w)); a tile is b1 consecutive rows by b2 consecutive
    columns (Alg. 2 pseudocode, the "(a l b j)" split).  c1q / c1k count row
    tiles of the query / key grid, c2 counts column tiles of both.
    """

    b1: int
    b2: int
    c1q: int
    c1k: int
    c2: int

    @property
    def ntq(self) -> int:
        return self.c1q * self.c2

    @property
    def ntk(self) -> int:
        return self.c1k * self.c2


def to_tiles(X: torch.Tensor, c1: int, b1: int, c2: int, b2: int) -> torch.Tensor:
    """[(a l b j), v] -> [(a b), l, j, v]   (Alg. 2 pseudocode, the rearranges)."""
    N, d = X.shape
    assert N == c1 * b1 * c2 * b2
    X = X.reshape(c1, b1, c2, b2, d)            # a l b j v
    X = X.permute(0, 2, 1, 3, 4)                # a b l j v
    return X.reshape(c1 * c2, b1, b2, d).contiguous()


def from_tiles(Z: torch.Tensor, c1: int, b1: int, c2: int, b2: int) -> torch.Tensor:
    """[(a b), l, j, v] -> [(a l b j), v]   (inverse of to_tiles)."""
    d = Z.shape[-1]
    Z = Z.reshape(c1, c2, b1, b2, d).permute(0, 2, 1, 3, 4)
    return Z.reshape(c1 * b1 * c2 * b2, d).contiguous()


def chunk_causal_visibility(geom: TileGeometry, h: int, causal_chunk: int,
                            q_frame_offset: int, tile_h: int = 0) -> torch.Tensor:
    """visible[m, n] for the tile-level chunk-causal reading (see module header).

    h = grid rows per frame.  Query tile row a covers grid rows a*b1 ... of
    frames starting at q_frame_offset; key tile row a' covers rows a'*b1 ... of
    frames starting at 0.  With neighbourhood tiles (tile_h = n_h > 0, rows
    ordered by neighbourhood_order) tile row a covers the n_f = b1 / n_h frames
    of frame group a // (h / n_h).  causal_chunk == 0 means no mask.
    """
    vis = torch.ones(geom.ntq, geom.ntk, dtype=torch.bool)
    if causal_chunk == 0:
        return vis

    def chunk_of_tile_row(a: int, first_frame: int) -> int:
        if tile_h > 0:
            n_f = geom.b1 // tile_h
            f0 = (a // (h // tile_h)) * n_f
            f1 = f0 + n_f - 1
        else:
            f0, f1 = (a * geom.b1) // h, (a * geom.b1 + geom.b1 - 1) // h
        lo, hi = (first_frame + f0) // causal_chunk, (first_frame + f1) // causal_chunk
        assert lo == hi, "a tile straddles a causal chunk"
        return lo

    for m in range(geom.ntq):
        q_chunk = chunk_of_tile_row(m // geom.c2, q_frame_offset)
        for n in range(geom.ntk):
            vis[m, n] = chunk_of_tile_row(n // geom.c2, 0) <= q_chunk
    return vis


# --------------------------------------------------------------------------
# dense attention (Sec. 2.2: Attn(Q,K,V) = softmax(Q K^T) V, row-wise softmax)
# --------------------------------------------------------------------------
def dense_attention(Q, K, V, scale: float = 1.0,
                    mask: Optional[torch.Tensor] = None) -> torch.Tensor:
    Q, K, V = Q.to(F64), K.to(F64), V.to(F64)
    S = scale * (Q @ K.T)
    if mask is not None:
        S = S.masked_fill(~mask, -math.inf)
    return torch.softmax(S, dim=1) @ V


def token_chunk_causal_mask(f_q: int, f_kv: int, h: int, w: int, causal_chunk: int,
                            q_frame_offset: int) -> Optional[torch.Tensor]:
    """Token-level chunk-causal mask [N_q, N_kv]: a key is visible iff its frame's
    chunk is not later than the query frame's chunk.  None when causal_chunk == 0."""
    if causal_chunk == 0:
        return None
    qf = (torch.arange(f_q * h * w) // (h * w) + q_frame_offset) // causal_chunk
    kf = (torch.arange(f_kv * h * w) // (h * w)) // causal_chunk
    return kf[None, :] <= qf[:, None]


# --------------------------------------------------------------------------
# Alg. 1: regular MonarchAttention (App. A.1)
# --------------------------------------------------------------------------
def _xlogx_sum(R: torch.Tensor, dim: int) -> torch.Tensor:
    """sum R log R along dim with 0 log 0 = 0."""
    return torch.where(R > 0, R * torch.log(torch.where(R > 0, R, torch.ones_like(R))),
                       torch.zeros_like(R)).sum(dim)


def _safe_rows_div(bR: torch.Tensor, cR: torch.Tensor) -> torch.Tensor:
    """beta_R / c_R along the last axis; rows with c_R == 0 become all-zero logits."""
    c = cR.unsqueeze(-1)
    return torch.where(c != 0, bR / torch.where(c != 0, c, torch.ones_like(c)),
                       torch.zeros_like(bR))


def monarch_attention_regular(Q, K, V, T: int, b1: int, b2: int, scale: float = 1.0,
                              return_factors: bool = False,
                              row_visible: Optional[torch.Tensor] = None):
    """App. A.1, the update equations of one iteration, written as batched matrix products.
    N = b1*b2; Q, K, V are read as b1 x b2 x d tensors Q[l, j, :], K[k, i, :], V[k, i, :].

    The factors are held the way the text of App. A.1 indexes them: L[j, l, k] (for column j,
    a b1 x b1 matrix from query row l to key row k, each row a distribution over k) and
    R[k, j, i] (for key row k, a b2 x b2 matrix from query column j to key column i, each row a
    distribution over i).  Column j of the query grid is the matrix Qcol[j] = Q[:, j, :], row k of
    the key grid the matrix Krow[k] = K[k, :, :]; every update below is then one batched product
    over j (the L side) or over k (the R side).

    Returns O [N, d]; on request also the factors, L as [j, k, l] (transposed, the layout
    materialise_regular takes) and R as [k, j, i].

    row_visible[l, k] (bool, optional): key row k is visible to query row l.  A hidden
    (l, k) is a zero of the attention matrix for every (j, i), i.e. a zero of L[j, l, k]:
    the softmax of L over k runs over the visible k only (see the module header)."""
    assert T >= 1
    N, d = Q.shape
    assert N == b1 * b2 and K.shape == (N, d) and V.shape[0] == N
    Qcol = Q.to(F64).reshape(b1, b2, d).transpose(0, 1)          # [j][l, v]
    Krow = K.to(F64).reshape(b1, b2, d)                          # [k][i, v]
    Vrow = V.to(F64).reshape(b1, b2, V.shape[1])                 # [k][i, v]
    if row_visible is not None:
        assert row_visible.shape == (b1, b1) and bool(row_visible.diagonal().all())
    Lf = torch.eye(b1, dtype=F64).repeat(b2, 1, 1)               # L^(0)[j][l, k] = delta(l, k)
    Rf = None
    for _ in range(T):
        # R update.  alpha_R[k, j, :] = sum_l L[j, l, k] Q[l, j, :],  c_R[k, j] = sum_l L[j, l, k]
        alpha_R = torch.matmul(Lf.transpose(1, 2), Qcol)         # [j][k, v]
        c_R = Lf.sum(dim=1)                                      # [j][k]
        # beta_R[k, j, i] = sum_v alpha_R[k, j, v] K[k, i, v]: for each k, (rows j) x Krow[k]^T
        beta_R = torch.matmul(alpha_R.transpose(0, 1), Krow.transpose(1, 2))      # [k][j, i]
        Z_R = _safe_rows_div(scale * beta_R, c_R.transpose(0, 1))
        Rf = torch.softmax(Z_R, dim=2)                           # over i
        # L update.  alpha_L[j, k, :] = sum_i R[k, j, i] K[k, i, :],  c_L[j, k] = sum_i R log R
        alpha_L = torch.matmul(Rf, Krow)                         # [k][j, v]
        c_L = _xlogx_sum(Rf, 2)                                  # [k][j]
        # beta_L[j, l, k] = sum_v alpha_L[j, k, v] Q[l, j, v]: for each j, Qcol[j] x (rows k)^T
        beta_L = torch.matmul(Qcol, alpha_L.permute(1, 2, 0))    # [j][l, k]
        Z_L = scale * beta_L - c_L.transpose(0, 1)[:, None, :]
        if row_visible is not None:
            Z_L = Z_L.masked_fill(~row_visible[None, :, :], -math.inf)
        Lf = torch.softmax(Z_L, dim=2)                           # over k
    # Y[k, j, :] = sum_i R[k, j, i] V[k, i, :],  O[l, j, :] = sum_k L[j, l, k] Y[k, j, :]
    Yf = torch.matmul(Rf, Vrow)                                  # [k][j, v]
    Ocol = torch.matmul(Lf, Yf.transpose(0, 1))                  # [j][l, v]
    O = Ocol.transpose(0, 1).reshape(N, -1)
    if return_factors:
        return O, Lf.transpose(1, 2).contiguous(), Rf
    return O


def materialise_regular(L: torch.Tensor, R: torch.Tensor) -> torch.Tensor:
    """Sec. 4.2: M[(l*b2 + j), (k*b2 + i)] = L[j,l,k] * R[k,j,i], with L stored
    as [j,k,l] like the pseudocode does."""
    b2, b1, _ = L.shape
    M4 = torch.einsum("jkl,kji->ljki", L, R)
    return M4.reshape(b1 * b2, b1 * b2)


# --------------------------------------------------------------------------
# Alg. 2: tiled MonarchAttention (App. A.2), rectangular + tile mask
# --------------------------------------------------------------------------
def _tiled_one_query_tile(Qm, Kt, Vt, T, scale):
    """App. A.2's update equations for ONE query tile (l_1, j_1 fixed) against the list of its
    visible key tiles (k_1, i_1) = n, as batched matrix products.

    Qm [b1, b2, d] is the query tile, Q[l, j, :]; Kt, Vt [nv, b1, b2, d] the key tiles,
    K[n, k, i, :].  The factors are held as App. A.2 indexes them with the tile pair dropped:
    L[n][j][l, k] and R[n][k][j, i].  The R side is the regular update once per key tile; the L
    side differs in one place: for every (j, l) the softmax runs over ALL (n, k) together.

    Returns the tile of the output O[l, j, :] and the factors, L as [n, j, k, l] (the layout
    materialise_tiled takes) and R as [n, k, j, i].
    """
    nv, b1, b2, _ = Kt.shape
    Qcol = Qm.transpose(0, 1)                                    # [j][l, v]
    Lf = torch.eye(b1, dtype=F64).repeat(nv, b2, 1, 1)           # L^(0)[n][j][l, k] = delta(l, k)
    Rf = None
    for _ in range(T):
        # R update, per key tile n
        alpha_R = torch.matmul(Lf.transpose(2, 3), Qcol)         # [n][j][k, v]
        c_R = Lf.sum(dim=2)                                      # [n][j][k]
        beta_R = torch.matmul(alpha_R.transpose(1, 2), Kt.transpose(2, 3))        # [n][k][j, i]
        Rf = torch.softmax(_safe_rows_div(scale * beta_R, c_R.transpose(1, 2)), dim=3)   # over i
        # L update: logits per key tile, then one softmax per (j, l) across every (n, k)
        alpha_L = torch.matmul(Rf, Kt)                           # [n][k][j, v]
        c_L = _xlogx_sum(Rf, 3)                                  # [n][k][j]
        beta_L = torch.matmul(Qcol, alpha_L.permute(0, 2, 3, 1))                  # [n][j][l, k]
        Z_L = scale * beta_L - c_L.transpose(1, 2)[:, :, None, :]
        joint = Z_L.permute(1, 2, 0, 3).reshape(b2, b1, nv * b1)                  # [j][l, (n k)]
        Lf = torch.softmax(joint, dim=2).reshape(b2, b1, nv, b1).permute(2, 0, 1, 3)   # [n][j][l, k]
    Yf = torch.matmul(Rf, Vt)                                    # [n][k][j, v]
    # O[l, j, :] = sum_{n, k} L[n, j, l, k] Y[n, k, j, :]
    Ocol = torch.matmul(Lf, Yf.transpose(1, 2)).sum(dim=0)       # [j][l, v]
    return Ocol.transpose(0, 1).contiguous(), Lf.transpose(2, 3).contiguous(), Rf


def monarch_attention_tiled(Q, K, V, T: int, geom: TileGeometry, scale: float = 1.0,
                            visible: Optional[torch.Tensor] = None,
                            return_factors: bool = False):
    """App. A.2 update equations / pseudocode (b), generalised to N_q != N_kv and
    to a tile-pair visibility table.  Query tiles are independent of each other
    (the joint softmax of L runs over key tiles only), so the loop over m below
    is the algorithm itself, not a blocking of it.

    Returns O [N_q, dv]; with return_factors also lists (per m) of the visible
    key-tile ids, L[n,j,k,l] and R[n,k,j,i].
    """
    assert T >= 1
    g = geom
    Qt = to_tiles(Q.to(F64), g.c1q, g.b1, g.c2, g.b2)            # m l j v
    Kt = to_tiles(K.to(F64), g.c1k, g.b1, g.c2, g.b2)            # n k i v
    Vt = to_tiles(V.to(F64), g.c1k, g.b1, g.c2, g.b2)
    if visible is None:
        visible = torch.ones(g.ntq, g.ntk, dtype=torch.bool)
    Z = torch.zeros(g.ntq, g.b1, g.b2, V.shape[1], dtype=F64)
    vis_ids: List[torch.Tensor] = []
    Ls, Rs = [], []
    for m in range(g.ntq):
        ids = torch.nonzero(visible[m]).flatten()
        assert ids.numel() > 0, "a query tile with no visible key tile has no softmax"
        Zm, Lm, Rm = _tiled_one_query_tile(Qt[m], Kt[ids], Vt[ids], T, scale)
        Z[m] = Zm
        if return_factors:
            vis_ids.append(ids); Ls.append(Lm); Rs.append(Rm)
    O = from_tiles(Z, g.c1q, g.b1, g.c2, g.b2)
    if return_factors:
        return O, vis_ids, Ls, Rs
    return O


def materialise_tiled(geom: TileGeometry, vis_ids: Sequence[torch.Tensor],
                      Ls: Sequence[torch.Tensor], Rs: Sequence[torch.Tensor]) -> torch.Tensor:
    """M[(m,l,j),(n,k,i)] = L[m,n,j,k,l] * R[m,n,k,j,i] in token order
    (Sec. 4.2, tiled factors); hidden tile pairs are zero."""
    g = geom
    nq = g.ntq * g.b1 * g.b2
    nk = g.ntk * g.b1 * g.b2
    # token index of (tile, row, col)
    def tok(c2, tile, r, c):
        a, b = tile // c2, tile % c2
        return ((a * g.b1 + r) * c2 + b) * g.b2 + c
    M = torch.zeros(nq, nk, dtype=F64)
    rows = torch.arange(g.b1)
    cols = torch.arange(g.b2)
    for m in range(g.ntq):
        qtok = tok(g.c2, m, rows[:, None], cols[None, :])        # l j
        for s, n in enumerate(vis_ids[m].tolist()):
            ktok = tok(g.c2, n, rows[:, None], cols[None, :])    # k i
            blk = torch.einsum("jkl,kji->ljki", Ls[m][s], Rs[m][s])
            M[qtok[:, :, None, None], ktok[None, None, :, :]] = blk
    return M


# --------------------------------------------------------------------------
# whole-operator front end (same argument meaning as the C ABI, one head)
# --------------------------------------------------------------------------
def geometry_from_grid(f_q: int, f_kv: int, h: int, w: int, b1: int, b2: int,
                       tile: int) -> TileGeometry:
    if tile == 0:
        assert f_q == f_kv and b1 == f_q * h and b2 == w
        return TileGeometry(b1, b2, 1, 1, 1)
    assert (f_q * h) % b1 == 0 and (f_kv * h) % b1 == 0 and w % b2 == 0
    return TileGeometry(b1, b2, (f_q * h) // b1, (f_kv * h) // b1, w // b2)


# --------------------------------------------------------------------------
# aligned block assignments (Sec. 4.1): which video axes index the b1 side and
# which the b2 side.  "fh_w" is the order the tokens are stored in.
# --------------------------------------------------------------------------
ASSIGNMENTS = ("fh_w", "w_fh", "fw_h", "h_fw", "f_hw", "hw_f")


def block_assignment_order(assign: str, f: int, h: int, w: int):
    """(order, rows, cols, rows_per_frame): order[x * cols + y] is the stored token
    (frame, height, width row-major) that sits at row x, column y of the block
    grid when the axes before the underscore index rows (first letter slowest)
    and the axes after it index columns.  rows_per_frame is rows / f when the
    frame axis is the slowest row axis, else 0 (frames are then not a row range)."""
    assert assign in ASSIGNMENTS
    row_axes, col_axes = assign.split("_")
    size = {"f": f, "h": h, "w": w}
    grid = torch.arange(f * h * w).reshape(f, h, w)
    names = "fhw"
    axes = [names.index(c) for c in row_axes + col_axes]
    rows = math.prod(size[c] for c in row_axes)
    cols = math.prod(size[c] for c in col_axes)
    order = grid.permute(*axes).reshape(rows * cols)
    rpf = rows // f if row_axes[0] == "f" else 0
    return order, rows, cols, rpf


def neighbourhood_order(f: int, h: int, w: int, n_f: int, n_h: int) -> torch.Tensor:
    """Stored tokens re-ordered so that every spatiotemporal neighbourhood of n_f frames by n_h
    grid rows (Sec. 4.2's example: tiles of n_f * n_h rows by n_w columns) is a run of
    n_f * n_h consecutive rows of w tokens: neighbourhoods ordered by (frame group, row band),
    rows inside one by (frame, row)."""
    assert f % n_f == 0 and h % n_h == 0
    g = torch.arange(f * h * w).reshape(f // n_f, n_f, h // n_h, n_h, w)   # fa u ha v x
    return g.permute(0, 2, 1, 3, 4).reshape(f * h * w)                      # fa ha u v x


def monarch_attn(Q, K, V, *, f_q: int, f_kv: int, h: int, w: int, b1: int, b2: int,
                 tile: int, iters: int, causal_chunk: int = 0, q_frame_offset: int = 0,
                 scale: float = 1.0, assign: str = "fh_w", tile_h: int = 0) -> torch.Tensor:
    """One head of the operator the library exports: regular (tile=0, Alg. 1) or
    tiled (tile=1, Alg. 2) MonarchAttention on (f,h,w) grids, for any of the six
    aligned block assignments (Sec. 4.1); tile_h = n_h > 0 tiles the (fh, w) grid into
    neighbourhoods of (b1 / n_h) frames x n_h rows x b2 columns (Sec. 4.2)."""
    if tile_h > 0:
        assert tile == 1 and assign == "fh_w" and b1 % tile_h == 0 and h % tile_h == 0
        n_f = b1 // tile_h
        oq = neighbourhood_order(f_q, h, w, n_f, tile_h)
        ok = neighbourhood_order(f_kv, h, w, n_f, tile_h)
        g = geometry_from_grid(f_q, f_kv, h, w, b1, b2, 1)
        vis = chunk_causal_visibility(g, h, causal_chunk, q_frame_offset, tile_h)
        out = monarch_attention_tiled(Q[oq], K[ok], V[ok], iters, g, scale, vis)
        O = torch.empty_like(out)
        O[oq] = out
        return O
    if assign != "fh_w":
        oq, rows_q, cols_q, rpf = block_assignment_order(assign, f_q, h, w)
        ok, rows_k, cols_k, _ = block_assignment_order(assign, f_kv, h, w)
        assert cols_q == cols_k, "the frame axis is on the column side: f_q must equal f_kv"
        if rpf == 0:
            assert causal_chunk == 0 and f_q == f_kv, "frames are not a row range"
            fq2, fk2, h2 = 1, 1, rows_q
        else:
            fq2, fk2, h2 = f_q, f_kv, rpf
        out = monarch_attn(Q[oq], K[ok], V[ok], f_q=fq2, f_kv=fk2, h=h2, w=cols_q, b1=b1, b2=b2,
                           tile=tile, iters=iters, causal_chunk=causal_chunk,
                           q_frame_offset=q_frame_offset, scale=scale)
        O = torch.empty_like(out)
        O[oq] = out
        return O
    g = geometry_from_grid(f_q, f_kv, h, w, b1, b2, tile)
    if tile == 0:
        vis_rows = None
        if causal_chunk > 0:
            assert f_q == f_kv and b1 == f_q * h
            rows = torch.arange(b1) // h                         # frame of a block row
            vis_rows = (rows[None, :] // causal_chunk) <= ((rows[:, None] + q_frame_offset) // causal_chunk)
        return monarch_attention_regular(Q, K, V, iters, b1, b2, scale, row_visible=vis_rows)
    vis = chunk_causal_visibility(g, h, causal_chunk, q_frame_offset)
    return monarch_attention_tiled(Q, K, V, iters, g, scale, vis)


def monarch_attn_grad(Q, K, V, dO, **kw):
    """Gradients (dQ, dK, dV) of sum(O * dO) for O = monarch_attn(Q, K, V, **kw): the backward
    pass that Monarch finetuning needs (Sec. 4.3).  Reverse-mode differentiation of the fp64
    definition above, every iteration included (nothing is treated as a constant)."""
    Qg, Kg, Vg = (x.detach().to(F64).clone().requires_grad_(True) for x in (Q, K, V))
    O = monarch_attn(Qg, Kg, Vg, **kw)
    gQ, gK, gV = torch.autograd.grad(O, (Qg, Kg, Vg), grad_outputs=dO.to(F64))
    return gQ, gK, gV


def dense_attn(Q, K, V, *, f_q: int, f_kv: int, h: int, w: int, causal_chunk: int = 0,
               q_frame_offset: int = 0, scale: float = 1.0) -> torch.Tensor:
    mask = token_chunk_causal_mask(f_q, f_kv, h, w, causal_chunk, q_frame_offset)
    return dense_attention(Q, K, V, scale, mask)
