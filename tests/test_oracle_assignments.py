"""CPU pins for the oracle's aligned block assignments (Sec. 4.1) and for tiles that are a
fraction of a frame (Sec. 4.2 with n_f = 1).  The index maps below are written out by hand and
do not call the oracle's own re-ordering."""
import itertools

import numpy as np
import pytest
import torch

from oracle import monarch_oracle as mo
from workloads import synthetic as syn

# (row index x, column index y) of grid cell (fi, hi, wi) on an (f, h, w) grid
XY = {
    "fh_w": lambda fi, hi, wi, f, h, w: (fi * h + hi, wi),
    "w_fh": lambda fi, hi, wi, f, h, w: (wi, fi * h + hi),
    "fw_h": lambda fi, hi, wi, f, h, w: (fi * w + wi, hi),
    "h_fw": lambda fi, hi, wi, f, h, w: (hi, fi * w + wi),
    "f_hw": lambda fi, hi, wi, f, h, w: (fi, hi * w + wi),
    "hw_f": lambda fi, hi, wi, f, h, w: (hi * w + wi, fi),
}
SIZES = {
    "fh_w": lambda f, h, w: (f * h, w), "w_fh": lambda f, h, w: (w, f * h),
    "fw_h": lambda f, h, w: (f * w, h), "h_fw": lambda f, h, w: (h, f * w),
    "f_hw": lambda f, h, w: (f, h * w), "hw_f": lambda f, h, w: (h * w, f),
}


def token_of(assign, f, h, w):
    """tok[x][y] = stored token (frame, height, width row-major) at block coordinates (x, y)."""
    X, Y = SIZES[assign](f, h, w)
    tok = -np.ones((X, Y), dtype=np.int64)
    for fi, hi, wi in itertools.product(range(f), range(h), range(w)):
        x, y = XY[assign](fi, hi, wi, f, h, w)
        assert tok[x, y] == -1
        tok[x, y] = (fi * h + hi) * w + wi
    assert (tok >= 0).all()
    return tok


def rnd(shape, seed, sigma=1.0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=torch.float64) * sigma


def materialise(assign, f, h, w, T, seed=0, d=8):
    N = f * h * w
    Q, K = rnd((N, d), seed), rnd((N, d), seed + 1)
    X, Y = SIZES[assign](f, h, w)
    return mo.monarch_attn(Q, K, torch.eye(N, dtype=torch.float64), f_q=f, f_kv=f, h=h, w=w, b1=X,
                           b2=Y, tile=0, iters=T, assign=assign).numpy()


def block_rank_defect(M, tok):
    """largest ratio s2/s1 over the blocks B[x0, y1] = M[tok(x0,y0), tok(x1,y1)] (fixed y0, x1):
    zero iff M[(x0,y0),(x1,y1)] = L[y0,x0,x1] * R[x1,y0,y1] (Sec. 4.2's entry formula)."""
    X, Y = tok.shape
    worst = 0.0
    for y0, x1 in itertools.product(range(Y), range(X)):
        B = M[np.ix_(tok[:, y0], tok[x1, :])]
        s = np.linalg.svd(B, compute_uv=False)
        if len(s) > 1:
            worst = max(worst, s[1] / s[0])
    return worst


@pytest.mark.parametrize("assign", mo.ASSIGNMENTS)
def test_materialised_matrix_has_the_assignments_block_structure(assign):
    f, h, w = 2, 3, 4
    M = materialise(assign, f, h, w, T=2)
    assert np.allclose(M.sum(1), 1.0, atol=1e-12)                 # row-stochastic
    assert block_rank_defect(M, token_of(assign, f, h, w)) < 1e-10
    # ... and it is NOT the structure of a different assignment (so the order matters)
    other = "w_fh" if assign != "w_fh" else "fh_w"
    assert block_rank_defect(M, token_of(other, f, h, w)) > 1e-3


def test_order_table_matches_the_hand_written_maps():
    f, h, w = 3, 2, 5
    for assign in mo.ASSIGNMENTS:
        order, rows, cols, rpf = mo.block_assignment_order(assign, f, h, w)
        tok = token_of(assign, f, h, w)
        assert (rows, cols) == tok.shape
        assert np.array_equal(order.numpy().reshape(rows, cols), tok)
        assert rpf == (rows // f if assign[0] == "f" else 0)
    # the stored order is the identity
    assert torch.equal(mo.block_assignment_order("fh_w", f, h, w)[0], torch.arange(f * h * w))


@pytest.mark.parametrize("assign", mo.ASSIGNMENTS)
@pytest.mark.parametrize("T", [1, 2])
def test_position_only_logits_give_dense_for_every_assignment(assign, T):
    # Sec. 4.1: any assignment of whole axes to the two block sides represents fully separable
    # positional logits exactly
    f, h, w = 2, 4, 6
    wl = syn.variant("C1", heads=1, f_q=f, f_kv=f, h=h, w=w, b1=f * h, b2=w, dtype="f32")
    Q, K, V = (torch.from_numpy(x).double() for x in syn.make_separable_head(wl, 0, 0))
    X, Y = SIZES[assign](f, h, w)
    O = mo.monarch_attn(Q, K, V, f_q=f, f_kv=f, h=h, w=w, b1=X, b2=Y, tile=0, iters=T,
                        scale=wl.scale, assign=assign)
    D = mo.dense_attn(Q, K, V, f_q=f, f_kv=f, h=h, w=w, scale=wl.scale)
    assert torch.allclose(O, D, atol=1e-6)


def test_assignments_that_coincide_on_degenerate_grids():
    d, T = 8, 2
    # one frame: (fh,w) = (h,fw) and (w,fh) = (fw,h); (f,hw) and (hw,f) are dense attention
    f, h, w = 1, 4, 5
    N = f * h * w
    Q, K, V = rnd((N, d), 1), rnd((N, d), 2), rnd((N, d), 3)

    def run(assign):
        X, Y = SIZES[assign](f, h, w)
        return mo.monarch_attn(Q, K, V, f_q=f, f_kv=f, h=h, w=w, b1=X, b2=Y, tile=0, iters=T, assign=assign)

    assert torch.allclose(run("fh_w"), run("h_fw"), atol=1e-12)
    assert torch.allclose(run("w_fh"), run("fw_h"), atol=1e-12)
    dense = torch.softmax(Q @ K.T, dim=1) @ V
    assert torch.allclose(run("f_hw"), dense, atol=1e-10)
    assert torch.allclose(run("hw_f"), dense, atol=1e-10)
    assert (run("fh_w") - run("w_fh")).abs().max() > 1e-3
    # one row per frame: (fh,w) = (f,hw) and (w,fh) = (hw,f)
    f, h, w = 3, 1, 5
    N = f * h * w
    Q, K, V = rnd((N, d), 4), rnd((N, d), 5), rnd((N, d), 6)
    assert torch.allclose(run("fh_w"), run("f_hw"), atol=1e-12)
    assert torch.allclose(run("w_fh"), run("hw_f"), atol=1e-12)


def test_swapping_height_and_width_of_the_stored_grid_swaps_the_assignment():
    # storing the video with height and width exchanged turns assignment (fw,h) into (fh,w)
    f, h, w, d, T = 2, 3, 4, 8, 2
    N = f * h * w
    Q, K, V = rnd((N, d), 7), rnd((N, d), 8), rnd((N, d), 9)
    swap = torch.arange(N).reshape(f, h, w).permute(0, 2, 1).reshape(N)   # token order of the (f,w,h) grid
    A = mo.monarch_attn(Q, K, V, f_q=f, f_kv=f, h=h, w=w, b1=f * w, b2=h, tile=0, iters=T, assign="fw_h")
    Bs = mo.monarch_attn(Q[swap], K[swap], V[swap], f_q=f, f_kv=f, h=w, w=h, b1=f * w, b2=h, tile=0,
                         iters=T, assign="fh_w")
    B = torch.empty_like(Bs)
    B[swap] = Bs
    assert torch.allclose(A, B, atol=1e-12)


# ---- tiles of a fraction of a frame (n_f = 1, n_h < h) and other contiguous row splits ------------

def loops_tiled_rect(Q, K, V, T, b1, b2, c1q, c1k, c2, vis, scale):
    """Alg. 2's update equations with explicit loops over tiles and indices (numpy scalars),
    rectangular and masked; tiles are contiguous row / column ranges of the (rows, w) grids."""
    Qn, Kn, Vn = Q.numpy(), K.numpy(), V.numpy()
    d = Qn.shape[1]
    W = c2 * b2

    def tok(a, b, r, c):
        return (a * b1 + r) * W + b * b2 + c

    O = np.zeros_like(Qn)
    for aq, bq in itertools.product(range(c1q), range(c2)):
        m = aq * c2 + bq
        keys = [(ak, bk) for ak in range(c1k) for bk in range(c2) if vis[m, ak * c2 + bk]]
        L = {nk: np.eye(b1)[None].repeat(b2, 0) for nk in keys}            # [j][k][l]
        R = {}
        for _ in range(T):
            for (ak, bk) in keys:
                Rn = np.zeros((b1, b2, b2))
                for k, j in itertools.product(range(b1), range(b2)):
                    a = sum(L[(ak, bk)][j, k, l] * Qn[tok(aq, bq, l, j)] for l in range(b1))
                    c = sum(L[(ak, bk)][j, k, l] for l in range(b1))
                    z = np.array([scale * np.dot(a, Kn[tok(ak, bk, k, i)]) / c for i in range(b2)])
                    e = np.exp(z - z.max())
                    Rn[k, j] = e / e.sum()
                R[(ak, bk)] = Rn
            Z = {}
            for (ak, bk) in keys:
                Zn = np.zeros((b2, b1, b1))
                for j, k in itertools.product(range(b2), range(b1)):
                    r = R[(ak, bk)][k, j]
                    aL = sum(r[i] * Kn[tok(ak, bk, k, i)] for i in range(b2))
                    cL = sum(r[i] * np.log(r[i]) for i in range(b2) if r[i] > 0)
                    for l in range(b1):
                        Zn[j, k, l] = scale * np.dot(aL, Qn[tok(aq, bq, l, j)]) - cL
                Z[(ak, bk)] = Zn
            for j, l in itertools.product(range(b2), range(b1)):
                z = np.array([Z[nk][j, k, l] for nk in keys for k in range(b1)])
                e = np.exp(z - z.max())
                e /= e.sum()
                for t, nk in enumerate(keys):
                    L[nk][j, :, l] = e[t * b1:(t + 1) * b1]
        for j, l in itertools.product(range(b2), range(b1)):
            acc = np.zeros(d)
            for (ak, bk) in keys:
                for k in range(b1):
                    Y = sum(R[(ak, bk)][k, j, i] * Vn[tok(ak, bk, k, i)] for i in range(b2))
                    acc += L[(ak, bk)][j, k, l] * Y
            O[tok(aq, bq, l, j)] = acc
    return torch.from_numpy(O)


@pytest.mark.parametrize("T", [1, 2])
def test_half_frame_tiles_against_explicit_loops(T):
    # h = 4 rows per frame, tiles of 2 rows (half a frame); 3 cached frames, chunks of 1 frame.
    # One query frame at absolute frame 2 sees all 6 key tile rows, at frame 1 only the first 4.
    f_q, f_kv, h, w, b1, b2, d = 1, 3, 4, 4, 2, 2, 6
    Q, K, V = rnd((f_q * h * w, d), 11), rnd((f_kv * h * w, d), 12), rnd((f_kv * h * w, d), 13)
    for qoff, nvis_rows in ((2, 6), (1, 4)):
        g = mo.geometry_from_grid(f_q, f_kv, h, w, b1, b2, 1)
        vis = mo.chunk_causal_visibility(g, h, 1, qoff)
        assert vis.shape == (4, 12)
        # written out: key tile row a' (2 grid rows) lies in frame a' // 2
        for m, n in itertools.product(range(4), range(12)):
            assert bool(vis[m, n]) == ((n // 2) // 2 <= qoff)
        assert int(vis[0].sum()) == nvis_rows * 2
        O = mo.monarch_attn(Q, K, V, f_q=f_q, f_kv=f_kv, h=h, w=w, b1=b1, b2=b2, tile=1, iters=T,
                            causal_chunk=1, q_frame_offset=qoff, scale=0.7)
        ref = loops_tiled_rect(Q, K, V, T, b1, b2, f_q * h // b1, f_kv * h // b1, w // b2, vis.numpy(), 0.7)
        assert torch.allclose(O, ref, atol=1e-10)


def test_tiles_straddling_a_chunk_are_refused():
    g = mo.geometry_from_grid(2, 2, 4, 4, 8, 2, 1)      # one tile row = 2 frames
    with pytest.raises(AssertionError):
        mo.chunk_causal_visibility(g, 4, 1, 0)
    g = mo.geometry_from_grid(2, 4, 4, 4, 8, 2, 1)
    vis = mo.chunk_causal_visibility(g, 4, 2, 2)        # 2-frame chunks: fine
    assert vis.tolist() == [[True] * 4, [True] * 4]


@pytest.mark.parametrize("assign,b1,b2", [("fw_h", 5, 2), ("fw_h", 10, 4), ("w_fh", 5, 4), ("h_fw", 2, 5)])
def test_tiled_assignments_with_position_only_logits_give_dense(assign, b1, b2):
    # tiles of any assignment are aligned sub-blocks, so separable logits stay exact (Sec. 4.2)
    f, h, w = 2, 4, 5
    wl = syn.variant("C1", heads=1, f_q=f, f_kv=f, h=h, w=w, b1=f * h, b2=w, dtype="f32")
    Q, K, V = (torch.from_numpy(x).double() for x in syn.make_separable_head(wl, 0, 0))
    O = mo.monarch_attn(Q, K, V, f_q=f, f_kv=f, h=h, w=w, b1=b1, b2=b2, tile=1, iters=2,
                        scale=wl.scale, assign=assign)
    D = mo.dense_attn(Q, K, V, f_q=f, f_kv=f, h=h, w=w, scale=wl.scale)
    assert torch.allclose(O, D, atol=1e-6)


def test_masked_kv_cache_with_frames_and_width_on_the_row_side():
    # (fw, h): rows = (frame, width); 1 query frame after 2 cached ones, 1-frame chunks, query at
    # absolute frame 1: frame 2 of the cache is hidden.  Position-only logits -> masked dense.
    f_q, f_kv, h, w = 1, 3, 4, 6
    wl = syn.variant("C3", heads=1, f_q=f_q, f_kv=f_kv, h=h, w=w, b1=w, b2=h, causal_chunk=1,
                     q_frame_offset=1, dtype="f32")
    Q, K, V = (torch.from_numpy(x).double() for x in syn.make_separable_head(wl, 0, 0))
    for b1, b2 in ((6, 4), (3, 2)):
        O = mo.monarch_attn(Q, K, V, f_q=f_q, f_kv=f_kv, h=h, w=w, b1=b1, b2=b2, tile=1, iters=2,
                            causal_chunk=1, q_frame_offset=1, scale=wl.scale, assign="fw_h")
        D = mo.dense_attn(Q, K, V, f_q=f_q, f_kv=f_kv, h=h, w=w, causal_chunk=1, q_frame_offset=1,
                          scale=wl.scale)
        assert torch.allclose(O, D, atol=1e-6)


# ---- neighbourhood tiles of several frames by a band of rows (Sec. 4.2's example) -----------------

def neighbourhood_loops(Q, K, V, T, f_q, f_kv, h, w, n_f, n_h, n_w, cc, qoff, scale):
    """Alg. 2's update equations with explicit loops; every tile is addressed through the grid
    coordinates of its tokens: tile (fa, ha, b), row (u, v), column c is grid cell
    (fa*n_f + u, ha*n_h + v, b*n_w + c)."""
    Qn, Kn, Vn = Q.numpy(), K.numpy(), V.numpy()
    d = Qn.shape[1]
    b1, b2 = n_f * n_h, n_w

    def tok(tile, r, c):
        fa, ha, b = tile
        u, v = divmod(r, n_h)
        return ((fa * n_f + u) * h + ha * n_h + v) * w + b * n_w + c

    def tiles(f):
        return [(fa, ha, b) for fa in range(f // n_f) for ha in range(h // n_h) for b in range(w // n_w)]

    O = np.zeros_like(Qn)
    for qt in tiles(f_q):
        keys = [kt for kt in tiles(f_kv)
                if cc == 0 or (kt[0] * n_f) // cc <= (qoff + qt[0] * n_f) // cc]
        L = {kt: np.eye(b1)[None].repeat(b2, 0) for kt in keys}            # [j][k][l]
        R = {}
        for _ in range(T):
            for kt in keys:
                Rn = np.zeros((b1, b2, b2))
                for k, j in itertools.product(range(b1), range(b2)):
                    a = sum(L[kt][j, k, l] * Qn[tok(qt, l, j)] for l in range(b1))
                    c = sum(L[kt][j, k, l] for l in range(b1))
                    z = np.array([scale * np.dot(a, Kn[tok(kt, k, i)]) / c for i in range(b2)])
                    e = np.exp(z - z.max())
                    Rn[k, j] = e / e.sum()
                R[kt] = Rn
            Z = {}
            for kt in keys:
                Zn = np.zeros((b2, b1, b1))
                for j, k in itertools.product(range(b2), range(b1)):
                    r = R[kt][k, j]
                    aL = sum(r[i] * Kn[tok(kt, k, i)] for i in range(b2))
                    cL = sum(r[i] * np.log(r[i]) for i in range(b2) if r[i] > 0)
                    for l in range(b1):
                        Zn[j, k, l] = scale * np.dot(aL, Qn[tok(qt, l, j)]) - cL
                Z[kt] = Zn
            for j, l in itertools.product(range(b2), range(b1)):
                z = np.array([Z[kt][j, k, l] for kt in keys for k in range(b1)])
                e = np.exp(z - z.max())
                e /= e.sum()
                for t, kt in enumerate(keys):
                    L[kt][j, :, l] = e[t * b1:(t + 1) * b1]
        for j, l in itertools.product(range(b2), range(b1)):
            acc = np.zeros(d)
            for kt in keys:
                for k in range(b1):
                    Y = sum(R[kt][k, j, i] * Vn[tok(kt, k, i)] for i in range(b2))
                    acc += L[kt][j, k, l] * Y
            O[tok(qt, l, j)] = acc
    return torch.from_numpy(O)


@pytest.mark.parametrize("cc,qoff", [(0, 0), (2, 2)])
def test_neighbourhood_tiles_against_explicit_loops(cc, qoff):
    # neighbourhoods of 2 frames x 2 rows x 2 columns on grids of 2 (queries) and 4 (keys) frames of
    # 4 x 4; with 2-frame chunks and the queries at frames 2..3 everything is visible, so also run
    # the queries at frames 0..1, which hides the second frame group
    f_q, f_kv, h, w, d = 2, 4, 4, 4, 5
    Q, K, V = rnd((f_q * h * w, d), 21), rnd((f_kv * h * w, d), 22), rnd((f_kv * h * w, d), 23)
    for off in ({qoff, 0} if cc else {0}):
        O = mo.monarch_attn(Q, K, V, f_q=f_q, f_kv=f_kv, h=h, w=w, b1=4, b2=2, tile=1, iters=2,
                            causal_chunk=cc, q_frame_offset=off, scale=0.7, tile_h=2)
        ref = neighbourhood_loops(Q, K, V, 2, f_q, f_kv, h, w, 2, 2, 2, cc, off, 0.7)
        assert torch.allclose(O, ref, atol=1e-10)
    # and the neighbourhood tiling differs from the contiguous split with the same block sizes
    Oc = mo.monarch_attn(Q, K, V, f_q=f_q, f_kv=f_kv, h=h, w=w, b1=4, b2=2, tile=1, iters=2, scale=0.7)
    On = mo.monarch_attn(Q, K, V, f_q=f_q, f_kv=f_kv, h=h, w=w, b1=4, b2=2, tile=1, iters=2, scale=0.7, tile_h=2)
    assert (Oc - On).abs().max() > 1e-3


def test_neighbourhood_tiles_reduce_to_the_contiguous_split():
    f, h, w, d = 2, 4, 6, 6
    Q, K, V = rnd((f * h * w, d), 31), rnd((f * h * w, d), 32), rnd((f * h * w, d), 33)
    base = dict(f_q=f, f_kv=f, h=h, w=w, b2=3, tile=1, iters=2, scale=0.5)
    # whole-height bands: neighbourhoods are whole frames
    assert torch.allclose(mo.monarch_attn(Q, K, V, b1=8, tile_h=4, **base), mo.monarch_attn(Q, K, V, b1=8, **base),
                          atol=1e-12)
    # one frame per neighbourhood: bands of 2 rows are contiguous rows
    assert torch.allclose(mo.monarch_attn(Q, K, V, b1=2, tile_h=2, **base), mo.monarch_attn(Q, K, V, b1=2, **base),
                          atol=1e-12)
    order = mo.neighbourhood_order(2, 4, 3, 2, 2)
    # written out for a (2, 4, 3) grid: band 0 = rows 0,1 of frame 0 then rows 0,1 of frame 1, ...
    assert order.tolist() == [0, 1, 2, 3, 4, 5, 12, 13, 14, 15, 16, 17,
                              6, 7, 8, 9, 10, 11, 18, 19, 20, 21, 22, 23]


def test_neighbourhood_tiles_with_position_only_logits_give_dense():
    f_q, f_kv, h, w = 2, 4, 4, 6
    wl = syn.variant("C3", heads=1, f_q=f_q, f_kv=f_kv, h=h, w=w, b1=4, b2=3, causal_chunk=2,
                     q_frame_offset=2, dtype="f32")
    Q, K, V = (torch.from_numpy(x).double() for x in syn.make_separable_head(wl, 0, 0))
    O = mo.monarch_attn(Q, K, V, f_q=f_q, f_kv=f_kv, h=h, w=w, b1=4, b2=3, tile=1, iters=2, causal_chunk=2,
                        q_frame_offset=2, scale=wl.scale, tile_h=2)
    D = mo.dense_attn(Q, K, V, f_q=f_q, f_kv=f_kv, h=h, w=w, causal_chunk=2, q_frame_offset=2, scale=wl.scale)
    assert torch.allclose(O, D, atol=1e-6)
